"""GPU parity of the update with 8-bit moments (SR_FLAG_FP8_MOMENTS: m as E4M3 codes, v as E5M2 codes,
a power-of-two scale per tensor) against the CPU oracle, through the C ABI: parameters and both code
arrays bit for bit.  NaN codes are compared as NaN codes (sign and payload of a NaN that arithmetic
produced are open), the parameter's NaNs as NaNs."""
import os

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2502_20566_amd import binding as B
from paper_2502_20566_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"
HYP = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
FP8 = B.SR_FLAG_FP8_MOMENTS


def bf16_bits(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def is_nan16(a):
    return ((a & 0x7F80) == 0x7F80) & ((a & 0x007F) != 0)


def nan8(codes, fmt):
    mag = codes & 0x7F
    return mag == 0x7F if fmt == 0 else mag > 0x7C


class State:
    """One list of tensors on the device and the same state on the host."""

    def __init__(self, sizes, exps, seed, offsets=None, ids=None, codes="any", views=0):
        rng = np.random.default_rng(seed)
        self.exps, self.ids = exps, ids or list(range(len(sizes)))
        self.offs = offsets or [0] * len(sizes)
        self.host, self.dev = [], []
        for n, (me, ve) in zip(sizes, exps):
            p = bf16_bits(rng.standard_normal(n) * 0.02)
            if codes == "any":                               # every code, NaN and infinity included
                m8 = rng.integers(0, 256, n).astype(np.uint8)
                v8 = rng.integers(0, 128, n).astype(np.uint8)
            else:                                            # moments of a running optimizer
                m8 = np.zeros(n, np.uint8)
                v8 = np.zeros(n, np.uint8)
            self.host.append(dict(p=p, m=m8, v=v8, m_exp=me, v_exp=ve))
            pad = views
            mk = lambda a, dt: torch.from_numpy(np.concatenate([np.zeros(pad, a.dtype), a, np.zeros(8, a.dtype)])).to(DEV)
            pd = W.u16_numpy_to_bf16(np.concatenate([np.zeros(pad, np.uint16), p, np.zeros(8, np.uint16)]), DEV)
            self.dev.append(dict(p=pd[pad:pad + n], m=mk(m8, np.uint8)[pad:pad + n], v=mk(v8, np.uint8)[pad:pad + n],
                                 g=torch.empty(n + pad + 8, dtype=torch.bfloat16, device=DEV)[pad:pad + n],
                                 whole=(pd,)))
        self.tl = B.TensorList([d["p"] for d in self.dev], [d["g"] for d in self.dev], [d["m"] for d in self.dev],
                               [d["v"] for d in self.dev], False, self.ids, self.offs, fp8_exponents=exps)

    def step(self, t, seed, g_scale, flags=0, norm=None, max_norm=0.0, rng=None, hyper=None):
        HYP = hyper or globals()["HYP"]
        rng = rng or np.random.default_rng(1000 + t)
        for h, d, (me, _) in zip(self.host, self.dev, self.exps):
            g = bf16_bits(rng.standard_normal(h["p"].size) * g_scale * 2.0 ** -me)
            h["g"] = g
            d["g"].copy_(W.u16_numpy_to_bf16(g, DEV))
        if norm is None:
            B.sr_adamw_step(self.tl, HYP, t, seed, flags | FP8)
        else:
            nt = torch.tensor([norm], dtype=torch.float32, device=DEV)
            B.sr_adamw_step(self.tl, HYP, t, seed, flags | FP8, nt, max_norm)
        torch.cuda.synchronize()
        hs = [dict(h, tensor_id=i, elem_offset=o) for h, i, o in zip(self.host, self.ids, self.offs)]
        ref.sr_adamw_step(hs, HYP, t, seed, flags | ref.FLAG_FP8_MOMENTS, norm, max_norm)

    def check(self, what):
        for k, (h, d) in enumerate(zip(self.host, self.dev)):
            gp = W.bf16_to_u16_numpy(d["p"])
            gn, wn = is_nan16(gp), is_nan16(h["p"])
            assert np.array_equal(gn, wn), f"{what}: tensor {k}: parameter NaN positions differ"
            bad = np.flatnonzero((gp != h["p"]) & ~gn)
            assert bad.size == 0, f"{what}: tensor {k}: {bad.size} parameters differ, first {bad[:4]}"
            for name, fmt in (("m", 0), ("v", 1)):
                got, want = d[name].cpu().numpy(), h[name]
                gn, wn = nan8(got, fmt), nan8(want, fmt)
                assert np.array_equal(gn, wn), f"{what}: tensor {k}: {name} NaN codes differ"
                bad = np.flatnonzero((got != want) & ~gn)
                assert bad.size == 0, (f"{what}: tensor {k}: {bad.size} codes of {name} differ, first {bad[:4]} "
                                       f"got {got[bad[:4]]} want {want[bad[:4]]}")


@pytest.mark.parametrize("flags", [0, B.SR_FLAG_RNE_PARAMS, B.SR_FLAG_EPS_IN_ROOT, B.SR_FLAG_DIV_BIAS])
def test_fp8_moments_every_code_as_input(flags):
    """Random codes of both formats as the incoming state (all 256 E4M3 codes, all non-negative E5M2
    codes, NaN and infinity included), sizes with several chunks and ragged tails, two tensors."""
    st = State([512 * 5 + 3, 1021], [(12, 30), (-2, 9)], seed=3 + flags)
    st.step(2, 0xC0FFEE, g_scale=4.0, flags=flags)
    st.check(f"flags {flags}")


def test_fp8_moments_many_steps_with_clip_and_offsets():
    """A running optimizer from zero moments: ten steps, clipping on, element offsets that are not
    multiples of 8 (edge blocks on both sides), misaligned views, tensor ids out of order."""
    st = State([4096 + 5, 77, 8, 1], [(14, 33), (10, 26), (0, 0), (14, 33)], seed=5, offsets=[3, 8, 16, 7],
               ids=[7, 2, 9, 4], codes="zero", views=3)
    for t in range(1, 11):
        st.step(t, 17, g_scale=3.0, norm=2.5, max_norm=1.0)
        st.check(f"step {t}")
    used_m = np.unique(st.host[0]["m"]).size
    used_v = np.unique(st.host[0]["v"]).size
    assert used_m > 60 and used_v > 20                        # the state really lives on the 8-bit grids


def test_fp8_moments_write_back_through_the_integer_path_only():
    """The test switch that sends every wave's 8-bit write-back down the integer path (no conversion
    instruction): the same scenarios must still equal the oracle, so the chip's scaled conversions
    and the integer path are shown to compute one function on the same inputs."""
    B.lib().sr_debug_set(B.SR_DEBUG_FP8_INTEGER, 1)
    try:
        st = State([512 * 5 + 3, 1021], [(12, 30), (-2, 9)], seed=31)
        st.step(2, 0xC0FFEE, g_scale=4.0)
        st.check("every code, integer path")
        st = State([4096 + 5, 77, 8, 1], [(14, 33), (10, 26), (0, 0), (14, 33)], seed=5, offsets=[3, 8, 16, 7],
                   ids=[7, 2, 9, 4], codes="zero", views=3)
        for t in range(1, 11):
            st.step(t, 17, g_scale=3.0, norm=2.5, max_norm=1.0, flags=B.SR_FLAG_RNE_PARAMS if t % 2 else 0)
            st.check(f"integer path step {t}")
        assert np.unique(st.host[0]["m"]).size > 60
    finally:
        B.lib().sr_debug_set(B.SR_DEBUG_FP8_INTEGER, 0)


def test_fp8_moments_top_of_range_and_nan_gradients():
    """Scales chosen too large on purpose: m saturates at 448 and v at 57344; NaN and infinite
    gradients; every wave holds some of each, so the integer path and the conversion instruction
    both run (waves of the second tensor hold nothing large)."""
    st = State([512 * 3, 512 * 2], [(22, 44), (12, 30)], seed=8, codes="zero")
    rng = np.random.default_rng(4)
    for t in (1, 2, 3):
        st.step(t, 5, g_scale=2.0 ** 12, rng=rng)
        st.check(f"step {t}")
    assert (st.host[0]["m"] & 0x7F == 0x7E).any() and (st.host[0]["v"] == 0x7B).any()
    assert not (st.host[0]["v"] & 0x7F == 0x7C).any()             # no infinity is ever stored
    g = st.host[0]["g"].copy()
    g[5], g[700], g[1300] = 0x7FC0, 0x7F80, 0xFF80            # NaN, +inf, -inf
    st.host[0]["g"] = g
    st.dev[0]["g"].copy_(W.u16_numpy_to_bf16(g, DEV))
    B.sr_adamw_step(st.tl, HYP, 4, 5, FP8)
    torch.cuda.synchronize()
    ref.sr_adamw_step([dict(h, tensor_id=i) for i, h in enumerate(st.host)], HYP, 4, 5, ref.FLAG_FP8_MOMENTS)
    st.check("special gradients")
    assert st.host[0]["m"][5] & 0x7F == 0x7F


@pytest.mark.parametrize("exps,g_scale", [((100, 100), 2.0 ** -12), ((100, 100), 2.0 ** -24), ((-100, -100), 1.0),
                                          ((97, -3), 2.0 ** -20), ((-100, 100), 2.0 ** 8)])
def test_fp8_moments_extreme_scales(exps, g_scale):
    """The largest scale exponents, with gradients so small (or large) that new moments are binary32
    subnormals, that their scaled values fall into the 8-bit formats' subnormal ranges or below them,
    or that squares overflow: the scaled conversion of the kernel and the multiply-then-round of the
    definition must still agree in every element."""
    st = State([2048 + 3, 517], [exps, exps], seed=31, views=1)
    rng = np.random.default_rng(6)
    for t in (1, 2, 3):
        st.step(t, 77, g_scale=g_scale, rng=rng)
        st.check(f"exponents {exps}, step {t}")


def test_fp8_moments_randomized_cases():
    """Thirty seeded random cases: list length, sizes, misalignment, element offsets, tensor ids, scale
    exponents, parameter rounding and variant flags, clipping, hyper-parameters including the corners
    (beta = 0, eps = 0, lr = 0, large lr, late steps), every code as incoming state."""
    rng = np.random.default_rng(4242)
    for case in range(int(os.environ.get("SR_TEST_CASES", "30"))):      # more cases on request
        flags = 0
        if rng.random() < 0.3:
            flags |= B.SR_FLAG_RNE_PARAMS
        if rng.random() < 0.3:
            flags |= B.SR_FLAG_EPS_IN_ROOT
        if rng.random() < 0.3:
            flags |= B.SR_FLAG_DIV_BIAS
        n_t = int(rng.integers(1, 70))
        sizes = [int(rng.choice([1, 5, 8, 64, 257, 512, 1000, 4099, 9000])) for _ in range(n_t)]
        exps = [(int(rng.integers(-20, 41)), int(rng.integers(-20, 61))) for _ in range(n_t)]
        offs = [int(rng.choice([0, 0, 8, 3, 1 << 32, (1 << 40) + 5])) for _ in range(n_t)]
        ids = [int(rng.integers(0, 1 << 32)) for _ in range(n_t)]
        st = State(sizes, exps, seed=900 + case, offsets=offs, ids=ids, views=int(rng.integers(0, 4)))
        hyper = dict(lr=float(rng.choice([0.0, 1e-5, 6e-4, 3e-3, 0.5])),
                     beta1=float(rng.choice([0.0, 0.5, 0.9, 0.99])),
                     beta2=float(rng.choice([0.0, 0.95, 0.999, 0.99999])),
                     eps=float(rng.choice([0.0, 1e-12, 1e-8, 1e-3])),
                     weight_decay=float(rng.choice([0.0, 0.1, 1.0])))
        t = int(rng.choice([1, 2, 17, 1000, 123456, 2 ** 32 - 1]))
        clip = None if rng.random() < 0.5 else float(rng.choice([1e-3, 0.05, 1.0, 100.0]))
        norm = None if clip is None else float(rng.choice([1e-4, 0.3, 7.0]))
        st.step(t, int(rng.integers(0, 1 << 62)), g_scale=float(rng.choice([0.25, 4.0, 64.0])), flags=flags,
                norm=norm, max_norm=clip or 0.0, rng=rng, hyper=hyper)
        st.check(f"case {case} flags {flags} hyper {hyper} t {t} clip {clip}")


def test_fp8_moments_arguments():
    n = 64
    p = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    m8 = torch.zeros(n, dtype=torch.uint8, device=DEV)
    f8 = torch.zeros(n, dtype=torch.float8_e4m3fn, device=DEV)
    f5 = torch.zeros(n, dtype=torch.float8_e5m2, device=DEV)
    tl = B.TensorList([p], [p.clone()], [f8], [f5], fp8_exponents=[(12, 30)])       # torch float8 tensors as storage
    B.sr_adamw_step(tl, HYP, 1, 0, FP8)
    torch.cuda.synchronize()
    for bad in (FP8 | B.SR_FLAG_RNE_MOMENTS, FP8 | B.SR_FLAG_EPS_IN_ROOT | B.SR_FLAG_RNE_MOMENTS):
        with pytest.raises(B.SrError):
            B.sr_adamw_step(tl, HYP, 1, 0, bad)
    for bad in (FP8 | B.SR_FLAG_FP32_MOMENTS, 0):               # the binding checks the list against the flag
        with pytest.raises(ValueError):
            B.sr_adamw_step(tl, HYP, 1, 0, bad)
    with pytest.raises(ValueError):
        B.TensorList([p], [p.clone()], [m8], [m8.clone()], fp8_exponents=[(101, 0)])
    tl.array[0].reserved = 1
    with pytest.raises(B.SrError):
        B.sr_adamw_step(tl, HYP, 1, 0, FP8)


def test_optimizer_object_with_8_bit_moments_and_resume():
    """SRAdamW(strategy="fp8_moments") equals direct calls through the binding (which the tests above
    pin to the oracle), through a resume from state_dict; a checkpoint written with other scale
    exponents is refused."""
    from paper_2502_20566_amd.optimizer import SRAdamW
    torch.manual_seed(0)
    model = torch.nn.Sequential(torch.nn.Linear(48, 80), torch.nn.Tanh(), torch.nn.Linear(80, 6)).to(DEV).to(torch.bfloat16)
    params = list(model.parameters())
    exps = (13, 27)
    ref_p = [p.detach().clone().view(-1) for p in params]
    ref_m = [torch.zeros(p.numel(), dtype=torch.uint8, device=DEV) for p in ref_p]
    ref_v = [torch.zeros(p.numel(), dtype=torch.uint8, device=DEV) for p in ref_p]
    opt = SRAdamW(params, lr=2e-3, seed=9, strategy="fp8_moments", fp8_exponents=exps)
    hyper = dict(lr=2e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    x = torch.randn(32, 48, device=DEV, dtype=torch.bfloat16)
    for t in range(1, 6):
        model(x).float().pow(2).mean().backward()
        grads = [p.grad.detach().clone().view(-1) for p in params]
        opt.step()
        opt.zero_grad()
        tl = B.TensorList(ref_p, grads, ref_m, ref_v, fp8_exponents=[exps] * len(ref_p))
        B.sr_adamw_step(tl, hyper, t, 9, FP8)
        torch.cuda.synchronize()
        for a, b, m, v in zip(params, ref_p, ref_m, ref_v):
            assert torch.equal(a.detach().view(-1).view(torch.int16), b.view(torch.int16))
            assert torch.equal(opt.state[a]["exp_avg"], m) and torch.equal(opt.state[a]["exp_avg_sq"], v)
        if t == 2:
            sd = opt.state_dict()
            sd["state"] = [{k: v_.clone() for k, v_ in st.items()} for st in sd["state"]]
            with pytest.raises(ValueError):
                SRAdamW(params, strategy="fp8_moments", fp8_exponents=(12, 27)).load_state_dict(sd)
            opt = SRAdamW(params, lr=2e-3, seed=0, strategy="fp8_moments", fp8_exponents=exps)
            opt.load_state_dict(sd)
    assert any(int(m.count_nonzero()) > 0 for m in ref_m)
    with pytest.raises(ValueError):
        SRAdamW(params, strategy="fp8_moments")
    with pytest.raises(ValueError):
        SRAdamW(params, strategy="sr", fp8_exponents=exps)


def test_stream_probe_of_the_8_bit_moment_pattern_leaves_the_data_unchanged():
    n = 512 * 7 + 13                                             # whole blocks only: the tail is not touched either
    p = (torch.randn(n, device=DEV) * 0.01).to(torch.bfloat16)
    g = (torch.randn(n, device=DEV) * 0.01).to(torch.bfloat16)
    m8 = torch.randint(0, 256, (n,), dtype=torch.uint8, device=DEV)
    v8 = torch.randint(0, 128, (n,), dtype=torch.uint8, device=DEV)
    before = [t.clone() for t in (p, g, m8, v8)]
    B.sr_stream_probe_fp8m(p, g, m8, v8)
    B.lib().sr_debug_set(B.SR_DEBUG_LAUNCH_LIMIT, 3)                          # and cut into several launches
    try:
        B.sr_stream_probe_fp8m(p, g, m8, v8)
    finally:
        B.lib().sr_debug_set(B.SR_DEBUG_LAUNCH_LIMIT, 0)
    torch.cuda.synchronize()
    for t, b in zip((p, g, m8, v8), before):
        assert torch.equal(t.view(torch.uint8), b.view(torch.uint8))
    e = torch.empty(0, dtype=torch.bfloat16, device=DEV)
    B.sr_stream_probe_fp8m(e, e, torch.empty(0, dtype=torch.uint8, device=DEV), torch.empty(0, dtype=torch.uint8, device=DEV))
