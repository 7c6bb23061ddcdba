"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Bar: BF16 outputs and SR decisions bit-exact (the tolerance of at
most 1 BF16 ulp on at most 1e-6 of the elements is written in `assert_bf16_parity`; expected
residue is zero), binary32 moments and master weights identical encodings, the norm equal or
within relative 1e-6 (its binary64 sum runs in a different order on the two sides).
NaNs produced by arithmetic are compared as NaNs (IEEE 754 leaves their sign and payload open);
NaNs that are merely cast keep specified bits and are compared exactly.
"""
import os

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2502_20566_amd import binding as B
from paper_2502_20566_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


# ------------------------------------------------------------------ helpers

def to_np(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return W.bf16_to_u16_numpy(t)
    return t.detach().cpu().numpy().copy()


def bf16_dev(bits: np.ndarray) -> torch.Tensor:
    return W.u16_numpy_to_bf16(np.ascontiguousarray(bits, dtype=np.uint16), DEV)


def is_nan16(a):
    return ((a & 0x7F80) == 0x7F80) & ((a & 0x007F) != 0)


def assert_bf16_parity(got: np.ndarray, want: np.ndarray, what: str, exact_nan: bool = False):
    assert got.shape == want.shape
    if not exact_nan:
        gn, wn = is_nan16(got), is_nan16(want)
        assert bool(np.all(gn == wn)), f"{what}: NaN positions differ"
        got, want = np.where(gn, 0, got), np.where(wn, 0, want)
    diff = got != want
    n_bad = int(diff.sum())
    if n_bad == 0:
        return
    # tolerance of the contract: <= 1 BF16 ulp on <= 1e-6 of the elements
    ulp = np.abs(got[diff].astype(np.int32) - want[diff].astype(np.int32))
    first = np.flatnonzero(diff)[:5]
    assert n_bad <= 1e-6 * got.size and int(ulp.max()) <= 1, \
        f"{what}: {n_bad} of {got.size} differ (max {int(ulp.max())} ulp), first at {first}"


def assert_f32_parity(got: np.ndarray, want: np.ndarray, what: str):
    # binary32 moments and master weights are stored unrounded by the same operations in the same
    # order on both sides: identical encodings (a NaN produced by arithmetic may differ in sign)
    both_nan = np.isnan(got) & np.isnan(want)
    ok = both_nan | (got.view(np.uint32) == want.view(np.uint32))
    assert bool(np.all(ok)), f"{what}: {int((~ok).sum())} of {got.size} binary32 values differ"


class Pair:
    """The same optimizer state on the device (library) and on the host (oracle)."""

    def __init__(self, params, ms, vs, fp32_moments, tensor_ids=None, elem_offsets=None, aux=None):
        self.fp32 = fp32_moments
        self.p, self.m, self.v, self.aux = params, ms, vs, aux
        self.g = [torch.empty_like(p) for p in params]
        self.ids = list(range(len(params))) if tensor_ids is None else list(tensor_ids)
        self.offs = [0] * len(params) if elem_offsets is None else list(elem_offsets)
        self.tl = B.TensorList(self.p, self.g, self.m, self.v, fp32_moments, self.ids, self.offs, aux)
        self.host = [dict(p=to_np(p), m=to_np(m), v=to_np(v), tensor_id=i, elem_offset=o)
                     for p, m, v, i, o in zip(params, ms, vs, self.ids, self.offs)]
        if aux is not None:
            for h, a in zip(self.host, aux):
                h["aux"] = to_np(a)
        self.norm = torch.zeros(1, dtype=torch.float32, device=DEV)
        self.ws = torch.empty(max(self.tl.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)

    def step(self, hyper, t, seed, clip=None, flags=0, check_norm=True):
        for h, g in zip(self.host, self.g):
            h["g"] = to_np(g)
        if self.fp32:
            flags |= B.SR_FLAG_FP32_MOMENTS
        norm_val = None
        if clip is not None:
            B.grad_global_norm(self.tl, self.norm, self.ws)
            norm_val = float(self.norm.item())
            if check_norm:
                want = ref.grad_global_norm([h["g"] for h in self.host])
                assert norm_val == want or abs(norm_val - want) <= 1e-6 * want, (norm_val, want)
            B.sr_adamw_step(self.tl, hyper, t, seed, flags, self.norm, clip)
        else:
            B.sr_adamw_step(self.tl, hyper, t, seed, flags)
        torch.cuda.synchronize()
        # the oracle takes the same FP32 norm bits the device used
        ref.sr_adamw_step(self.host, hyper, t, seed, flags, norm=norm_val,
                          max_norm=0.0 if clip is None else clip)

    def compare(self, what):
        for i, h in enumerate(self.host):
            assert_bf16_parity(to_np(self.p[i]), h["p"], f"{what} p[{i}]")
            if self.fp32:
                assert_f32_parity(to_np(self.m[i]), h["m"], f"{what} m[{i}]")
                assert_f32_parity(to_np(self.v[i]), h["v"], f"{what} v[{i}]")
            else:
                assert_bf16_parity(to_np(self.m[i]), h["m"], f"{what} m[{i}]")
                assert_bf16_parity(to_np(self.v[i]), h["v"], f"{what} v[{i}]")
            if self.aux is not None:
                got = to_np(self.aux[i])
                if got.dtype == np.uint16:
                    assert_bf16_parity(got, h["aux"], f"{what} aux[{i}]")
                else:
                    assert_f32_parity(got, h["aux"], f"{what} aux[{i}]")


def make_pair(cfg: W.Config, shapes=None):
    shapes = cfg.shapes if shapes is None else shapes
    params = W.make_params(shapes, DEV, W.data_seed(cfg.index, 0), cfg.param_std)
    ms, vs = W.make_moments(shapes, DEV, cfg.fp32_moments)
    return Pair(params, ms, vs, cfg.fp32_moments)


def run_config(cfg: W.Config, shapes, steps):
    pair = make_pair(cfg, shapes)
    for t in range(1, steps + 1):
        W.fill_grads(pair.g, W.data_seed(cfg.index, t), cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
        pair.step(cfg.hyper, t, cfg.seed, clip=cfg.clip)
        pair.compare(f"{cfg.name} step {t}")
    return pair


# ------------------------------------------------------------- sr_cast_f32_bf16

def gpu_cast(x: torch.Tensor, seed, step, tid):
    out = torch.empty(x.numel(), dtype=torch.bfloat16, device=DEV)
    B.sr_cast_f32_bf16(x, out, seed, step, tid)
    torch.cuda.synchronize()
    return to_np(out)


def test_cast_config1_workload_bit_exact():
    x = W.make_cast_input(1 << 20, DEV, W.data_seed(1, 0))
    got = gpu_cast(x, 0, 1, 0)
    want = ref.sr_cast_f32_bf16(x.cpu().numpy(), 0, 1, 0)
    assert_bf16_parity(got, want, "cast config 1", exact_nan=True)
    assert bool(np.all(got == want))
    # a different seed, step or tensor id draws differently
    for args in ((1, 1, 0), (0, 2, 0), (0, 1, 1)):
        other = gpu_cast(x, *args)
        assert bool(np.all(other == ref.sr_cast_f32_bf16(x.cpu().numpy(), *args)))
        assert 0.2 < float((other != got).mean()) < 0.5


@pytest.mark.parametrize("n", [1, 7, 8, 9, 63, 511, 512, 513, 4097, 2 * 256 * 8 * 3 + 5])
def test_cast_ragged_sizes_and_misaligned_views(n):
    base = W.make_cast_input(n + 16, DEV, 77)
    for off in (0, 1, 3):
        x = base[off:off + n]
        out_base = torch.zeros(n + 16, dtype=torch.bfloat16, device=DEV)
        for ooff in (0, 1):
            dst = out_base[ooff:ooff + n]
            out_base.zero_()
            B.sr_cast_f32_bf16(x, dst, 5, 3, 2)
            torch.cuda.synchronize()
            want = ref.sr_cast_f32_bf16(x.cpu().numpy(), 5, 3, 2)
            assert bool(np.all(to_np(dst) == want))
            # nothing outside the destination range was written
            whole = to_np(out_base)
            assert not whole[:ooff].any() and not whole[ooff + n:].any()


def test_cast_special_values_exact_bits():
    specials = [0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00000, 0xFFC00000, 0x7F800001,
                0xFF80FFFF, 0x7FFFFFFF, 0x7FA12345, 0x7F7FFFFF, 0xFF7FFFFF, 0x7F7F0001, 0x00000001,
                0x80000001, 0x007FFFFF, 0x00800000, 0x0000FFFF, 0x00010000, 0x3F800000, 0x3F80FFFF,
                0x3FFFFFFF, 0xBFFFFFFF, 0x7F7F8000]
    bits = np.array(specials * 1024, dtype=np.uint32)
    x = torch.from_numpy(bits.view(np.int32)).to(DEV).view(torch.float32)
    for seed in (0, 1, 2):
        got = gpu_cast(x, seed, 1, 0)
        want = ref.sr_cast_f32_bf16(bits.view(np.float32), seed, 1, 0)
        assert bool(np.all(got == want))
    # +-FLT_MAX overflows to infinity for nearly every draw
    fm = got.reshape(1024, len(specials))[:, specials.index(0x7F7FFFFF)]
    assert (fm == 0x7F80).mean() > 0.99


def test_cast_unbiased_on_device():
    # E[Q_SR(x)] = x with the device's own draws: 4096 elements of one value, many steps
    x = torch.full((1 << 16,), 1.0 + 2.0 ** -7 * 0.3, dtype=torch.float32, device=DEV)
    got = gpu_cast(x, 123, 9, 4)
    vals = ref.bf16_bits_to_f32(got).astype(np.float64)
    k = int(x[:1].view(torch.int32).item() & 0xFFFF)
    q = k / 65536.0
    assert abs(vals.mean() - float(x[0])) <= 5 * 2.0 ** -7 * np.sqrt(q * (1 - q) / vals.size)


def test_cast_empty():
    x = torch.empty(0, dtype=torch.float32, device=DEV)
    out = torch.empty(0, dtype=torch.bfloat16, device=DEV)
    B.sr_cast_f32_bf16(x, out, 0, 1, 0)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ sr_adamw_step

def test_adamw_config1_flat_bit_exact():
    cfg = W.config(1)
    pair = run_config(cfg, cfg.shapes, 1)
    # at step 1 from zero moments every parameter with a non-zero gradient moves by about lr
    moved = (to_np(pair.p[0]) != W.bf16_to_u16_numpy(
        W.make_params(cfg.shapes, DEV, W.data_seed(1, 0), cfg.param_std)[0])).mean()
    assert moved > 0.5


def test_adamw_gpt_list_ten_steps_bit_exact():
    # config 2 recipe on a small GPT shape list: 2 + 12*3 + 2 = 40 tensors, ragged sizes
    cfg = W.config(2)
    shapes = W.gpt_shapes(72, 3, 200, 1003, 33)
    pair = run_config(cfg, shapes, 10)
    assert len(pair.host) == 40


def test_adamw_more_tensors_than_one_launch_batch():
    """A launch takes 320 tensors (update, accumulation) or 400 (norm): a list of 868 tensors is
    three launches of each, with clipping so that the norm's batches are cut too; then the same
    list through the accumulation with the fused norm."""
    cfg = W.config(3)
    shapes = W.gpt_shapes(24, 72, 40, 101, 16)
    assert len(shapes) == 868
    pair = run_config(cfg, shapes, 2)
    micro = [torch.empty_like(g) for g in pair.g]
    W.fill_grads(micro, 61, cfg.grad_std)
    al = B.AccumList(pair.g, micro)
    ws = torch.empty(max(al.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    host = [to_np(g) for g in pair.g]
    B.sr_grad_accumulate(al, 0.5, 7, 3, 0, pair.norm, ws)
    torch.cuda.synchronize()
    for i, h in enumerate(host):
        ref.grad_accumulate(h, to_np(micro[i]), 0.5, 7, 3, tensor_id=i)
        assert bool(np.all(to_np(pair.g[i]) == h)), f"accumulate tensor {i}"
    want, got = ref.grad_global_norm(host), float(pair.norm.item())
    assert got == want or abs(got - want) <= 1e-6 * want


def test_adamw_clip_with_outliers_bit_exact():
    cfg = W.config(3)
    shapes = W.gpt_shapes(64, 2, 256, 5003, 64)
    pair = run_config(cfg, shapes, 10)
    assert float(pair.norm.item()) > 10.0                  # clipping is strongly active


@pytest.mark.parametrize("fp32", [False, True])
def test_adamw_skips_the_step_on_a_nonfinite_norm(fp32):
    """SR_FLAG_SKIP_NONFINITE_NORM: a NaN or infinite norm (here from a planted NaN / infinite
    gradient, through grad_global_norm) leaves p, m, v untouched on both sides; with a finite
    norm the flag changes nothing; without the flag the poisoned step is applied as the clip
    formula says (NaN everywhere, or a zero gradient scale) and still equals the oracle."""
    cfg = W.config(4 if fp32 else 3)
    shapes = W.gpt_shapes(48, 1, 192, 1001, 32)
    pair = make_pair(cfg, shapes)
    SKIP = B.SR_FLAG_SKIP_NONFINITE_NORM
    W.fill_grads(pair.g, W.data_seed(3, 1), cfg.grad_std)
    pair.step(cfg.hyper, 1, 9, clip=1.0, flags=SKIP)                  # finite norm: an ordinary step
    pair.compare("finite norm with the guard")
    assert not bool(np.all(to_np(pair.m[0]).view(np.uint8) == 0))
    for t, bad in ((2, float("nan")), (3, float("inf")), (4, float("-inf"))):
        W.fill_grads(pair.g, W.data_seed(3, t), cfg.grad_std)
        pair.g[2][5] = bad
        before = [(to_np(p), to_np(m), to_np(v)) for p, m, v in zip(pair.p, pair.m, pair.v)]
        pair.step(cfg.hyper, t, 9, clip=1.0, flags=SKIP, check_norm=False)
        assert not np.isfinite(pair.norm.item())
        for (p0, m0, v0), p, m, v in zip(before, pair.p, pair.m, pair.v):
            for a, b in ((p0, p), (m0, m), (v0, v)):
                assert bool(np.all(a.view(np.uint8) == to_np(b).view(np.uint8)))
        pair.compare(f"skipped step {t}")
    # without the guard: an infinite norm scales the gradient to zero, a NaN norm poisons the state
    W.fill_grads(pair.g, W.data_seed(3, 5), cfg.grad_std)
    pair.g[2][5] = float("inf")
    pair.step(cfg.hyper, 5, 9, clip=1.0, check_norm=False)
    pair.compare("unguarded infinite norm")
    pair.g[2][5] = float("nan")
    pair.step(cfg.hyper, 6, 9, clip=1.0, check_norm=False)
    pair.compare("unguarded NaN norm")
    assert bool(np.all(is_nan16(to_np(pair.p[0]))))


def test_adamw_fp32_moments_clip_bit_exact():
    cfg = W.config(4)
    shapes = W.gpt_shapes(80, 2, 320, 4099, 64)
    pair = run_config(cfg, shapes, 5)
    # FP32 moments agree to the bit, not just to 1e-6
    for i, h in enumerate(pair.host):
        assert bool(np.all(to_np(pair.m[i]) == h["m"])) and bool(np.all(to_np(pair.v[i]) == h["v"]))


def test_adamw_warm_state_flat_bit_exact():
    # config 5 recipe at 2^22 + 5 elements: warm moments, SR on all three outputs
    cfg = W.config(5)
    shapes = [("flat", ((1 << 22) + 5,), "weight")]
    run_config(cfg, shapes, 6)


def test_adamw_rne_moments_variant():
    cfg = W.config(2)
    shapes = W.gpt_shapes(40, 1, 96, 301, 16)
    pair = make_pair(cfg, shapes)
    for t in range(1, 4):
        W.fill_grads(pair.g, W.data_seed(2, t), cfg.grad_std)
        pair.step(cfg.hyper, t, 3, flags=B.SR_FLAG_RNE_MOMENTS)
        pair.compare(f"rne moments step {t}")


def _random_state(n, seed, fp32=False):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    p = (torch.randn(n, device=DEV, generator=g) * 0.02).to(torch.bfloat16)
    gr = (torch.randn(n, device=DEV, generator=g) * 1e-3).to(torch.bfloat16)
    m = torch.randn(n, device=DEV, generator=g) * 1e-3
    v = torch.rand(n, device=DEV, generator=g) * 1e-6
    if not fp32:
        m, v = m.to(torch.bfloat16), v.to(torch.bfloat16)
    return p, gr, m, v


@pytest.mark.parametrize("mode", ["sr", "fp32", "nearest", "kahan", "master"])
def test_adamw_ragged_misaligned_and_offset_tensors(mode):
    """Sizes around the 8-element block and the chunk size, views that start 2 bytes off a
    16-byte boundary, element offsets that are not multiples of 8: same bits as the oracle,
    for every variant of the step."""
    fp32 = mode in ("fp32", "master")
    flags = {"sr": 0, "fp32": 0, "nearest": B.SR_FLAG_RNE_PARAMS | B.SR_FLAG_RNE_MOMENTS,
             "kahan": B.SR_FLAG_KAHAN, "master": B.SR_FLAG_MASTER_FP32}[mode]
    sizes = [1, 7, 8, 9, 15, 17, 255, 256, 257, 511, 512, 513, 1000, 4096, 4097, 2 * 256 * 8 + 3, 40000]
    params, grads, ms, vs, offs, aux = [], [], [], [], [], []
    for i, n in enumerate(sizes):
        shift = i % 3                                     # 0: aligned, 1 or 2 elements off
        p, g, m, v = _random_state(n + 8, 100 + i, fp32)
        params.append(p[shift:shift + n]); grads.append(g[shift:shift + n])
        mshift = shift if i % 2 == 0 else (shift + 1) % 3   # moments sometimes aligned differently
        ms.append(m[mshift:mshift + n]); vs.append(v[shift:shift + n])
        offs.append([0, 8, 5, 1 << 33, (1 << 35) + 3][i % 5])
        ashift = shift if i % 4 != 1 else (shift + 2) % 3
        if mode == "kahan":
            a = (torch.randn(n + 8, device=DEV) * 1e-5).to(torch.bfloat16)
            aux.append(a[ashift:ashift + n])
        elif mode == "master":
            a = params[-1].float() + torch.randn(n, device=DEV) * 1e-5      # master near its BF16 copy
            buf = torch.zeros(n + 8, device=DEV)
            buf[ashift:ashift + n] = a
            aux.append(buf[ashift:ashift + n])
    pair = Pair(params, ms, vs, fp32, tensor_ids=[7 * i + 1 for i in range(len(sizes))], elem_offsets=offs,
                aux=aux if aux else None)
    for g_dst, g_src in zip(pair.g, grads):
        g_dst.copy_(g_src)
    hyper = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    for t in (1, 2):
        pair.step(hyper, t, seed=0xDEADBEEFCAFE, clip=0.01, flags=flags)
        pair.compare(f"ragged {mode} step {t}")


def _mode_run(flags, fp32, make_aux, steps=5, clip=None):
    cfg = W.config(2)
    shapes = W.gpt_shapes(72, 2, 200, 1003, 33)
    params = W.make_params(shapes, DEV, W.data_seed(2, 0), cfg.param_std)
    ms, vs = W.make_moments(shapes, DEV, fp32)
    aux = make_aux(params) if make_aux else None
    pair = Pair(params, ms, vs, fp32, aux=aux)
    for t in range(1, steps + 1):
        W.fill_grads(pair.g, W.data_seed(2, t), 1e-3)
        pair.step(cfg.hyper, t, 11, clip=clip, flags=flags)
        pair.compare(f"flags {flags} step {t}")
    return pair


@pytest.mark.parametrize("fp32", [False, True])
def test_adamw_counter_indices_at_the_top_of_their_range(fp32):
    """elem_offset + numel may reach 2^64 - 9 (the last counter block must not wrap): slices that end on
    the largest index the library accepts, aligned and mid-block, several chunks long, against the
    oracle; one element further is refused."""
    top = (1 << 64) - 1
    sizes = [5, 8, 1000, 3 * 512 + 77, 20000]
    params, grads, ms, vs, offs = [], [], [], [], []
    for i, n in enumerate(sizes):
        p, g, m, v = _random_state(n, 900 + i, fp32)
        params.append(p); grads.append(g); ms.append(m); vs.append(v)
        end = top - 8 - (0, 1, 7, 8, 13)[i]                  # elem_offset + numel
        offs.append(end - n)
    pair = Pair(params, ms, vs, fp32, tensor_ids=[11 * i + 2 for i in range(len(sizes))], elem_offsets=offs)
    for gd, gs in zip(pair.g, grads):
        gd.copy_(gs)
    hyper = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    for t in (1, 2):
        pair.step(hyper, t, 0xFEDCBA9876543210)
        pair.compare(f"top-of-range offsets (fp32 moments {fp32}) step {t}")
    bad = B.TensorList(params[:1], pair.g[:1], ms[:1], vs[:1], fp32, [2], [top - 8 - sizes[0] + 1])
    with pytest.raises(B.SrError):
        B.sr_adamw_step(bad, hyper, 3, 1, B.SR_FLAG_FP32_MOMENTS if fp32 else 0)


def test_adamw_all_nearest_bf16_strategy():
    # Section 5.1's "BF16" strategy: every write-back rounded to nearest, no random bits
    a = _mode_run(B.SR_FLAG_RNE_PARAMS | B.SR_FLAG_RNE_MOMENTS, False, None)
    assert a is not None


def test_adamw_nearest_parameter_with_stochastic_or_fp32_moments():
    _mode_run(B.SR_FLAG_RNE_PARAMS, False, None, steps=3)
    _mode_run(B.SR_FLAG_RNE_PARAMS, True, None, steps=3, clip=0.5)


def test_adamw_fp32_master_weights():
    # O2-style mixed precision: binary32 master and moments, BF16 model copy = RNE(master)
    pair = _mode_run(B.SR_FLAG_MASTER_FP32, True, lambda ps: [p.float().clone() for p in ps], clip=0.5)
    for i, h in enumerate(pair.host):
        assert bool(np.all(to_np(pair.aux[i]) == h["aux"]))          # master agrees to the bit
        want = torch.from_numpy(h["aux"]).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert bool(np.all(to_np(pair.p[i]) == want))


@pytest.mark.parametrize("variant", [B.SR_FLAG_EPS_IN_ROOT, B.SR_FLAG_DIV_BIAS,
                                     B.SR_FLAG_EPS_IN_ROOT | B.SR_FLAG_DIV_BIAS])
def test_adamw_arithmetic_variants(variant):
    # eps inside the root (Appendix B's form) and divisions by 1 - beta^t (lines 7-8 as printed),
    # on the default strategy, with FP32 moments + clip, and with Kahan
    _mode_run(variant, False, None, steps=4)
    _mode_run(variant, True, None, steps=3, clip=0.5)
    _mode_run(variant | B.SR_FLAG_KAHAN, False, lambda ps: [torch.zeros_like(p) for p in ps], steps=3)


def test_adamw_kahan_compensation():
    pair = _mode_run(B.SR_FLAG_KAHAN, False, lambda ps: [torch.zeros_like(p) for p in ps], steps=6)
    assert any(h["aux"].any() for h in pair.host)                     # compensation is in use


def test_adamw_does_not_write_outside_its_tensors():
    n = 1003
    bufs = [torch.full((n + 32,), 1.5, dtype=torch.bfloat16, device=DEV) for _ in range(4)]
    p, g, m, v = (b[9:9 + n] for b in bufs)
    tl = B.TensorList([p], [g], [m], [v])
    B.sr_adamw_step(tl, dict(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1), 1, 0)
    torch.cuda.synchronize()
    for b in (bufs[0], bufs[2], bufs[3]):
        outside = torch.cat([b[:9], b[9 + n:]])
        assert bool((outside == 1.5).all())
    assert bool((bufs[1] == 1.5).all())                    # gradients are never written


def test_adamw_geometry_and_list_independence():
    """Shared randomness (Algorithm 1 lines 9, 11): results depend on (seed, step, tensor id,
    element index) only -- not on list order, on how the list is split over calls, on a tensor
    being passed as shards with element offsets, or on running it twice from the same state."""
    sizes = [5000, 123, 8192, 77, 30001]
    hyper = dict(lr=6e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)

    def fresh():
        return [_random_state(n, 500 + i) for i, n in enumerate(sizes)]

    def run(order_calls, shard=False):
        st = fresh()
        for call in order_calls:
            ps, gs, ms, vs, ids, offs = [], [], [], [], [], []
            for i in call:
                p, g, m, v = st[i]
                if shard and sizes[i] > 4000:
                    cut = 2051                            # shard boundary inside an 8-block
                    for lo, hi in ((0, cut), (cut, sizes[i])):
                        ps.append(p[lo:hi]); gs.append(g[lo:hi]); ms.append(m[lo:hi]); vs.append(v[lo:hi])
                        ids.append(i); offs.append(lo)
                else:
                    ps.append(p); gs.append(g); ms.append(m); vs.append(v); ids.append(i); offs.append(0)
            tl = B.TensorList(ps, gs, ms, vs, False, ids, offs)
            B.sr_adamw_step(tl, hyper, 3, 42)
        torch.cuda.synchronize()
        return [[to_np(x) for x in (p, m, v)] for p, _, m, v in st]

    base = run([[0, 1, 2, 3, 4]])
    for variant in (run([[4, 3, 2, 1, 0]]), run([[2, 0], [4], [1, 3]]), run([[0, 1, 2, 3, 4]], shard=True),
                    run([[0, 1, 2, 3, 4]])):
        for a, b in zip(base, variant):
            for x, y in zip(a, b):
                assert bool(np.all(x == y))


def test_adamw_non_finite_and_extreme_inputs():
    """Infinities, NaNs, huge and subnormal values in every input: same outputs as the oracle
    (NaNs compared as NaNs), no flush to zero, overflow goes to infinity."""
    vals = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x007F, 0x0080, 0x7F7F, 0xFF7F, 0x7F80, 0xFF80,
                     0x7FC0, 0xFFC1, 0x3F80, 0xBF80, 0x0100, 0x7E00, 0x1234, 0x9234, 0x4000, 0x3C23],
                    dtype=np.uint16)
    rng = np.random.default_rng(0)
    n = 1 << 15
    cols = [vals[rng.integers(0, vals.size, n)] for _ in range(4)]
    cols[3] = cols[3] & 0x7FFF                             # second moment: non-negative patterns
    # half of the elements keep ordinary values in some inputs so that mixed cases occur
    ordinary = _random_state(n, 9)
    mix = rng.random((4, n)) < 0.5
    tensors = []
    for c, o, mk in zip(cols, ordinary, mix):
        tensors.append(bf16_dev(np.where(mk, c, to_np(o))))
    p, g, m, v = tensors
    pair = Pair([p], [m], [v], False)
    pair.g[0].copy_(g)
    hyper = dict(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    pair.step(hyper, 2, seed=17)
    pair.compare("extreme inputs")
    out = to_np(pair.p[0])
    assert is_nan16(out).any() and (out == 0x7F80).any()


def test_adamw_zero_lr_keeps_parameters():
    p, g, m, v = _random_state(10000, 3)
    before = to_np(p)
    tl = B.TensorList([p], [g], [m], [v])
    B.sr_adamw_step(tl, dict(lr=0.0, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0), 1, 5)
    torch.cuda.synchronize()
    assert bool(np.all(to_np(p) == before))


# ------------------------------------------------------------------ grad_global_norm

def _gpu_norm(grads):
    z = [torch.empty_like(g) for g in grads]
    tl = B.TensorList(z, grads, z, z)
    out = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(tl.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    B.grad_global_norm(tl, out, ws)
    torch.cuda.synchronize()
    return float(out.item())


def test_norm_exact_cases_on_device():
    ints = torch.randint(-3, 4, (1000003,), device=DEV).to(torch.bfloat16)
    S = int((ints.to(torch.int64) ** 2).sum().item())
    assert _gpu_norm([ints[:400001], ints[400001:]]) == float(np.float32(np.sqrt(np.float64(S))))
    a = torch.full((1 << 16,), -0.0078125, dtype=torch.bfloat16, device=DEV)
    assert _gpu_norm([a]) == 0.0078125 * 256.0
    tiny = torch.full((1 << 20,), 2.0 ** -10, dtype=torch.bfloat16, device=DEV)
    big = torch.tensor([4096.0], dtype=torch.bfloat16, device=DEV)
    assert _gpu_norm([big, tiny]) == float(np.float32(np.sqrt(np.float64(2 ** 24 + 1))))
    assert _gpu_norm([]) == 0.0
    assert _gpu_norm([tiny[:0]]) == 0.0


def test_norm_no_underflow_or_overflow_of_squares():
    small = torch.full((4096,), 1e-30, dtype=torch.bfloat16, device=DEV)     # squares < FP32 range
    want = ref.grad_global_norm([to_np(small)])
    assert want > 0 and _gpu_norm([small]) == want
    huge = torch.full((4096,), 1e30, dtype=torch.bfloat16, device=DEV)       # squares > FP32 range
    want = ref.grad_global_norm([to_np(huge)])
    assert np.isfinite(want) and _gpu_norm([huge]) == want


def test_norm_matches_oracle_on_gpt_list_and_misaligned_views():
    cfg = W.config(3)
    shapes = W.gpt_shapes(64, 2, 256, 5003, 64)
    grads = W.make_grads(shapes, DEV, W.data_seed(3, 1), cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
    want = ref.grad_global_norm([to_np(g) for g in grads])
    got = _gpu_norm(grads)
    assert got == want or abs(got - want) <= 1e-6 * want
    views = [g[1:] for g in grads if g.numel() > 1]
    want = ref.grad_global_norm([to_np(g) for g in views])
    got = _gpu_norm(views)
    assert got == want or abs(got - want) <= 1e-6 * want
    # non-finite gradients give a non-finite norm
    grads[3][5] = float("inf")
    assert np.isinf(_gpu_norm(grads))
    grads[3][5] = float("nan")
    assert np.isnan(_gpu_norm(grads))


def test_sum_of_squares_of_shards_adds_up_to_the_global_norm():
    """A gradient list split over four ranks: each rank's binary64 sum of squares, added on the host
    as one all-reduce of a double would, rooted and rounded once, is the norm of the whole list."""
    grads = W.make_grads(W.gpt_shapes(48, 2, 192, 1001, 32), DEV, 9, 1e-3, 0.01, 1.0)
    whole = B.TensorList(grads, grads, grads, grads)
    ws = torch.empty(max(whole.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    B.grad_global_norm(whole, norm, ws)
    total = 0.0
    for r in range(4):
        part = grads[r::4]
        tl = B.TensorList(part, part, part, part)
        s = torch.zeros(1, dtype=torch.float64, device=DEV)
        B.grad_sum_of_squares(tl, s, ws)
        torch.cuda.synchronize()
        want = sum(float((g.double() ** 2).sum().item()) for g in part)
        assert abs(float(s.item()) - want) <= 1e-12 * want
        total += float(s.item())
    got = float(np.float32(np.sqrt(total)))
    full = float(norm.item())
    assert got == full or abs(got - full) <= float(np.spacing(np.float32(full)))
    assert full == ref.grad_global_norm([to_np(g) for g in grads]) or \
        abs(full - ref.grad_global_norm([to_np(g) for g in grads])) <= 1e-6 * full


def test_norm_is_reproducible():
    g = W.make_grads(W.gpt_shapes(64, 2, 256, 5003, 64), DEV, 5, 1e-3)
    assert len({_gpu_norm(g) for _ in range(3)}) == 1


# ------------------------------------------------------------------ sr_grad_accumulate

def test_grad_accumulate_micro_batches_bit_exact_with_fused_norm():
    """Four micro-batches accumulated in BF16 with SR over a ragged, partly misaligned list; every
    step bit-exact; the norm written by the last call equals the oracle's norm of the result; a
    clipped update then consumes accumulator and norm."""
    sizes = [1, 9, 511, 512, 4097, 8192 * 3 + 5, 70001]
    accs, micro, offs = [], [], []
    for i, n in enumerate(sizes):
        shift = i % 3
        accs.append(torch.zeros(n + 8, dtype=torch.bfloat16, device=DEV)[shift:shift + n])
        micro.append(torch.empty(n + 8, dtype=torch.bfloat16, device=DEV)[(shift + i) % 2:(shift + i) % 2 + n])
        offs.append([0, 8, 3, 1 << 34][i % 4])
    al = B.AccumList(accs, micro, tensor_ids=[3 * i for i in range(len(sizes))], elem_offsets=offs)
    host = [to_np(a) for a in accs]
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(al.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    K = 4
    for k in range(K):
        W.fill_grads(micro, 900 + k, 1e-3)
        flags = B.SR_ACC_FIRST if k == 0 else 0
        last = k == K - 1
        B.sr_grad_accumulate(al, 1.0 / K, 100 + k, 77, flags, norm if last else None, ws if last else None)
        torch.cuda.synchronize()
        for i, h in enumerate(host):
            ref.grad_accumulate(h, to_np(micro[i]), 1.0 / K, 100 + k, 77, tensor_id=3 * i, elem_offset=offs[i],
                                flags=(ref.ACC_FIRST if k == 0 else 0))
            assert bool(np.all(to_np(accs[i]) == h)), f"micro-batch {k} tensor {i}"
    want = ref.grad_global_norm(host)
    got = float(norm.item())
    assert got == want or abs(got - want) <= 1e-6 * want
    # nearest-rounding variant
    W.fill_grads(micro, 999, 1e-3)
    B.sr_grad_accumulate(al, 0.5, 200, 77, B.SR_ACC_RNE)
    torch.cuda.synchronize()
    for i, h in enumerate(host):
        ref.grad_accumulate(h, to_np(micro[i]), 0.5, 200, 77, tensor_id=3 * i, elem_offset=offs[i], flags=ref.ACC_RNE)
        assert bool(np.all(to_np(accs[i]) == h))


def test_grad_accumulate_counter_indices_at_the_top_of_their_range():
    """Accumulation on slices that end on the largest counter index the library accepts
    (elem_offset + numel = 2^64 - 9 and a little below, aligned and mid-block), with the fused norm."""
    top = (1 << 64) - 1
    sizes = [3, 8, 513, 4 * 512 + 31, 30000]
    accs = [(torch.randn(n, device=DEV) * 1e-3).to(torch.bfloat16) for n in sizes]
    micro = [torch.empty(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    offs = [top - 8 - back - n for n, back in zip(sizes, (0, 3, 8, 1, 16))]
    al = B.AccumList(accs, micro, tensor_ids=[5 * i + 1 for i in range(len(sizes))], elem_offsets=offs)
    host = [to_np(a) for a in accs]
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(al.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    for k in range(2):
        W.fill_grads(micro, 950 + k, 1e-3)
        B.sr_grad_accumulate(al, 0.5, 7 + k, 0x0123456789ABCDEF, 0, norm, ws)
        torch.cuda.synchronize()
        for i, h in enumerate(host):
            ref.grad_accumulate(h, to_np(micro[i]), 0.5, 7 + k, 0x0123456789ABCDEF, tensor_id=5 * i + 1, elem_offset=offs[i])
            assert bool(np.all(to_np(accs[i]) == h)), f"micro-batch {k} tensor {i}"
        want = ref.grad_global_norm(host)
        got = float(norm.item())
        assert got == want or abs(got - want) <= 1e-6 * want
    bad = B.AccumList(accs[:1], micro[:1], tensor_ids=[1], elem_offsets=[top - 8 - sizes[0] + 1])
    with pytest.raises(B.SrError):
        B.sr_grad_accumulate(bad, 0.5, 9, 1, 0)


def test_grad_accumulate_norm_feeds_a_clipped_step():
    cfg = W.config(3)
    shapes = W.gpt_shapes(64, 2, 256, 5003, 64)
    pair = make_pair(cfg, shapes)
    micro = [torch.empty_like(g) for g in pair.g]
    al = B.AccumList(pair.g, micro)
    ws = torch.empty(max(al.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    for k in range(2):
        W.fill_grads(micro, 50 + k, cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
        B.sr_grad_accumulate(al, 0.5, 1 + k, 3, B.SR_ACC_FIRST if k == 0 else 0, pair.norm if k == 1 else None, ws)
    torch.cuda.synchronize()
    fused = float(pair.norm.item())
    # the separate two-pass norm of the same buffers gives the same value (same squares, same
    # binary64 arithmetic, different chunking: equal or one rounding apart)
    B.grad_global_norm(pair.tl, pair.norm, pair.ws)
    torch.cuda.synchronize()
    two_pass = float(pair.norm.item())
    assert fused == two_pass or abs(fused - two_pass) <= 1e-6 * two_pass
    want = ref.grad_global_norm([to_np(g) for g in pair.g])
    assert fused == want or abs(fused - want) <= 1e-6 * want
    pair.norm.fill_(fused)
    for h, g in zip(pair.host, pair.g):
        h["g"] = to_np(g)
    B.sr_adamw_step(pair.tl, cfg.hyper, 1, 0, 0, pair.norm, cfg.clip)
    torch.cuda.synchronize()
    ref.sr_adamw_step(pair.host, cfg.hyper, 1, 0, 0, norm=fused, max_norm=cfg.clip)
    pair.compare("step after fused accumulate+norm")


def test_grad_accumulate_special_values_and_empty():
    vals = np.array([0x0000, 0x8000, 0x0001, 0x8001, 0x7F7F, 0xFF7F, 0x7F80, 0xFF80, 0x7FC0, 0xFFC1,
                     0x3F80, 0xBF80, 0x0080, 0x1234, 0x9234], dtype=np.uint16)
    rng = np.random.default_rng(1)
    n = 1 << 14
    a = bf16_dev(vals[rng.integers(0, vals.size, n)])
    g = bf16_dev(vals[rng.integers(0, vals.size, n)])
    ha, hg = to_np(a), to_np(g)
    al = B.AccumList([a], [g])
    B.sr_grad_accumulate(al, 2.0, 5, 9)
    torch.cuda.synchronize()
    ref.grad_accumulate(ha, hg, 2.0, 5, 9)
    assert_bf16_parity(to_np(a), ha, "accumulate specials")
    B.sr_grad_accumulate(B.AccumList([], []), 1.0, 1, 0)
    e = torch.empty(0, dtype=torch.bfloat16, device=DEV)
    B.sr_grad_accumulate(B.AccumList([e], [e]), 1.0, 1, 0)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ randomized sweep

def test_adamw_randomized_cases():
    """Forty seeded random cases: list length, sizes, alignments, element offsets, tensor ids,
    strategy and variant flags, clipping, and hyper-parameters including the corners (beta = 0,
    eps = 0, zero weight decay, large learning rate, late steps)."""
    rng = np.random.default_rng(2024)
    strategies = [0, B.SR_FLAG_RNE_MOMENTS, B.SR_FLAG_RNE_PARAMS | B.SR_FLAG_RNE_MOMENTS, B.SR_FLAG_RNE_PARAMS,
                  B.SR_FLAG_FP32_MOMENTS, B.SR_FLAG_FP32_MOMENTS | B.SR_FLAG_RNE_PARAMS,
                  B.SR_FLAG_KAHAN, B.SR_FLAG_MASTER_FP32 | B.SR_FLAG_FP32_MOMENTS]
    for case in range(int(os.environ.get("SR_TEST_CASES", "40"))):     # more cases on request
        flags = strategies[case % len(strategies)]
        if rng.random() < 0.3:
            flags |= B.SR_FLAG_EPS_IN_ROOT
        if rng.random() < 0.3:
            flags |= B.SR_FLAG_DIV_BIAS
        fp32 = bool(flags & B.SR_FLAG_FP32_MOMENTS)
        n_t = int(rng.integers(1, 70))
        params, ms, vs, aux, grads, offs, ids = [], [], [], [], [], [], []
        for i in range(n_t):
            n = int(rng.choice([1, 5, 8, 64, 257, 512, 1000, 4099, 20000]))
            sh = [int(rng.integers(0, 3)) if rng.random() < 0.3 else 0 for _ in range(5)]
            p, g, m, v = _random_state(n + 8, 7000 + 100 * case + i, fp32)
            params.append(p[sh[0]:sh[0] + n]); grads.append(g[sh[1]:sh[1] + n])
            ms.append(m[sh[2]:sh[2] + n]); vs.append(v[sh[3]:sh[3] + n])
            offs.append(int(rng.choice([0, 0, 8, 3, 1 << 32, (1 << 40) + 5])))
            ids.append(int(rng.integers(0, 1 << 32)))
            if flags & B.SR_FLAG_KAHAN:
                aux.append((torch.randn(n + 8, device=DEV) * 1e-5).to(torch.bfloat16)[sh[4]:sh[4] + n])
            elif flags & B.SR_FLAG_MASTER_FP32:
                buf = torch.zeros(n + 8, device=DEV)
                buf[sh[4]:sh[4] + n] = params[-1].float() + torch.randn(n, device=DEV) * 1e-5
                aux.append(buf[sh[4]:sh[4] + n])
        pair = Pair(params, ms, vs, fp32, tensor_ids=ids, elem_offsets=offs, aux=aux if aux else None)
        for gd, gs in zip(pair.g, grads):
            gd.copy_(gs)
        hyper = dict(lr=float(rng.choice([0.0, 1e-5, 6e-4, 3e-3, 0.5])),
                     beta1=float(rng.choice([0.0, 0.5, 0.9, 0.99])),
                     beta2=float(rng.choice([0.0, 0.95, 0.999, 0.99999])),
                     eps=float(rng.choice([0.0, 1e-12, 1e-8, 1e-3])),
                     weight_decay=float(rng.choice([0.0, 0.1, 1.0])))
        t = int(rng.choice([1, 2, 17, 1000, 123456, 2 ** 32 - 1]))
        clip = None if rng.random() < 0.5 else float(rng.choice([1e-3, 0.05, 1.0, 100.0]))
        seed = int(rng.integers(0, 2 ** 63))
        pair.step(hyper, t, seed, clip=clip, flags=flags & ~B.SR_FLAG_FP32_MOMENTS)
        pair.compare(f"random case {case} flags {flags} t {t} clip {clip} hyper {hyper}")


# ------------------------------------------------------- resume and stagnation behaviour

def test_resume_from_copied_state_is_bit_identical():
    """The optimizer RNG is stateless: ten steps straight equal five steps, a 'restart' from a
    copy of the tensors in new buffers, and five more -- only (seed, step) carry over."""
    cfg = W.config(2)
    shapes = W.gpt_shapes(48, 1, 128, 501, 16)
    def fresh():
        p = W.make_params(shapes, DEV, 31, cfg.param_std)
        m, v = W.make_moments(shapes, DEV, False)
        g = [torch.empty_like(x) for x in p]
        return p, g, m, v
    p, g, m, v = fresh()
    tl = B.TensorList(p, g, m, v)
    for t in range(1, 11):
        W.fill_grads(g, 400 + t, 1e-3)
        B.sr_adamw_step(tl, cfg.hyper, t, 99)
    p2, g2, m2, v2 = fresh()
    tl2 = B.TensorList(p2, g2, m2, v2)
    for t in range(1, 6):
        W.fill_grads(g2, 400 + t, 1e-3)
        B.sr_adamw_step(tl2, cfg.hyper, t, 99)
    torch.cuda.synchronize()
    p3 = [x.clone() for x in p2]; m3 = [x.clone() for x in m2]; v3 = [x.clone() for x in v2]
    g3 = [torch.empty_like(x) for x in p3]
    del tl2, p2, m2, v2
    tl3 = B.TensorList(p3, g3, m3, v3)
    for t in range(6, 11):
        W.fill_grads(g3, 400 + t, 1e-3)
        B.sr_adamw_step(tl3, cfg.hyper, t, 99)
    torch.cuda.synchronize()
    for a, b in zip(p + m + v, p3 + m3 + v3):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_sub_spacing_updates_stagnate_under_nearest_rounding_only():
    """Section 2.1: with updates far below half a BF16 spacing, Q(x + u) = x for nearest rounding
    while E[Q_SR(x + u)] = x + u.  Parameters at 1.0 (spacing 2^-8 below), update about 6e-4."""
    n = 1 << 20
    hyper = dict(lr=6e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0)
    g = torch.full((n,), 1e-4, dtype=torch.bfloat16, device=DEV)

    def run(flags):
        p = torch.ones(n, dtype=torch.bfloat16, device=DEV)
        m = torch.zeros_like(p); v = torch.zeros_like(p)
        B.sr_adamw_step(B.TensorList([p], [g], [m], [v]), hyper, 1, 4, flags)
        torch.cuda.synchronize()
        return p.float()
    nearest = run(B.SR_FLAG_RNE_PARAMS | B.SR_FLAG_RNE_MOMENTS)
    assert bool((nearest == 1.0).all())
    sr = run(0)
    update = 6e-4                                            # lr * g/(|g| + eps) at step 1
    moved = float((1.0 - sr.double()).mean())
    q = update / 2.0 ** -8
    assert abs(moved - update) <= 5 * 2.0 ** -8 * np.sqrt(q * (1 - q) / n) + 1e-6
    assert set(torch.unique(sr).tolist()) == {1.0, 1.0 - 2.0 ** -8}


def test_norm_and_step_are_capturable_in_a_hip_graph():
    """The library only launches kernels whose tables travel in their arguments (no allocation,
    no memset, no host synchronisation), so norm + clipped step can be captured once and replayed.
    Three replays, with eager work and synchronisations between them, equal three eager calls."""
    cfg = W.config(3)
    shapes = W.gpt_shapes(48, 2, 192, 1001, 32)

    def fresh():
        p = W.make_params(shapes, DEV, 61, cfg.param_std)
        m, v = W.make_moments(shapes, DEV, False)
        g = W.make_grads(shapes, DEV, 62, cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
        tl = B.TensorList(p, g, m, v)
        return p, g, m, v, tl, torch.zeros(1, dtype=torch.float32, device=DEV), \
            torch.empty(max(tl.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)

    p, g, m, v, tl, norm, ws = fresh()
    for _ in range(3):
        B.grad_global_norm(tl, norm, ws)
        B.sr_adamw_step(tl, cfg.hyper, 5, 8, 0, norm, cfg.clip)
    torch.cuda.synchronize()
    eager = [to_np(x) for x in p + m + v]

    p2, g2, m2, v2, tl2, norm2, ws2 = fresh()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.grad_global_norm(tl2, norm2, ws2)
            B.sr_adamw_step(tl2, cfg.hyper, 5, 8, 0, norm2, cfg.clip)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    # capture does not execute: state is still the initial one
    scratch = torch.zeros(1024, device=DEV)
    for _ in range(3):
        graph.replay()
        scratch += 1.0                                    # unrelated eager work between replays
        torch.cuda.synchronize()
    for a, b in zip(eager, [to_np(x) for x in p2 + m2 + v2]):
        assert bool(np.all(a == b))


def test_stream_probe_leaves_data_unchanged():
    n = 100003
    ts = [(torch.randn(n + 8, device=DEV) * 0.01).to(torch.bfloat16)[1:1 + n] for _ in range(4)]
    before = [to_np(t) for t in ts]
    B.sr_stream_probe(*ts)
    aligned = [(torch.randn(4096, device=DEV) * 0.01).to(torch.bfloat16) for _ in range(4)]
    b2 = [to_np(t) for t in aligned]
    B.sr_stream_probe(*aligned)
    torch.cuda.synchronize()
    for t, b in zip(ts + aligned, before + b2):
        assert bool(np.all(to_np(t) == b))
    e = torch.empty(0, dtype=torch.bfloat16, device=DEV)
    B.sr_stream_probe(e, e, e, e)


def test_optimizer_object_drives_the_same_steps():
    """SRAdamW (bookkeeping only) on a small torch module equals direct calls through the binding,
    including clipping, an lr schedule, and a resume through state_dict."""
    from paper_2502_20566_amd.optimizer import SRAdamW
    torch.manual_seed(0)
    model = torch.nn.Sequential(torch.nn.Linear(64, 96), torch.nn.LayerNorm(96), torch.nn.Linear(96, 10)).to(DEV).to(torch.bfloat16)
    params = list(model.parameters())
    ref_p = [p.detach().clone().view(-1) for p in params]
    ref_m = [torch.zeros_like(p) for p in ref_p]
    ref_v = [torch.zeros_like(p) for p in ref_p]
    hyper = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    opt = SRAdamW(params, lr=3e-3, max_norm=0.5, seed=21)
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    x = torch.randn(32, 64, device=DEV, dtype=torch.bfloat16)
    for t in range(1, 6):
        lr = 3e-3 * (1.0 - 0.1 * t)
        loss = model(x).float().pow(2).mean()
        loss.backward()
        grads = [p.grad.detach().clone().view(-1) for p in params]
        opt.step(lr=lr)
        opt.zero_grad()
        tl = B.TensorList(ref_p, grads, ref_m, ref_v)
        ws = torch.empty(max(tl.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
        B.grad_global_norm(tl, norm, ws)
        B.sr_adamw_step(tl, dict(hyper, lr=lr), t, 21, 0, norm, 0.5)
        torch.cuda.synchronize()
        for a, b in zip(params, ref_p):
            assert torch.equal(a.detach().view(-1).view(torch.int16), b.view(torch.int16))
        if t == 3:                                            # resume into a fresh object
            sd = opt.state_dict()
            sd["state"] = [{k: v_.clone() for k, v_ in st.items()} for st in sd["state"]]
            opt = SRAdamW(params, lr=1.0, max_norm=0.5, seed=0)
            opt.load_state_dict(sd)


def test_optimizer_parameter_groups_and_torch_scheduler():
    """Two groups (weights with decay, biases and gains without), a torch LR scheduler driving
    `param_groups`, FP32 moments: equal to direct calls with one list per group, global tensor ids
    and one norm over all gradients."""
    from paper_2502_20566_amd.optimizer import SRAdamW
    torch.manual_seed(1)
    model = torch.nn.Sequential(torch.nn.Linear(40, 72), torch.nn.LayerNorm(72), torch.nn.Linear(72, 8)).to(DEV).to(torch.bfloat16)
    decay = [p for p in model.parameters() if p.ndim == 2]
    no_decay = [p for p in model.parameters() if p.ndim < 2]
    opt = SRAdamW([{"params": decay}, {"params": no_decay, "weight_decay": 0.0, "lr": 2e-3}], lr=1e-3,
                  betas=(0.9, 0.99), max_norm=1.0, seed=5, strategy="fp32_moments")
    sched = torch.optim.lr_scheduler.LambdaLR(opt, lambda e: 1.0 / (1 + e))
    groups = [decay, no_decay]
    ref_p = [[p.detach().clone().view(-1) for p in g] for g in groups]
    ref_m = [[torch.zeros(p.numel(), device=DEV) for p in g] for g in groups]
    ref_v = [[torch.zeros(p.numel(), device=DEV) for p in g] for g in groups]
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    x = torch.randn(16, 40, device=DEV, dtype=torch.bfloat16)
    for t in range(1, 5):
        model(x).float().pow(2).mean().backward()
        grads = [[p.grad.detach().clone().view(-1) for p in g] for g in groups]
        lrs = [g["lr"] for g in opt.param_groups]
        assert lrs == pytest.approx([1e-3 / t, 2e-3 / t])
        opt.step()
        opt.zero_grad()
        sched.step()
        flat_g = grads[0] + grads[1]
        every = B.TensorList(ref_p[0] + ref_p[1], flat_g, flat_g, flat_g)
        ws = torch.empty(max(every.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
        B.grad_global_norm(every, norm, ws)
        first = 0
        for gi in range(2):
            tl = B.TensorList(ref_p[gi], grads[gi], ref_m[gi], ref_v[gi], True,
                              tensor_ids=list(range(first, first + len(groups[gi]))))
            first += len(groups[gi])
            hyper = dict(lr=lrs[gi], beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.1 if gi == 0 else 0.0)
            B.sr_adamw_step(tl, hyper, t, 5, B.SR_FLAG_FP32_MOMENTS, norm, 1.0)
        torch.cuda.synchronize()
        for g, rp, rm in zip(groups, ref_p, ref_m):
            for a, b, m in zip(g, rp, rm):
                assert torch.equal(a.detach().view(-1).view(torch.int16), b.view(torch.int16))
                assert torch.equal(opt.state[a]["exp_avg"], m)
