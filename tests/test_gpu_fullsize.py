"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times.  Configs 2 and 3: every element of every tensor against the oracle after every one
of their 10 steps.  Configs 4 and 5: the GPU updates the whole parameter set; the oracle follows
seeded windows of it -- the first and last 2^20 elements of every tensor and 64 random windows of
2^20 elements, for config 5 also windows that straddle element index 2^32 -- through every step from
step 1, compared after every step (the update is element-wise and the RNG is random-access, so a
window with its element offset is self-contained).  Configs 4 and 5 in addition: one step (the third) of the
whole parameter set, every element.
"""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2502_20566_amd import binding as B
from paper_2502_20566_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


def to_np(t):
    if t.dtype == torch.bfloat16:
        return W.bf16_to_u16_numpy(t)
    return t.detach().cpu().numpy().copy()


def same_bf16(got, want):
    """Bit-exact, NaNs compared as NaNs; returns the number of mismatches."""
    gn = ((got & 0x7F80) == 0x7F80) & ((got & 0x7F) != 0)
    wn = ((want & 0x7F80) == 0x7F80) & ((want & 0x7F) != 0)
    return int(((got != want) & ~(gn & wn)).sum())


class Windows:
    """Host copies of slices [lo, lo+n) of some tensors, advanced by the oracle.  The slices of one
    array live back to back in one host array (one device gather and one download per array and
    step); the oracle sees each slice as a tensor of its own with its element offset."""

    def __init__(self, params, ms, vs, picks, fp32):
        self.picks = picks                      # list of (tensor index, lo, n)
        self.fp32 = fp32
        self.p, self.m, self.v = self.gather(params), self.gather(ms), self.gather(vs)
        self.host, at = [], 0
        for i, lo, n in picks:
            self.host.append(dict(p=self.p[at:at + n], m=self.m[at:at + n], v=self.v[at:at + n],
                                  tensor_id=i, elem_offset=lo))
            at += n
        self.numel = at

    def gather(self, tensors):
        return to_np(torch.cat([tensors[i][lo:lo + n] for i, lo, n in self.picks]))

    def step(self, grads, hyper, t, seed, norm, max_norm):
        g, at = self.gather(grads), 0
        for h, (i, lo, n) in zip(self.host, self.picks):
            h["g"] = g[at:at + n]
            at += n
        flags = ref.FLAG_FP32_MOMENTS if self.fp32 else 0
        ref.sr_adamw_step(self.host, hyper, t, seed, flags, norm=norm, max_norm=max_norm)

    def mismatches(self, params, ms, vs):
        bad = same_bf16(self.gather(params), self.p)
        gm, gv = self.gather(ms), self.gather(vs)
        if self.fp32:
            bad += int((gm.view(np.uint32) != self.m.view(np.uint32)).sum())
            bad += int((gv.view(np.uint32) != self.v.view(np.uint32)).sum())
        else:
            bad += same_bf16(gm, self.m) + same_bf16(gv, self.v)
        return bad


def window_picks(sizes, rng, width, n_random):
    """The windows followed through a full-size run: the first and the last `width` elements of
    every tensor (the whole tensor when it is no longer than two widths) and n_random windows of
    `width` elements at seeded random places, drawn over all elements of the tensors longer than
    one width (so a tensor's share of them follows its size)."""
    picks = []
    for i, n in enumerate(sizes):
        if n <= 2 * width:
            picks.append((i, 0, n))
        else:
            picks += [(i, 0, width), (i, n - width, width)]
    big = [(i, n) for i, n in enumerate(sizes) if n > width]
    weights = np.array([n for _, n in big], dtype=np.float64)
    for k in rng.choice(len(big), size=n_random, p=weights / weights.sum()):
        i, n = big[int(k)]
        picks.append((i, int(rng.integers(0, n - width + 1)), width))
    return picks


def setup(cfg):
    params = W.make_params(cfg.shapes, DEV, W.data_seed(cfg.index, 0), cfg.param_std)
    ms, vs = W.make_moments(cfg.shapes, DEV, cfg.fp32_moments)
    grads = [torch.empty_like(p) for p in params]
    tl = B.TensorList(params, grads, ms, vs, cfg.fp32_moments)
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = torch.empty(max(tl.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    return params, grads, ms, vs, tl, norm, ws


def gpu_step(cfg, tl, t, norm, ws):
    flags = B.SR_FLAG_FP32_MOMENTS if cfg.fp32_moments else 0
    if cfg.clip is not None:
        B.grad_global_norm(tl, norm, ws)
        B.sr_adamw_step(tl, cfg.hyper, t, cfg.seed, flags, norm, cfg.clip)
        torch.cuda.synchronize()
        return float(norm.item())
    B.sr_adamw_step(tl, cfg.hyper, t, cfg.seed, flags)
    torch.cuda.synchronize()
    return None


def full_compare(cfg, steps, check_norm_with_oracle):
    params, grads, ms, vs, tl, norm, ws = setup(cfg)
    host = [dict(p=to_np(p), m=to_np(m), v=to_np(v)) for p, m, v in zip(params, ms, vs)]
    for t in range(1, steps + 1):
        W.fill_grads(grads, W.data_seed(cfg.index, t), cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
        for h, g in zip(host, grads):
            h["g"] = to_np(g)
        nv = gpu_step(cfg, tl, t, norm, ws)
        if nv is not None and check_norm_with_oracle:
            want = ref.grad_global_norm([h["g"] for h in host])
            assert nv == want or abs(nv - want) <= 1e-6 * want, (t, nv, want)
        ref.sr_adamw_step(host, cfg.hyper, t, cfg.seed, 0, norm=nv, max_norm=cfg.clip or 0.0)
        bad = 0
        for i, h in enumerate(host):
            bad += same_bf16(to_np(params[i]), h["p"]) + same_bf16(to_np(ms[i]), h["m"]) + same_bf16(to_np(vs[i]), h["v"])
        assert bad == 0, f"{cfg.name} step {t}: {bad} mismatching values"
    return params, host


def test_config2_full_buffers_ten_steps():
    cfg = W.config(2)
    p0 = W.make_params(cfg.shapes, DEV, W.data_seed(2, 0), cfg.param_std)
    params, host = full_compare(cfg, 10, False)
    # parameters keep moving under SR (no stagnation); report how many updates were sub-spacing
    wte_before = ref.bf16_bits_to_f32(to_np(p0[0])).astype(np.float64)
    wte_after = ref.bf16_bits_to_f32(host[0]["p"]).astype(np.float64)
    assert float((wte_after != wte_before).mean()) > 0.05


def test_config3_full_buffers_clip():
    """All 10 steps of the configuration, every element of every tensor after every step; the
    device's norm against the oracle's at every step."""
    cfg = W.config(3)
    assert cfg.steps == 10
    full_compare(cfg, cfg.steps, True)


def test_config4_full_size_windows_fp32_moments_clip():
    """The whole 2.65e9-element list is updated on the GPU; the oracle follows the first and the
    last 2^20 elements of every one of the 388 tensors (whole tensors up to 2^21 elements) and 64
    random windows of 2^20 elements through all 5 steps, compared after every step."""
    cfg = W.config(4)
    params, grads, ms, vs, tl, norm, ws = setup(cfg)
    assert len(params) == 388 and cfg.steps == 5
    picks = window_picks([p.numel() for p in params], np.random.default_rng(4), 1 << 20, 64)
    assert {i for i, _, _ in picks} == set(range(len(params)))
    win = Windows(params, ms, vs, picks, True)
    assert win.numel > 300 * (1 << 20)
    for t in range(1, cfg.steps + 1):
        W.fill_grads(grads, W.data_seed(4, t), cfg.grad_std)
        nv = gpu_step(cfg, tl, t, norm, ws)
        # the norm against a binary64 reduction by an independent library routine
        s = 0.0
        for g in grads:
            s += float(g.double().pow(2).sum().item())
        want = float(np.float32(np.sqrt(s)))
        assert nv == want or abs(nv - want) <= 1e-6 * want, (t, nv, want)
        win.step(grads, cfg.hyper, t, cfg.seed, nv, cfg.clip)
        assert win.mismatches(params, ms, vs) == 0, f"config 4 step {t}"


def test_config4_every_element_of_one_step():
    """All 2 651 591 680 elements of the 388-tensor list with binary32 moments and clipping: three
    steps on the GPU, the state before the third kept on the device, and the oracle redoes that
    step tensor by tensor (in slabs of 2^27 elements, each a slice with its element offset) with
    the norm the device computed; p and the binary32 m and v must come out bit for bit."""
    cfg = W.config(4)
    params, grads, ms, vs, tl, norm, ws = setup(cfg)
    for t in (1, 2):
        W.fill_grads(grads, W.data_seed(4, t), cfg.grad_std)
        gpu_step(cfg, tl, t, norm, ws)
    W.fill_grads(grads, W.data_seed(4, 3), cfg.grad_std)
    before = [[x.clone() for x in arr] for arr in (params, ms, vs)]
    nv = gpu_step(cfg, tl, 3, norm, ws)
    slab, done = 1 << 27, 0
    for i in range(len(params)):
        n = params[i].numel()
        for lo in range(0, n, slab):
            k = min(slab, n - lo)
            h = dict(p=to_np(before[0][i][lo:lo + k]), m=to_np(before[1][i][lo:lo + k]), v=to_np(before[2][i][lo:lo + k]),
                     g=to_np(grads[i][lo:lo + k]), tensor_id=i, elem_offset=lo)
            ref.sr_adamw_step([h], cfg.hyper, 3, cfg.seed, ref.FLAG_FP32_MOMENTS, norm=nv, max_norm=cfg.clip)
            bad = same_bf16(to_np(params[i][lo:lo + k]), h["p"])
            bad += int((to_np(ms[i][lo:lo + k]).view(np.uint32) != h["m"].view(np.uint32)).sum())
            bad += int((to_np(vs[i][lo:lo + k]).view(np.uint32) != h["v"].view(np.uint32)).sum())
            assert bad == 0, f"config 4, whole list: mismatches in tensor {i} at element {lo}"
            done += k
    assert done == 2651591680


def test_config5_full_size_windows_through_warm_start():
    """The 6.7B flat buffer through its 100 warm steps and the timed step 101: the oracle follows
    the first and last 2^20 elements, windows that straddle element index 2^32 (where the counter's
    low word wraps), a few ragged ones, and 64 random windows of 2^20 elements; every window is
    compared after every step."""
    cfg = W.config(5)
    params, grads, ms, vs, tl, norm, ws = setup(cfg)
    n = params[0].numel()
    assert n == 6658465792
    w = 1 << 20
    picks = window_picks([n], np.random.default_rng(5), w, 64)
    picks += [(0, (1 << 32) - w // 2, w), (0, (1 << 32) + 3, w - 5), (0, (1 << 32) - 1, 2),
              (0, 3 * (1 << 31) - 77, w), (0, n - 7, 7), (0, 12345, 999)]
    win = Windows(params, ms, vs, picks, False)
    steps = cfg.warm_steps + 1
    for t in range(1, steps + 1):
        W.fill_grads(grads, W.data_seed(5, t), cfg.grad_std)
        gpu_step(cfg, tl, t, norm, ws)
        win.step(grads, cfg.hyper, t, cfg.seed, None, 0.0)
        assert win.mismatches(params, ms, vs) == 0, f"config 5 step {t}"
    # after the warm start the second moment is alive and updates are far below a BF16 spacing
    v_end = ref.bf16_bits_to_f32(win.host[0]["v"])
    assert float((v_end > 0).mean()) > 0.99


def test_config5_every_element_of_one_step():
    """The whole 6.7B flat buffer, every one of its 6 658 465 792 elements: three steps on the GPU
    (so that the moments are alive), the state before the third kept on the device, and the oracle
    redoes that step slab by slab (2^27 elements, each a slice with its element offset) on the
    host; p, m and v of every slab must come out bit for bit."""
    cfg = W.config(5)
    params, grads, ms, vs, tl, norm, ws = setup(cfg)
    n = params[0].numel()
    for t in (1, 2):
        W.fill_grads(grads, W.data_seed(5, t), cfg.grad_std)
        gpu_step(cfg, tl, t, norm, ws)
    W.fill_grads(grads, W.data_seed(5, 3), cfg.grad_std)
    before = [params[0].clone(), ms[0].clone(), vs[0].clone()]
    gpu_step(cfg, tl, 3, norm, ws)
    slab, bad, moved = 1 << 27, 0, 0
    for lo in range(0, n, slab):
        k = min(slab, n - lo)
        h = dict(p=to_np(before[0][lo:lo + k]), m=to_np(before[1][lo:lo + k]), v=to_np(before[2][lo:lo + k]),
                 g=to_np(grads[0][lo:lo + k]), tensor_id=0, elem_offset=lo)
        p0 = h["p"].copy()
        ref.sr_adamw_step([h], cfg.hyper, 3, cfg.seed, 0)
        moved += int((h["p"] != p0).sum())
        bad += same_bf16(to_np(params[0][lo:lo + k]), h["p"])
        bad += same_bf16(to_np(ms[0][lo:lo + k]), h["m"]) + same_bf16(to_np(vs[0][lo:lo + k]), h["v"])
        assert bad == 0, f"config 5, whole buffer: mismatches in the slab at element {lo}"
    assert moved > n // 100                                   # the step did move parameters


def test_config5_full_size_windows_8_bit_moments():
    """The 6.7B flat buffer with the moments held in 8 bits (extension), 40 steps from zero: the
    oracle follows the same windows, codes and parameters bit for bit (NaN codes as NaN codes)."""
    import bench
    cfg = W.config(5)
    exps = bench.fp8_scale_exponents(cfg)
    params = W.make_params(cfg.shapes, DEV, W.data_seed(cfg.index, 0), cfg.param_std)
    n = params[0].numel()
    ms = [torch.zeros(n, dtype=torch.uint8, device=DEV)]
    vs = [torch.zeros(n, dtype=torch.uint8, device=DEV)]
    grads = [torch.empty_like(params[0])]
    tl = B.TensorList(params, grads, ms, vs, fp8_exponents=[exps])
    rng = np.random.default_rng(58)
    w = 1 << 16
    picks = [(0, w), (n - w, w), ((1 << 32) - w // 2, w), ((1 << 32) + 3, w - 5), (n - 7, 7), (12345, 999)]
    picks += [(int(rng.integers(0, n - w)), w) for _ in range(10)]
    host = [dict(p=to_np(params[0][lo:lo + k]), m=to_np(ms[0][lo:lo + k]), v=to_np(vs[0][lo:lo + k]),
                 m_exp=exps[0], v_exp=exps[1], tensor_id=0, elem_offset=lo) for lo, k in picks]
    for t in range(1, 41):
        W.fill_grads(grads, W.data_seed(5, t), cfg.grad_std)
        B.sr_adamw_step(tl, cfg.hyper, t, cfg.seed, B.SR_FLAG_FP8_MOMENTS)
        torch.cuda.synchronize()
        for h, (lo, k) in zip(host, picks):
            h["g"] = to_np(grads[0][lo:lo + k])
        ref.sr_adamw_step(host, cfg.hyper, t, cfg.seed, ref.FLAG_FP8_MOMENTS)
        if t in (1, 2, 20, 40):
            bad = 0
            for h, (lo, k) in zip(host, picks):
                bad += same_bf16(to_np(params[0][lo:lo + k]), h["p"])
                gm, gv = to_np(ms[0][lo:lo + k]), to_np(vs[0][lo:lo + k])
                bad += int(((gm != h["m"]) & ~((gm & 0x7F) == 0x7F)).sum())
                bad += int(((gv != h["v"]) & ~((gv & 0x7F) > 0x7C)).sum())
            assert bad == 0, f"config 5, 8-bit moments, step {t}: {bad} mismatches"
    # the state lives inside the formats: nothing saturated, nothing infinite, most of v alive
    m_end, v_end = host[0]["m"], host[0]["v"]
    assert not ((m_end & 0x7F) >= 0x7E).any() and not (v_end >= 0x7C).any()
    assert float((v_end > 0).mean()) > 0.99


def _quantize_params(params, p_exp, seed):
    """The BF16 weights onto the E4M3 grid of scale 2^p_exp with the library's stochastic cast."""
    out = []
    for i, p in enumerate(params):
        q = torch.empty(p.numel(), dtype=torch.uint8, device=DEV)
        for at in range(0, p.numel(), 1 << 28):
            B.sr_cast_f32_fp8(p[at:at + (1 << 28)].float() * float(2.0 ** p_exp), q[at:at + (1 << 28)], B.SR_FP8_E4M3, seed, 0, i)
        out.append(q)
    torch.cuda.synchronize()
    return out


def _same_codes(got, want, nan):
    return int(((got != want) & ~(nan(got) & nan(want))).sum())


def test_config2_list_with_8_bit_parameters():
    """The 148-tensor list at full size with the parameters held as E4M3 codes (extension) and BF16
    moments: every element of every tensor against the oracle for three steps."""
    cfg = W.config(2)
    p_exp = 8
    params = _quantize_params(W.make_params(cfg.shapes, DEV, W.data_seed(2, 0), cfg.param_std), p_exp, 3)
    ms, vs = W.make_moments(cfg.shapes, DEV, False)
    grads = [torch.empty(p.numel(), dtype=torch.bfloat16, device=DEV) for p in params]
    tl = B.TensorList(params, grads, ms, vs, fp8_param_exponents=[p_exp] * len(params))
    host = [dict(p=p.cpu().numpy(), m=to_np(m), v=to_np(v), p_exp=p_exp) for p, m, v in zip(params, ms, vs)]
    nan4 = lambda c: (c & 0x7F) == 0x7F
    for t in range(1, 4):
        W.fill_grads(grads, W.data_seed(2, t), cfg.grad_std)
        for h, g in zip(host, grads):
            h["g"] = to_np(g)
        B.sr_adamw_step(tl, cfg.hyper, t, cfg.seed, B.SR_FLAG_FP8_PARAMS)
        torch.cuda.synchronize()
        ref.sr_adamw_step(host, cfg.hyper, t, cfg.seed, ref.FLAG_FP8_PARAMS)
        bad = 0
        for i, h in enumerate(host):
            bad += _same_codes(params[i].cpu().numpy(), h["p"], nan4) + same_bf16(to_np(ms[i]), h["m"]) + same_bf16(to_np(vs[i]), h["v"])
        assert bad == 0, f"config 2, 8-bit parameters, step {t}: {bad} mismatches"
    # under SR the codes keep moving although every update is well below one E4M3 spacing
    start = _quantize_params(W.make_params(cfg.shapes[:1], DEV, W.data_seed(2, 0), cfg.param_std), p_exp, 3)[0]
    assert 1e-4 < float((params[0] != start).float().mean()) < 0.9


def test_config5_flat_buffer_all_state_in_8_bits():
    """The 6.7B flat buffer with parameters and both moments in 8 bits (extension), six steps from
    zero moments: the oracle follows the first and last 2^18 elements, a window across element
    index 2^32 and 16 random windows, codes bit for bit (NaN codes as NaN codes)."""
    import bench
    cfg = W.config(5)
    exps = bench.fp8_scale_exponents(cfg)
    p_exp = 8
    params = _quantize_params(W.make_params(cfg.shapes, DEV, W.data_seed(5, 0), cfg.param_std), p_exp, 5)
    n = params[0].numel()
    ms = [torch.zeros(n, dtype=torch.uint8, device=DEV)]
    vs = [torch.zeros(n, dtype=torch.uint8, device=DEV)]
    grads = [torch.empty(n, dtype=torch.bfloat16, device=DEV)]
    tl = B.TensorList(params, grads, ms, vs, fp8_exponents=[exps], fp8_param_exponents=[p_exp])
    w = 1 << 18
    picks = [(lo, k) for _, lo, k in window_picks([n], np.random.default_rng(59), w, 16)]
    picks += [((1 << 32) - w // 2, w), ((1 << 32) + 3, w - 5), (n - 7, 7)]
    host = [dict(p=params[0][lo:lo + k].cpu().numpy(), m=to_np(ms[0][lo:lo + k]), v=to_np(vs[0][lo:lo + k]),
                 p_exp=p_exp, m_exp=exps[0], v_exp=exps[1], tensor_id=0, elem_offset=lo) for lo, k in picks]
    nan4, nan5 = (lambda c: (c & 0x7F) == 0x7F), (lambda c: (c & 0x7F) > 0x7C)
    for t in range(1, 7):
        W.fill_grads(grads, W.data_seed(5, t), cfg.grad_std)
        B.sr_adamw_step(tl, cfg.hyper, t, cfg.seed, B.SR_FLAG_FP8_PARAMS | B.SR_FLAG_FP8_MOMENTS)
        torch.cuda.synchronize()
        for h, (lo, k) in zip(host, picks):
            h["g"] = to_np(grads[0][lo:lo + k])
        ref.sr_adamw_step(host, cfg.hyper, t, cfg.seed, ref.FLAG_FP8_PARAMS | ref.FLAG_FP8_MOMENTS)
        bad = 0
        for h, (lo, k) in zip(host, picks):
            bad += _same_codes(params[0][lo:lo + k].cpu().numpy(), h["p"], nan4)
            bad += _same_codes(to_np(ms[0][lo:lo + k]), h["m"], nan4) + _same_codes(to_np(vs[0][lo:lo + k]), h["v"], nan5)
        assert bad == 0, f"config 5, all state in 8 bits, step {t}: {bad} mismatches"


def test_cast_every_binary32_encoding():
    """All 2^32 binary32 encodings (every exponent, subnormal, infinity and NaN payload), each with
    the draw its index gets: the GPU cast equals the by-value oracle bit for bit."""
    chunk = 1 << 28
    bad = 0
    for c in range(16):
        bits = torch.arange(c * chunk, (c + 1) * chunk, dtype=torch.int64, device=DEV).to(torch.int32)  # wraps
        x = bits.view(torch.float32)
        out = torch.empty(chunk, dtype=torch.bfloat16, device=DEV)
        B.sr_cast_f32_bf16(x, out, 0x5EED, 1 + c, 3)
        torch.cuda.synchronize()
        want = ref.sr_cast_f32_bf16(x.cpu().numpy(), 0x5EED, 1 + c, 3)
        bad += int((to_np(out) != want).sum())
        del bits, x, out
    assert bad == 0


def test_grad_accumulate_full_size_with_fused_norm():
    """Config-3 parameter list (355M elements, 292 tensors): two micro-batches accumulated with SR;
    every element against the oracle; the fused norm (several hundred thousand partial sums, folded
    in two levels) against the oracle's norm of the result."""
    cfg = W.config(3)
    accs = [torch.zeros(W.numel_of(sh), dtype=torch.bfloat16, device=DEV) for _, sh, _ in cfg.shapes]
    micro = [torch.empty_like(a) for a in accs]
    al = B.AccumList(accs, micro)
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = torch.empty(al.workspace_bytes(), dtype=torch.uint8, device=DEV)
    host = [to_np(a) for a in accs]
    for k in range(2):
        W.fill_grads(micro, W.data_seed(3, 70 + k), cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
        B.sr_grad_accumulate(al, 0.5, 10 + k, 5, B.SR_ACC_FIRST if k == 0 else 0, norm if k == 1 else None, ws)
        torch.cuda.synchronize()
        for i, h in enumerate(host):
            ref.grad_accumulate(h, to_np(micro[i]), 0.5, 10 + k, 5, tensor_id=i, flags=ref.ACC_FIRST if k == 0 else 0)
    bad = sum(int((to_np(a) != h).sum()) for a, h in zip(accs, host))
    assert bad == 0
    want = ref.grad_global_norm(host)
    got = float(norm.item())
    assert got == want or abs(got - want) <= 1e-6 * want, (got, want)


# ------------------------------------------------------------------ beyond one dispatch

ONE_DISPATCH = 1 << 26            # workgroups of 64 lanes in 2^32 work-items


def _need_free_memory(gib: float):
    """These two tests want most of the card: release what earlier tests left cached, and skip
    (rather than fail on an allocation) when the device does not have the room right now."""
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < gib * (1 << 30):
        pytest.skip(f"needs {gib:.0f} GiB of free device memory, {free / (1 << 30):.0f} GiB available")


def _fill_normal(t: torch.Tensor, seed: int, std: float):
    gen = torch.Generator(device=DEV).manual_seed(seed)
    for s0 in range(0, t.numel(), 1 << 28):
        piece = t[s0:s0 + (1 << 28)]
        piece.copy_(torch.randn(piece.numel(), device=DEV, generator=gen) * std)


def test_cast_larger_than_one_dispatch():
    """The BF16 cast gives a workgroup 256 elements, so 2^34 elements fill one dispatch.  An array of
    2^34 + 2^20 + 5 binary32 values (68.7 GB in, 34.4 GB out) takes two launches; windows at the
    start, across the cut and at the ragged end equal the oracle."""
    _need_free_memory(110)
    n = ONE_DISPATCH * 256 + (1 << 20) + 5
    x = torch.empty(n, dtype=torch.float32, device=DEV)
    _fill_normal(x, 11, 1.0)
    out = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    B.sr_cast_f32_bf16(x, out, 99, 3, 8)
    torch.cuda.synchronize()
    w = 1 << 16
    for lo, m in ((0, w), (ONE_DISPATCH * 256 - w, 2 * w), (n - w - 5, w + 5), (12345678901, w)):
        want = ref.sr_cast_f32_bf16(x[lo:lo + m].cpu().numpy(), 99, 3, 8, elem_offset=lo)
        assert np.array_equal(to_np(out[lo:lo + m]), want), lo
    del x, out
    torch.cuda.empty_cache()


def test_fp32_moment_update_larger_than_one_dispatch():
    """With binary32 moments a workgroup owns 256 elements: one flat tensor of 2^34 + 2^20 + 24
    elements (206 GB of p, g, m, v) is cut into two pieces, launched separately.  Two steps with
    clipping (the norm over 2.6e5 chunks); windows at the start, across the cut and at the end
    follow the oracle."""
    _need_free_memory(215)
    n = ONE_DISPATCH * 256 + (1 << 20) + 24
    p = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    g = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    _fill_normal(p, 21, 0.02)
    m = torch.zeros(n, dtype=torch.float32, device=DEV)
    v = torch.zeros(n, dtype=torch.float32, device=DEV)
    tl = B.TensorList([p], [g], [m], [v], True, tensor_ids=[6])
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    ws = torch.empty(tl.workspace_bytes(), dtype=torch.uint8, device=DEV)
    w = 1 << 16
    picks = [(0, 0, w), (0, ONE_DISPATCH * 256 - w, 2 * w), (0, n - w, w), (0, 9876543210, w)]
    win = Windows([p], [m], [v], picks, True)
    for h in win.host:
        h["tensor_id"] = 6
    hyper = dict(lr=1.6e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    for t in (1, 2):
        _fill_normal(g, 30 + t, 1e-4)
        B.grad_global_norm(tl, norm, ws)
        B.sr_adamw_step(tl, hyper, t, 17, B.SR_FLAG_FP32_MOMENTS, norm, 1.0)
        torch.cuda.synchronize()
        nv = float(norm.item())
        assert abs(nv - 1e-4 * np.sqrt(n)) < 0.01 * nv                   # sigma * sqrt(n)
        win.step([g], hyper, t, 17, nv, 1.0)
        assert win.mismatches([p], [m], [v]) == 0, f"step {t}"
    del p, g, m, v
    torch.cuda.empty_cache()
