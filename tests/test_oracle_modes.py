"""Pins of the oracle's comparison strategies (CPU only): the all-nearest-rounding "BF16" strategy
and O2-style FP32 master weights of Section 5.1, and BF16 + Kahan summation (Section 1's related
work).  Pinned against torch's BF16 cast (a library's round-to-nearest-even), a free-running
torch.optim.AdamW in FP32, a binary64 AdamW trajectory, and the stagnation argument of Section 2.1.
"""
import numpy as np
import pytest

from oracle import ref

torch = pytest.importorskip("torch")

HYP = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)


def f32(x):
    return np.float32(x)


def trunc_bits(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def val(bits16):
    return ref.bf16_bits_to_f32(np.asarray(bits16, np.uint16))


def torch_rne_bits(x: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def adamw64(p, g, m, v, hyper, t):
    """Algorithm 1 lines 5-10 (eps outside the root) in binary64 from float32-valued hypers."""
    b1, b2, lr, eps, wd = (float(f32(hyper[k])) for k in ("beta1", "beta2", "lr", "eps", "weight_decay"))
    m = b1 * m + (1 - b1) * g
    v = b2 * v + (1 - b2) * g * g
    u = (m / (1 - b1 ** t)) / (np.sqrt(v / (1 - b2 ** t)) + eps)
    return p - (lr * u + lr * wd * p), m, v


def test_all_nearest_strategy_equals_library_cast_of_the_unrounded_values():
    n = 4096
    rng = np.random.default_rng(0)
    p = trunc_bits(rng.standard_normal(n) * 0.02)
    m = trunc_bits(rng.standard_normal(n) * 1e-3)
    v = trunc_bits(rng.random(n) * 1e-6)
    flags = ref.FLAG_RNE_PARAMS | ref.FLAG_RNE_MOMENTS
    for t in (1, 2, 3):
        g = trunc_bits(rng.standard_normal(n) * 1e-3)
        s = ref.adamw_scalars(step=t, **HYP)
        y, m1, v1 = ref.adamw_unrounded(p, g, m, v, s)
        outs = []
        for seed in (0, 1):                                   # no random bits: the seed is irrelevant
            pp, mm, vv = p.copy(), m.copy(), v.copy()
            ref.sr_adamw_step([dict(p=pp, g=g, m=mm, v=vv)], HYP, t, seed, flags)
            outs.append((pp, mm, vv))
        for a, b in zip(outs[0], outs[1]):
            assert bool(np.all(a == b))
        p, m, v = outs[0]
        assert bool(np.all(p == torch_rne_bits(y)))
        assert bool(np.all(m == torch_rne_bits(m1)))
        assert bool(np.all(v == torch_rne_bits(v1)))
    # RNE on the parameter only (moments still stochastic) is also available
    pp, mm, vv = p.copy(), m.copy(), v.copy()
    s = ref.adamw_scalars(step=4, **HYP)
    y, _, _ = ref.adamw_unrounded(p, g, m, v, s)
    ref.sr_adamw_step([dict(p=pp, g=g, m=mm, v=vv)], HYP, 4, 0, ref.FLAG_RNE_PARAMS)
    assert bool(np.all(pp == torch_rne_bits(y)))


def test_master_weights_follow_a_free_running_fp32_torch_adamw():
    n, T = 2048, 25
    rng = np.random.default_rng(1)
    x32 = (rng.standard_normal(n) * 0.02).astype(np.float32)
    p16 = torch_rne_bits(x32)
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    tp = torch.nn.Parameter(torch.from_numpy(x32.copy()))
    opt = torch.optim.AdamW([tp], lr=HYP["lr"], betas=(HYP["beta1"], HYP["beta2"]), eps=HYP["eps"],
                            weight_decay=HYP["weight_decay"], foreach=False)
    flags = ref.FLAG_MASTER_FP32 | ref.FLAG_FP32_MOMENTS
    x0 = x32.astype(np.float64)
    for t in range(1, T + 1):
        g = trunc_bits(rng.standard_normal(n) * 1e-3)
        tp.grad = torch.from_numpy(val(g).copy())
        opt.step()
        ref.sr_adamw_step([dict(p=p16, g=g, m=m, v=v, aux=x32)], HYP, t, 0, flags)
        assert bool(np.all(p16 == torch_rne_bits(x32)))      # the BF16 model copy is RNE(master)
    ty = tp.detach().numpy().astype(np.float64)
    moved = np.abs(ty - x0)
    # both are FP32 AdamW with different operation orders: over 25 steps their roundings walk a
    # few binary32 spacings apart -- thousands of times closer than a BF16 parameter could follow
    scale = np.maximum(np.abs(ty), np.abs(x0)).astype(np.float32)
    # (an element that passes close to zero keeps the absolute error of its larger past values)
    assert bool(np.all(np.abs(x32 - ty) <= 16 * np.spacing(scale) + 4e-6 * HYP["lr"] * T))
    assert float(np.median(moved / np.spacing(scale))) > 1e5
    assert float(np.median(moved)) > 1e-3
    st = opt.state[tp]
    # moments: absolute agreement at the scale of the gradients (sums can cancel)
    assert float(np.max(np.abs(m - st["exp_avg"].numpy()))) < 1e-6 * 1e-3
    assert float(np.max(np.abs(v - st["exp_avg_sq"].numpy()))) < 1e-6 * 1e-5


def _run_strategy(flags, p0, grads, with_aux):
    n = p0.size
    p, m, v = p0.copy(), np.zeros(n, np.uint16), np.zeros(n, np.uint16)
    aux = np.zeros(n, np.uint16) if with_aux else None
    for t, g in enumerate(grads, 1):
        d = dict(p=p, g=g, m=m, v=v)
        if with_aux:
            d["aux"] = aux
        ref.sr_adamw_step([d], dict(HYP, lr=2e-5, weight_decay=0.0), t, 7, flags)
    return p, aux


def test_kahan_tracks_the_exact_trajectory_where_nearest_rounding_stagnates():
    """Parameters near 1.0 (BF16 spacing 2^-7 ... 2^-8), 200 steps whose updates (about 2e-5) are
    far below half a spacing: nearest rounding never moves, Kahan's p - c follows the binary64
    trajectory to within one spacing of the small compensation term, SR follows it in the mean."""
    n, T = 4096, 200
    rng = np.random.default_rng(2)
    p0 = trunc_bits(np.full(n, 1.0, np.float32))
    grads = [trunc_bits(np.abs(rng.standard_normal(n)) * 1e-3 + 1e-4) for _ in range(T)]   # same sign: steady drift
    hyper = dict(HYP, lr=2e-5, weight_decay=0.0)
    # binary64 trajectory with BF16-rounded moments replaced by exact ones (moments only matter
    # through u ~ 1, so the drift is ~ lr per step either way)
    x, m, v = np.ones(n), np.zeros(n), np.zeros(n)
    for t, g in enumerate(grads, 1):
        x, m, v = adamw64(x, val(g).astype(np.float64), m, v, hyper, t)
    drift = 1.0 - x
    assert 2e-3 < float(drift.mean()) < 5e-3                   # ~ T * lr, about one spacing (2^-8 = 3.9e-3)

    p_nr, _ = _run_strategy(ref.FLAG_RNE_PARAMS | ref.FLAG_RNE_MOMENTS, p0, grads, False)
    assert bool(np.all(p_nr == p0))                             # Q(x + u) = x: stagnation

    p_k, c_k = _run_strategy(ref.FLAG_KAHAN, p0, grads, True)
    xk = val(p_k).astype(np.float64) - val(c_k).astype(np.float64)
    # the compensated value follows the drift; allow the effect of BF16-rounded moments (a few %)
    err = np.abs((1.0 - xk) - drift)
    assert float(np.median(err / drift)) < 0.05
    assert bool(np.all(err < 0.25 * drift + 2.0 ** -12))
    assert float((p_k != p0).mean()) > 0.3                      # parameters did cross to the next level

    p_sr, _ = _run_strategy(0, p0, grads, False)
    mean_move = float((1.0 - val(p_sr).astype(np.float64)).mean())
    assert abs(mean_move - float(drift.mean())) < 0.1 * float(drift.mean())


def test_kahan_single_step_algebra():
    """One step against numpy binary32 operations taken one at a time and torch's RNE cast."""
    n = 2048
    rng = np.random.default_rng(3)
    p = trunc_bits(rng.standard_normal(n) * 0.02)
    g = trunc_bits(rng.standard_normal(n) * 1e-3)
    m = trunc_bits(rng.standard_normal(n) * 1e-3)
    v = trunc_bits(rng.random(n) * 1e-6)
    c = trunc_bits(rng.standard_normal(n) * 1e-5)
    s = ref.adamw_scalars(step=3, **HYP)
    y, m1, v1 = ref.adamw_unrounded(p, g, m, v, s)
    pv = val(p)
    total = (pv - y).astype(np.float32)          # not the kernel's `sum` in general: recompute it
    mh = (m1 * s.rbc1).astype(np.float32)
    d = (np.sqrt((v1 * s.rbc2).astype(np.float32)).astype(np.float32) + s.eps).astype(np.float32)
    u = (mh / d).astype(np.float32)
    total = ((s.lr * u).astype(np.float32) + (s.lw * pv).astype(np.float32)).astype(np.float32)
    yk = ((-total).astype(np.float32) - val(c)).astype(np.float32)
    t = (pv + yk).astype(np.float32)
    pn = torch_rne_bits(t)
    cn = torch_rne_bits(((val(pn) - pv).astype(np.float32) - yk).astype(np.float32))
    pp, mm, vv, cc = p.copy(), m.copy(), v.copy(), c.copy()
    ref.sr_adamw_step([dict(p=pp, g=g, m=mm, v=vv, aux=cc)], HYP, 3, 0, ref.FLAG_KAHAN)
    assert bool(np.all(pp == pn)) and bool(np.all(cc == cn))
    assert bool(np.all(mm == torch_rne_bits(m1))) and bool(np.all(vv == torch_rne_bits(v1)))


# ------------------------------------------------ variants of the arithmetic

def _alg1_exact_variant(p, g, m, v, hyper, t, eps_in_root):
    """Lines 5-10 in exact rational arithmetic (60-digit decimal root); eps outside the root
    (standard AdamW) or inside it (the form used in Appendix B)."""
    import decimal
    from fractions import Fraction
    decimal.getcontext().prec = 60
    b1, b2, lr, eps, wd = (Fraction(float(f32(hyper[k]))) for k in ("beta1", "beta2", "lr", "eps", "weight_decay"))
    P, G, M, V = (Fraction(float(x)) for x in (p, g, m, v))
    m1 = b1 * M + (1 - b1) * G
    v1 = b2 * V + (1 - b2) * G * G
    mhat = m1 / (1 - b1 ** t)
    vhat = v1 / (1 - b2 ** t)
    arg = vhat + eps if eps_in_root else vhat
    root = Fraction((decimal.Decimal(arg.numerator) / decimal.Decimal(arg.denominator)).sqrt())
    den = root if eps_in_root else root + eps
    return float(P - (lr * mhat / den + lr * wd * P))


@pytest.mark.parametrize("flags", [ref.FLAG_EPS_IN_ROOT, ref.FLAG_DIV_BIAS, ref.FLAG_EPS_IN_ROOT | ref.FLAG_DIV_BIAS])
def test_arithmetic_variants_against_exact_evaluation(flags):
    n = 16
    rng = np.random.default_rng(20)
    p = trunc_bits(rng.standard_normal(n) * 0.02)
    g = trunc_bits(rng.standard_normal(n) * 1e-5)          # small gradients: eps placement matters
    m = (rng.standard_normal(n) * 1e-5).astype(np.float32)
    v = (rng.random(n) * 1e-10).astype(np.float32)
    hyper = dict(HYP, eps=1e-6)
    for t in (1, 7):
        s = ref.adamw_scalars(step=t, **hyper)
        y, _, _ = ref.adamw_unrounded(p, g, m, v, s, flags=flags | ref.FLAG_FP32_MOMENTS)
        y_std, _, _ = ref.adamw_unrounded(p, g, m, v, s, flags=ref.FLAG_FP32_MOMENTS)
        inside = bool(flags & ref.FLAG_EPS_IN_ROOT)
        for i in range(n):
            want = _alg1_exact_variant(val(p)[i], val(g)[i], m[i], v[i], hyper, t, inside)
            upd = abs(float(val(p)[i]) - want)
            assert abs(float(y[i]) - want) <= 0.5 * float(np.spacing(f32(abs(want)))) + 16 * 2.0 ** -24 * upd
        if inside:
            # with gradients this small the two placements of eps give clearly different updates
            assert float(np.max(np.abs(y - y_std))) > 1e-5
        else:
            # dividing by 1 - beta^t instead of multiplying by its reciprocal: a few roundings apart
            assert bool(np.all(np.abs(y - y_std) <= 4 * np.spacing(np.abs(y_std)) + 1e-9))
            assert bool(np.any(y != y_std)) or t == 1


def test_eps_inside_root_step1_closed_form():
    # m = v = 0, step 1: the update is lr g / sqrt(g^2 + eps)
    n = 2048
    rng = np.random.default_rng(21)
    p = trunc_bits(rng.standard_normal(n) * 0.02)
    g = trunc_bits(rng.standard_normal(n) * 1e-4)
    z = np.zeros(n, np.uint16)
    hyper = dict(HYP, eps=1e-8, weight_decay=0.0)
    s = ref.adamw_scalars(step=1, **hyper)
    y, _, _ = ref.adamw_unrounded(p, g, z, z, s, flags=ref.FLAG_EPS_IN_ROOT)
    pv, gv = val(p).astype(np.float64), val(g).astype(np.float64)
    upd = float(f32(hyper["lr"])) * gv / np.sqrt(gv * gv + float(f32(1e-8)))
    want = pv - upd
    assert bool(np.all(np.abs(y - want) <= 0.5 * np.spacing(np.abs(want).astype(np.float32)) + 16 * 2.0 ** -24 * np.abs(upd)))
    assert float(np.median(np.abs(upd))) > 1e-3


def test_variants_flow_through_the_full_step():
    n = 1024
    rng = np.random.default_rng(22)
    p0 = trunc_bits(rng.standard_normal(n) * 0.02)
    g = trunc_bits(rng.standard_normal(n) * 1e-5)
    z = np.zeros(n, np.uint16)
    outs = {}
    for flags in (0, ref.FLAG_EPS_IN_ROOT, ref.FLAG_DIV_BIAS):
        pp, mm, vv = p0.copy(), z.copy(), z.copy()
        ref.sr_adamw_step([dict(p=pp, g=g, m=mm, v=vv)], dict(HYP, eps=1e-6), 3, 5, flags)
        s = ref.adamw_scalars(step=3, **dict(HYP, eps=1e-6))
        y, _, _ = ref.adamw_unrounded(p0, g, z, z, s, flags=flags)
        lo = (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
        assert bool(np.all((pp == lo) | (pp == lo + 1)))     # the step rounds this variant's y
        outs[flags] = pp
    assert bool(np.any(outs[0] != outs[ref.FLAG_EPS_IN_ROOT]))
