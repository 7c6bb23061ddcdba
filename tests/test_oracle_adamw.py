"""Pins of the CPU oracle's AdamW step and gradient norm (CPU only).

Pinned against: the step-1 closed form of Algorithm 1 (m = v = 0 gives
Delta = lr g/(|g| + eps) + lr wd x), exact-rational evaluation of lines 5-10
from the same state, torch.optim.AdamW run on FP32 state (a library routine
with a different operation order), a brute-force SR written from Eq.(2) by
searching all 65536 BF16 values, exactly representable norms, and the
stagnation argument of Section 2.1.
"""
import decimal
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref

HYP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1)


def f32(x):
    return np.float32(x)


def to_bf16_bits_trunc(x: np.ndarray) -> np.ndarray:
    """Some BF16 bit patterns near x (truncation; only used to make test inputs)."""
    return (np.asarray(x, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def val(bits16):
    return ref.bf16_bits_to_f32(np.asarray(bits16, np.uint16))


def ulp32(x):
    x = np.abs(np.asarray(x, np.float64))
    e = np.floor(np.log2(np.maximum(x, 2.0 ** -126)))
    return 2.0 ** (e - 23)


def make_state(n, seed, p_std=0.02, g_std=1e-3):
    rng = np.random.default_rng(seed)
    p = to_bf16_bits_trunc(rng.standard_normal(n) * p_std)
    g = to_bf16_bits_trunc(rng.standard_normal(n) * g_std)
    return p, g


# ------------------------------------------------------------ host scalars

def test_scalars_closed_forms():
    s = ref.adamw_scalars(step=1, **HYP)
    b1, b2 = float(f32(0.9)), float(f32(0.999))
    assert s.omb1 == f32(1.0 - b1) and s.omb2 == f32(1.0 - b2)
    # t = 1: 1/(1 - beta^1) is the reciprocal of the same 1 - beta
    assert s.rbc1 == f32(1.0 / (1.0 - b1)) and s.rbc2 == f32(1.0 / (1.0 - b2))
    assert s.lw == f32(float(f32(1e-3)) * float(f32(0.1)))
    assert s.lr == f32(1e-3) and s.eps == f32(1e-8) and s.clip == 1.0
    # exact rational powers for t > 1 (float(Fraction) rounds correctly to double)
    for t in (2, 3, 10, 100, 101, 1000, 12345):
        s = ref.adamw_scalars(step=t, **HYP)
        for got, b in ((s.rbc1, b1), (s.rbc2, b2)):
            exact = 1 / (1 - Fraction(b) ** t)
            want = f32(float(exact))
            assert abs(float(got) - float(want)) <= float(np.spacing(want))
    s = ref.adamw_scalars(step=1000000, **HYP)
    assert s.rbc1 == 1.0 and s.rbc2 == 1.0


def test_clip_coefficient():
    s = ref.adamw_scalars(step=1, norm=5.0, max_norm=1.0, **HYP)
    assert s.clip == f32(1.0) / (f32(5.0) + f32(1e-6))
    s = ref.adamw_scalars(step=1, norm=0.5, max_norm=1.0, **HYP)
    assert s.clip == 1.0                                   # never scales up
    s = ref.adamw_scalars(step=1, norm=float("inf"), max_norm=1.0, **HYP)
    assert s.clip == 0.0
    s = ref.adamw_scalars(step=1, norm=float("nan"), max_norm=1.0, **HYP)
    assert np.isnan(s.clip)


def test_guard_against_a_nonfinite_norm():
    """FLAG_SKIP_NONFINITE_NORM: a NaN or infinite norm leaves the state as it is (whatever the
    other flags), a finite one gives exactly the unguarded step; without the guard a NaN norm
    poisons every output and an infinite one is a step with a zero gradient."""
    n = 1000
    for flags in (0, ref.FLAG_FP32_MOMENTS, ref.FLAG_RNE_MOMENTS):
        def state():
            p, g = make_state(n, 5)
            if flags & ref.FLAG_FP32_MOMENTS:
                m, v = np.full(n, 1e-3, np.float32), np.full(n, 1e-6, np.float32)
            else:
                m, v = to_bf16_bits_trunc(np.full(n, 1e-3)), to_bf16_bits_trunc(np.full(n, 1e-6))
            return dict(p=p, g=g, m=m, v=v)
        for norm in (float("nan"), float("inf"), float("-inf")):
            t, t0 = state(), state()
            ref.sr_adamw_step([t], HYP, 3, 1, flags | ref.FLAG_SKIP_NONFINITE_NORM, norm=norm, max_norm=1.0)
            assert all(np.array_equal(t[k].view(np.uint8), t0[k].view(np.uint8)) for k in "pmv")
        a, b = state(), state()
        ref.sr_adamw_step([a], HYP, 3, 1, flags | ref.FLAG_SKIP_NONFINITE_NORM, norm=2.5, max_norm=1.0)
        ref.sr_adamw_step([b], HYP, 3, 1, flags, norm=2.5, max_norm=1.0)
        assert all(np.array_equal(a[k].view(np.uint8), b[k].view(np.uint8)) for k in "pmv")
        assert not np.array_equal(a["p"], state()["p"])
        # unguarded: infinite norm = the same step with a zero gradient and no clipping
        c, d = state(), state()
        ref.sr_adamw_step([c], HYP, 3, 1, flags, norm=float("inf"), max_norm=1.0)
        d["g"] = np.zeros(n, np.uint16)
        ref.sr_adamw_step([d], HYP, 3, 1, flags)
        assert all(np.array_equal(c[k].view(np.uint8), d[k].view(np.uint8)) for k in "pmv")
        e = state()
        ref.sr_adamw_step([e], HYP, 3, 1, flags, norm=float("nan"), max_norm=1.0)
        assert np.all(np.isnan(val(e["p"])))


# ----------------------------------------------------- step-1 closed form

def test_step1_closed_form():
    n = 4096
    p, g = make_state(n, 0)
    z = np.zeros(n, np.uint16)
    s = ref.adamw_scalars(step=1, **HYP)
    y, m1, v1 = ref.adamw_unrounded(p, g, z, z, s)
    pv, gv = val(p).astype(np.float64), val(g).astype(np.float64)
    lr, eps, wd = float(f32(1e-3)), float(f32(1e-8)), float(f32(0.1))
    upd = lr * gv / (np.abs(gv) + eps)
    dec = lr * wd * pv
    want = pv - upd - dec
    tol = 0.5 * ulp32(want) + 8 * 2.0 ** -24 * (np.abs(upd) + np.abs(dec)) + 2.0 ** -149
    assert bool(np.all(np.abs(y.astype(np.float64) - want) <= tol))
    # the update is far larger than the tolerance, so a dropped term or a sign error fails
    assert float(np.median(np.abs(upd) / tol)) > 1e3
    # moments at step 1 from zero state
    assert bool(np.all(np.abs(m1 - (1 - float(f32(0.9))) * gv) <= ulp32(m1)))
    assert bool(np.all(np.abs(v1 - (1 - float(f32(0.999))) * gv * gv) <= ulp32(v1)))


def test_zero_gradient_and_zero_lr_special_cases():
    n = 1024
    p, _ = make_state(n, 1)
    z = np.zeros(n, np.uint16)
    s = ref.adamw_scalars(step=1, **HYP)
    y, m1, v1 = ref.adamw_unrounded(p, z, z, z, s)
    pv = val(p)
    # g = 0: update is 0/(0 + eps) = 0, so y = p - lw p in two single roundings
    assert bool(np.all(y == (pv - (s.lw * pv).astype(np.float32)).astype(np.float32)))
    assert bool(np.all(m1 == 0)) and bool(np.all(v1 == 0))
    # lr = 0 and wd = 0: y = p, already on the BF16 grid: every draw gives p back, bit for bit
    _, g = make_state(n, 2)
    h = dict(HYP, lr=0.0, weight_decay=0.0)
    for seed in (0, 1, 2):
        pp, mm, vv = p.copy(), z.copy(), z.copy()
        ref.sr_adamw_step([dict(p=pp, g=g, m=mm, v=vv)], h, step=1, seed=seed)
        assert bool(np.all(pp == p))


# ------------------------------------- exact evaluation of Algorithm 1, t > 1

def _alg1_exact(p, g, m, v, hyper, t, clip=1.0):
    """Lines 5-10 of Algorithm 1 in exact rational arithmetic (sqrt in 60-digit decimal),
    eps outside the root, from float inputs taken as exact rationals."""
    decimal.getcontext().prec = 60
    b1, b2 = Fraction(float(f32(hyper["beta1"]))), Fraction(float(f32(hyper["beta2"])))
    lr, eps, wd = (Fraction(float(f32(hyper[k]))) for k in ("lr", "eps", "weight_decay"))
    P, G, M, V = Fraction(float(p)), Fraction(float(g)) * Fraction(float(clip)), Fraction(float(m)), Fraction(float(v))
    m1 = b1 * M + (1 - b1) * G
    v1 = b2 * V + (1 - b2) * G * G
    mhat = m1 / (1 - b1 ** t)
    vhat = v1 / (1 - b2 ** t)
    root = decimal.Decimal(vhat.numerator) / decimal.Decimal(vhat.denominator)
    root = Fraction(root.sqrt())
    y = P - (lr * mhat / (root + eps) + lr * wd * P)
    return float(y), float(m1), float(v1)


@pytest.mark.parametrize("clip_norm", [None, 7.5])
def test_against_exact_rational_evaluation(clip_norm):
    n, T = 8, 3
    rng = np.random.default_rng(3)
    p = to_bf16_bits_trunc(rng.standard_normal(n) * 0.02)
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v = (rng.random(n) * 1e-6).astype(np.float32)
    hyper = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    for t in range(5, 5 + T):
        g = to_bf16_bits_trunc(rng.standard_normal(n) * 1e-3)
        s = ref.adamw_scalars(step=t, norm=clip_norm, max_norm=1.0, **hyper)
        y, m1, v1 = ref.adamw_unrounded(p, g, m, v, s, flags=ref.FLAG_FP32_MOMENTS)
        for i in range(n):
            ye, me, ve = _alg1_exact(val(p)[i], val(g)[i], m[i], v[i], hyper, t, clip=s.clip)
            assert abs(float(m1[i]) - me) <= 1.5 * ulp32(me)
            assert abs(float(v1[i]) - ve) <= 2.0 * ulp32(ve)
            upd = abs(float(val(p)[i]) - ye)
            assert abs(float(y[i]) - ye) <= 0.5 * ulp32(ye) + 12 * 2.0 ** -24 * upd
            assert upd > 1e3 * 12 * 2.0 ** -24 * upd
        # advance the state with the oracle's own step (FP32 moments: only p is rounded)
        ref.sr_adamw_step([dict(p=p, g=g, m=m, v=v)], hyper, step=t, seed=11,
                          flags=ref.FLAG_FP32_MOMENTS, norm=clip_norm, max_norm=1.0)
        assert bool(np.all(m == m1)) and bool(np.all(v == v1))


# ------------------------------------------- torch.optim.AdamW on FP32 state

def test_against_torch_adamw_fp32_moments():
    torch = pytest.importorskip("torch")
    n, T = 2048, 6
    rng = np.random.default_rng(4)
    p = to_bf16_bits_trunc(rng.standard_normal(n) * 0.02)
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32)
    hyper = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    tp = torch.nn.Parameter(torch.from_numpy(val(p).copy()))
    opt = torch.optim.AdamW([tp], lr=hyper["lr"], betas=(hyper["beta1"], hyper["beta2"]),
                            eps=hyper["eps"], weight_decay=hyper["weight_decay"], foreach=False)
    for t in range(1, T + 1):
        g = to_bf16_bits_trunc(rng.standard_normal(n) * 1e-3)
        s = ref.adamw_scalars(step=t, **hyper)
        m_prev, v_prev = m.astype(np.float64), v.astype(np.float64)
        y, m1, v1 = ref.adamw_unrounded(p, g, m, v, s, flags=ref.FLAG_FP32_MOMENTS)
        with torch.no_grad():
            tp.copy_(torch.from_numpy(val(p).copy()))       # same (rounded) parameter on both sides
        tp.grad = torch.from_numpy(val(g).copy())
        opt.step()
        st = opt.state[tp]
        assert int(st["step"]) == t
        # torch forms the moments by lerp, so the two roundings differ: bound the difference
        # relative to the operands (the sum can cancel), a few binary32 roundings wide
        gv = val(g).astype(np.float64)
        assert bool(np.all(np.abs(m1 - st["exp_avg"].numpy()) <= 4 * 2.0 ** -24 * (np.abs(m_prev) + np.abs(gv))))
        assert bool(np.all(np.abs(v1 - st["exp_avg_sq"].numpy()) <= 4 * 2.0 ** -24 * (np.abs(v_prev) + gv * gv)))
        ty = tp.detach().numpy().astype(np.float64)
        upd = np.abs(val(p).astype(np.float64) - ty)
        # torch decays first (p (1 - lr wd)) and then subtracts: roundings at the scale of p
        # on both sides, plus a few on the update; the update itself is ~1e6 times larger
        # (the moment sum can cancel, so its rounding is bounded through its operands)
        d = np.sqrt(v1.astype(np.float64) * float(s.rbc2)) + float(s.eps)
        scale = float(s.lr) * float(s.rbc1) * (np.abs(m_prev) + np.abs(gv)) / d
        bound = 2.5 * ulp32(val(p)) + 16 * 2.0 ** -24 * scale
        assert bool(np.all(np.abs(y - ty) <= bound))
        assert float(np.median(upd / bound)) > 1e4
        ref.sr_adamw_step([dict(p=p, g=g, m=m, v=v)], hyper, step=t, seed=5,
                          flags=ref.FLAG_FP32_MOMENTS)
        # both sides start the next step from the same moments (no drift accumulates)
        st["exp_avg"].copy_(torch.from_numpy(m))
        st["exp_avg_sq"].copy_(torch.from_numpy(v))


# ----------------------------------------------- brute force on tiny inputs

_ALL_BF16 = None


def _brute_force_sr(y: np.float32, r: int) -> int:
    """Eq.(2) by search: among all finite BF16 values find the neighbours of y, round away
    from zero iff r + 65536 (|y| - lo)/(hi - lo) >= 65536."""
    global _ALL_BF16
    if _ALL_BF16 is None:
        bits = np.arange(0, 0x7F80, dtype=np.uint16)          # non-negative finite BF16 values
        _ALL_BF16 = [(Fraction(float(x)), int(b)) for b, x in zip(bits, val(bits))]
    a = abs(Fraction(float(y)))
    sign = 0x8000 if np.signbit(y) else 0
    lo_i = max(i for i, (x, _) in enumerate(_ALL_BF16) if x <= a)
    lo, lo_bits = _ALL_BF16[lo_i]
    if lo_i + 1 < len(_ALL_BF16):
        hi, hi_bits = _ALL_BF16[lo_i + 1]
    else:
        hi, hi_bits = Fraction(2) ** 128, 0x7F80
    k = 65536 * (a - lo) / (hi - lo)
    assert k.denominator == 1
    return sign | (hi_bits if r + k >= 65536 else lo_bits)


def test_full_step_brute_force_tiny():
    n, T = 8, 3
    rng = np.random.default_rng(6)
    p = to_bf16_bits_trunc(rng.standard_normal(n) * 0.02)
    m = np.zeros(n, np.uint16)
    v = np.zeros(n, np.uint16)
    hyper = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    seed, tid = 0xABCDEF0123, 9
    for t in range(1, T + 1):
        g = to_bf16_bits_trunc(rng.standard_normal(n) * 1e-3)
        # independent evaluation: numpy float32 scalars, one IEEE operation per line
        s = ref.adamw_scalars(step=t, **hyper)
        want_p, want_m, want_v = [], [], []
        for i in range(n):
            P, G, M, V = (f32(val(a)[i]) for a in (p, g, m, v))
            b1, b2 = f32(hyper["beta1"]), f32(hyper["beta2"])
            omb1 = f32(1.0 - float(b1)); omb2 = f32(1.0 - float(b2))
            rbc1 = f32(float(1 / (1 - Fraction(float(b1)) ** t)))
            rbc2 = f32(float(1 / (1 - Fraction(float(b2)) ** t)))
            m1 = f32(f32(b1 * M) + f32(omb1 * G))
            v1 = f32(f32(b2 * V) + f32(omb2 * f32(G * G)))
            d = f32(np.sqrt(f32(v1 * rbc2)) + f32(hyper["eps"]))
            u = f32(f32(m1 * rbc1) / d)
            lw = f32(float(f32(hyper["lr"])) * float(f32(hyper["weight_decay"])))
            y = f32(P - f32(f32(f32(hyper["lr"]) * u) + f32(lw * P)))
            want_p.append(_brute_force_sr(y, ref.r16(seed, t, tid, i, 0)))
            want_m.append(_brute_force_sr(m1, ref.r16(seed, t, tid, i, 1)))
            want_v.append(_brute_force_sr(v1, ref.r16(seed, t, tid, i, 2)))
        ref.sr_adamw_step([dict(p=p, g=g, m=m, v=v, tensor_id=tid)], hyper, step=t, seed=seed)
        assert [int(x) for x in p] == want_p
        assert [int(x) for x in m] == want_m
        assert [int(x) for x in v] == want_v


def test_step_draw_distribution_of_one_element():
    # one element, many seeds: the rounded parameter takes the upper neighbour for a fraction
    # of seeds equal to the position of the unrounded value inside its BF16 cell
    p, g = make_state(1, 7)
    z = np.zeros(1, np.uint16)
    s = ref.adamw_scalars(step=1, **HYP)
    y, _, _ = ref.adamw_unrounded(p, g, z, z, s)
    k = int(y.view(np.uint32)[0] & 0xFFFF)
    lo = int(y.view(np.uint32)[0] >> 16)
    n_seeds = 20000
    ups = 0
    for seed in range(n_seeds):
        pp, mm, vv = p.copy(), z.copy(), z.copy()
        ref.sr_adamw_step([dict(p=pp, g=g, m=mm, v=vv)], HYP, step=1, seed=seed)
        assert int(pp[0]) in (lo, lo + 1)
        ups += int(pp[0]) == lo + 1
    q = k / 65536.0
    assert abs(ups / n_seeds - q) <= 5 * np.sqrt(q * (1 - q) / n_seeds) + 1e-12


# ------------------------------------------------ list / window independence

def test_list_split_and_windows_give_identical_bits():
    rng = np.random.default_rng(8)
    sizes = [1000, 8, 1, 4099, 64]
    hyper = dict(lr=6e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)

    def fresh():
        r = np.random.default_rng(9)
        ts = []
        for i, n in enumerate(sizes):
            ts.append(dict(p=to_bf16_bits_trunc(r.standard_normal(n) * 0.02),
                           g=to_bf16_bits_trunc(r.standard_normal(n) * 1e-4),
                           m=to_bf16_bits_trunc(r.standard_normal(n) * 1e-4),
                           v=to_bf16_bits_trunc(r.random(n) * 1e-8), tensor_id=i))
        return ts
    whole = fresh()
    ref.sr_adamw_step(whole, hyper, step=4, seed=3)
    # reversed order, two separate calls
    parts = fresh()
    ref.sr_adamw_step(parts[3:][::-1], hyper, step=4, seed=3)
    ref.sr_adamw_step(parts[:3], hyper, step=4, seed=3)
    for a, b in zip(whole, parts):
        for key in "pmv":
            assert bool(np.all(a[key] == b[key]))
    # a window of tensor 3 with its element offset equals the slice of the whole
    win = fresh()[3]
    lo, hi = 1003, 3001
    w = {k: win[k][lo:hi].copy() for k in "pgmv"}
    w.update(tensor_id=3, elem_offset=lo)
    ref.sr_adamw_step([w], hyper, step=4, seed=3)
    for key in "pmv":
        assert bool(np.all(w[key] == whole[3][key][lo:hi]))
    # thread count does not matter
    one = fresh()
    ref.sr_adamw_step(one, hyper, step=4, seed=3, nthreads=1)
    for a, b in zip(whole, one):
        assert bool(np.all(a["p"] == b["p"]))
    del rng


# ------------------------------------------------------------ gradient norm

def test_norm_exact_cases():
    rng = np.random.default_rng(10)
    ints = rng.integers(-3, 4, size=100000).astype(np.float32)      # small integers are BF16 values
    g = to_bf16_bits_trunc(ints)
    assert bool(np.all(val(g) == ints))
    S = int((ints.astype(np.int64) ** 2).sum())
    assert ref.grad_global_norm([g[:40000], g[40000:]]) == f32(np.sqrt(np.float64(S)))
    # all-equal inputs, N a perfect square: |a| sqrt(N) exactly
    a = f32(-0.0078125)
    g = to_bf16_bits_trunc(np.full(1 << 16, a, np.float32))
    assert ref.grad_global_norm([g]) == f32(abs(float(a)) * 256.0)
    # one large and many tiny terms: naive float32 accumulation would lose the tiny ones
    tiny = to_bf16_bits_trunc(np.full(1 << 20, 2.0 ** -10, np.float32))
    big = to_bf16_bits_trunc(np.array([4096.0], np.float32))
    assert ref.grad_global_norm([big, tiny]) == f32(np.sqrt(np.float64(2 ** 24 + 1)))
    assert ref.grad_global_norm([]) == 0.0
    assert ref.grad_global_norm([g[:0]]) == 0.0


def test_norm_against_exact_fraction_sum():
    import math
    rng = np.random.default_rng(12)
    x = rng.standard_normal(5000) * 1e-3
    x[::97] = rng.standard_normal(x[::97].size)             # outliers
    g = to_bf16_bits_trunc(x)
    S = sum(Fraction(float(t)) ** 2 for t in val(g))
    want = f32(math.sqrt(float(S)))                          # float(Fraction) is correctly rounded
    assert ref.grad_global_norm([g]) == want
    assert abs(float(want) - math.fsum(float(t) ** 2 for t in val(g)) ** 0.5) < 1e-6 * float(want)


# ----------------------------------------------- stagnation (Section 2.1)

def test_nearest_rounding_stagnates_and_sr_does_not():
    """Updates below half a BF16 spacing: nearest rounding returns the old parameter every
    time, SR moves it by the update in expectation."""
    n = 1 << 14
    p = to_bf16_bits_trunc(np.full(n, 1.0, np.float32))          # spacing 2^-7 above 1.0
    g = to_bf16_bits_trunc(np.full(n, 1e-4, np.float32))
    hyper = dict(lr=6e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0)
    s = ref.adamw_scalars(step=1, **hyper)
    z = np.zeros(n, np.uint16)
    y, _, _ = ref.adamw_unrounded(p, g, z, z, s)
    update = float(val(p)[0]) - float(y[0])
    assert 0 < update < 2.0 ** -9                                   # well below half a spacing
    assert all(ref.rne_round(v) == int(p[0]) for v in y[:16])       # Q(x + u) = x
    pp, mm, vv = p.copy(), z.copy(), z.copy()
    ref.sr_adamw_step([dict(p=pp, g=g, m=mm, v=vv)], hyper, step=1, seed=1)
    moved = float(val(p).astype(np.float64).mean() - val(pp).astype(np.float64).mean())
    spacing_below = 2.0 ** -8                                        # y < 1.0 lies in the binade below
    q = update / spacing_below
    assert abs(moved - update) <= 5 * spacing_below * np.sqrt(q * (1 - q) / n)
    # RNE moments variant: parameter still SR, moments deterministic
    pr, mr, vr = p.copy(), z.copy(), z.copy()
    ref.sr_adamw_step([dict(p=pr, g=g, m=mr, v=vr)], hyper, step=1, seed=1, flags=ref.FLAG_RNE_MOMENTS)
    assert bool(np.all(pr == pp)) and len(set(mr.tolist())) == 1 and len(set(vr.tolist())) == 1
