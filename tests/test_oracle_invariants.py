"""Order and symmetry invariants of the oracle's stochastic roundings (Eq.(2), Section 2.1), for BF16
and for both 8-bit grids: with the draw fixed the rounding is a non-decreasing function of the value,
with the value fixed its magnitude is a non-decreasing function of the draw, it commutes with the
sign, and the result is always one of the two grid neighbours.  None of these is how the oracle
computes (frexp / floor / ldexp per value); an off-by-one in an exponent limit, a wrong comparison
direction or a sign handled on the wrong side of the rounding breaks at least one of them."""
import numpy as np
import pytest

from oracle import ref


def bf16_val(bits):
    return ref.bf16_bits_to_f32(np.asarray(bits, np.uint16)).astype(np.float64)


def samples(rng, n, lo_exp, hi_exp):
    mant = 1.0 + rng.random(n)
    e = rng.integers(lo_exp, hi_exp, n)
    return np.sort((np.ldexp(mant, e) * rng.choice([-1.0, 1.0], n)).astype(np.float32))


def test_bf16_rounding_is_monotone_in_the_value_and_commutes_with_the_sign():
    rng = np.random.default_rng(1)
    y = samples(rng, 20000, -140, 127)                    # binary32 subnormals up to the top binade
    for r in (0, 1, 12345, 32768, 65535):
        rr = np.full(y.size, r, np.uint32)
        q = ref.sr_round_many(y, rr)
        v = bf16_val(q)
        fin = np.isfinite(v)
        assert np.all(np.diff(v[fin]) >= 0)
        assert np.array_equal(ref.sr_round_many(-y, rr), q ^ np.uint16(0x8000))
        # one of the two neighbours: less than one BF16 spacing (2^-7 relative) away, or infinity
        # above the largest finite value; the subnormal range of BF16 has the fixed spacing 2^-133
        assert np.all(np.abs(v[fin] - y[fin]) < np.maximum(np.abs(y[fin].astype(np.float64)) * 2.0 ** -7, 2.0 ** -133))


def test_bf16_rounding_is_monotone_in_the_draw():
    rng = np.random.default_rng(2)
    y = samples(rng, 300, -140, 127)
    draws = np.sort(rng.integers(0, 65536, 64)).astype(np.uint32)
    for x in y:
        v = np.abs(bf16_val(ref.sr_round_many(np.full(draws.size, x, np.float32), draws)))
        v = np.where(np.isinf(v), 1e300, v)                        # infinity is the top of the order
        assert np.all(np.diff(v) >= 0) and np.unique(v).size <= 2


@pytest.mark.parametrize("fmt,lo_exp,hi_exp,maxfin,tiny", [(ref.E4M3, -14, 9, 448.0, 2.0 ** -9), (ref.E5M2, -22, 16, 57344.0, 2.0 ** -16)])
def test_fp8_rounding_is_monotone_and_commutes_with_the_sign(fmt, lo_exp, hi_exp, maxfin, tiny):
    rng = np.random.default_rng(3 + fmt)
    y = samples(rng, 4000, lo_exp, hi_exp)
    mb = 3 if fmt == ref.E4M3 else 2
    for r in (0, 1 << 12, 0x7FFFFFFF, 0x80000000, 0xFFFFF000, 0xFFFFFFFF):
        codes = np.array([ref.sr_round_fp8(x, r, fmt) for x in y])
        v = np.array([ref.fp8_decode(int(c), fmt) for c in codes])
        fin = np.isfinite(v)
        assert not np.isnan(v).any()
        assert np.all(np.diff(np.where(fin, v, np.sign(v) * 1e30)) >= 0)
        assert np.array_equal(np.array([ref.sr_round_fp8(-x, r, fmt) for x in y]), codes ^ 0x80)
        inside = fin & (np.abs(y) < maxfin)
        assert np.all(np.abs(v[inside] - y[inside]) < np.maximum(np.abs(y[inside].astype(np.float64)) * 2.0 ** -mb, tiny))
    draws = np.sort(rng.integers(0, 1 << 32, 48))
    for x in y[::40]:
        mags = np.array([ref.fp8_decode(ref.sr_round_fp8(x, int(r), fmt) & 0x7F, fmt) for r in draws])
        mags = np.where(np.isinf(mags), 1e30, mags)                # E5M2's infinity is the top of the order
        assert np.all(np.diff(mags) >= 0) and np.unique(mags).size <= 2


@pytest.mark.parametrize("flags", [0, ref.FLAG_RNE_MOMENTS, ref.FLAG_RNE_PARAMS | ref.FLAG_RNE_MOMENTS,
                                   ref.FLAG_EPS_IN_ROOT, ref.FLAG_DIV_BIAS])
def test_adamw_step_commutes_with_a_sign_flip_of_p_g_and_m(flags):
    """Algorithm 1 is odd in (x, g, m) for a fixed v: flipping their signs flips the new parameter and
    first moment and leaves the second moment alone, unrounded and -- the roundings being sign-symmetric
    for a given draw -- rounded as well.  A wrong sign on the weight-decay term, on the update direction
    or inside a rounding breaks it."""
    n = 4000
    rng = np.random.default_rng(9)
    bits = lambda x: (np.asarray(x, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    p, g, m = bits(rng.standard_normal(n) * 0.02), bits(rng.standard_normal(n) * 1e-3), bits(rng.standard_normal(n) * 1e-3)
    v = bits(rng.random(n) * 1e-6)
    hyper = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    flip = np.uint16(0x8000)
    for t in (1, 50):
        s = ref.adamw_scalars(step=t, norm=2.0, max_norm=1.0, **hyper)
        y, m1, v1 = ref.adamw_unrounded(p, g, m, v, s, flags)
        yn, m1n, v1n = ref.adamw_unrounded(p ^ flip, g ^ flip, m ^ flip, v, s, flags)
        assert np.array_equal(yn.view(np.uint32), y.view(np.uint32) ^ np.uint32(1 << 31))
        assert np.array_equal(m1n.view(np.uint32), m1.view(np.uint32) ^ np.uint32(1 << 31))
        assert np.array_equal(v1n.view(np.uint32), v1.view(np.uint32))
        a = dict(p=p.copy(), g=g, m=m.copy(), v=v.copy())
        b = dict(p=p ^ flip, g=g ^ flip, m=m ^ flip, v=v.copy())
        ref.sr_adamw_step([a], hyper, t, 77, flags, norm=2.0, max_norm=1.0)
        ref.sr_adamw_step([b], hyper, t, 77, flags, norm=2.0, max_norm=1.0)
        assert np.array_equal(b["p"], a["p"] ^ flip) and np.array_equal(b["m"], a["m"] ^ flip)
        assert np.array_equal(b["v"], a["v"])
        assert np.count_nonzero(a["p"] != p) > n // 10            # the step moved something
