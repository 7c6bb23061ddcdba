"""Pins of the oracle's update with the PARAMETER held in 8 bits (an extension: the conclusion of the
paper names FP8 as the next target of SR and gives no design; p is kept as E4M3 codes with a
power-of-two scale per tensor).  The decode and the update arithmetic are pinned to the BF16 path
(itself pinned to torch.optim.AdamW and to exact rationals) on parameter values both can hold, with
torch's float8 decoder supplying the values; the write-back to exact-rational thresholds on
neighbours found by search in torch's decoded grid, with the 32-bit draws read from the Philox
stream directly; the mean over seeds to Eq.(2)'s unbiasedness."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref

torch = pytest.importorskip("torch")

HYP = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
E4M3_VALUES = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
E5M2_VALUES = torch.arange(256, dtype=torch.uint8).view(torch.float8_e5m2).float().numpy().astype(np.float64)
FINITE = np.flatnonzero(np.isfinite(E4M3_VALUES))


def trunc_bits(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def state(n, seed, p_exp):
    rng = np.random.default_rng(seed)
    p8 = FINITE[rng.integers(0, FINITE.size, n)].astype(np.uint8)
    g = trunc_bits(rng.standard_normal(n) * 1e-3)
    m = trunc_bits(rng.standard_normal(n) * 1e-3)
    v = trunc_bits(rng.random(n) * 1e-6)
    return p8, g, m, v


@pytest.mark.parametrize("p_exp", [0, 13, -4, 40])
def test_decode_and_arithmetic_equal_the_bf16_path(p_exp):
    """Every E4M3 value times a power of two is a BF16 value: the same parameters held in BF16 give
    bit-identical unrounded results, and (same draws of streams 1 and 2) the same new moments."""
    n = 4000
    p8, g, m, v = state(n, 1, p_exp)
    p_bf = trunc_bits(E4M3_VALUES[p8] * 2.0 ** -p_exp)
    assert np.array_equal(ref.bf16_bits_to_f32(p_bf).astype(np.float64), E4M3_VALUES[p8] * 2.0 ** -p_exp)
    for t, flags in ((1, 0), (9, ref.FLAG_EPS_IN_ROOT), (200, ref.FLAG_DIV_BIAS)):
        s = ref.adamw_scalars(step=t, norm=2.0, max_norm=1.0, **HYP)
        m1, v1, m2, v2 = m.copy(), v.copy(), m.copy(), v.copy()
        ref.sr_adamw_tensor_fp8p(p8.copy(), g, m1, v1, 6, s, t, 77, p_exp, flags, elem_offset=24)
        ref.sr_adamw_tensor(p_bf.copy(), g, m2, v2, 6, s, t, 77, flags, elem_offset=24)
        assert np.array_equal(m1, m2) and np.array_equal(v1, v2)


def neighbours(a: Fraction):
    grid = sorted((Fraction(float(E4M3_VALUES[c])), c) for c in range(128) if np.isfinite(E4M3_VALUES[c]))
    lo = max(x for x in grid if x[0] <= a)
    above = [x for x in grid if x[0] > a]
    return lo, (min(above) if above else None)


@pytest.mark.parametrize("p_exp,lr", [(13, 3e-3), (13, 0.5), (-2, 3e-3), (9, 30.0)])
def test_write_back_is_eq2_with_the_20_bit_draw_of_stream_0(p_exp, lr):
    """y 2^p_exp between grid neighbours lo <= a < hi goes up exactly when the top 20 bits of the
    element's word of stream 0 plus floor(2^20 (a - lo)/(hi - lo)) reach 2^20; from 448 upwards it
    is stored as 448.  y comes from the BF16 path's unrounded result on the same values."""
    n, tid, step, seed, off = 3000, 11, 5, 0xABCDEF0123, 52
    hyp = dict(HYP, lr=lr)
    p8, g, m, v = state(n, 2, p_exp)
    s = ref.adamw_scalars(step=step, **hyp)
    y, _, _ = ref.adamw_unrounded(trunc_bits(E4M3_VALUES[p8] * 2.0 ** -p_exp), g, m, v, s)
    out = p8.copy()
    ref.sr_adamw_tensor_fp8p(out, g, m.copy(), v.copy(), tid, s, step, seed, p_exp, elem_offset=off)
    ups = sat = 0
    for i in range(n):
        ys = np.float32(y[i]) * np.float32(2.0 ** p_exp)              # the definition's binary32 product
        a = Fraction(float(ys))
        sign = 0x80 if (a < 0 or (a == 0 and np.signbit(ys))) else 0
        a = abs(a)
        if a >= 448:
            assert out[i] == sign | 0x7E
            sat += 1
            continue
        (lo, clo), hi = neighbours(a)
        assert hi is not None
        k = (a - lo) * (1 << 20) // (hi[0] - lo)
        r = ref.r32(seed, step, tid, off + i, 0) >> 12
        up = r + k >= (1 << 20)
        assert out[i] == sign | (hi[1] if up else clo), (i, float(a), r, int(k))
        ups += int(up)
    if lr < 0.01:
        assert ups > 100 and sat < n // 20                # only parameters that already sit at +-448 saturate
    if lr >= 30:
        assert sat > 100


def test_written_parameter_is_unbiased_over_seeds():
    """E[decode(p8')] 2^-p_exp = y for values inside the normal range: mean over 4000 seeds within
    five standard deviations of Eq.(2)'s two-point law."""
    n, p_exp = 48, 13
    p8, g, m, v = state(n, 3, p_exp)
    p8 = np.where((p8 & 0x7F) < 0x10, p8 | 0x20, p8).astype(np.uint8)       # keep clear of the subnormal range
    s = ref.adamw_scalars(step=3, **HYP)
    y, _, _ = ref.adamw_unrounded(trunc_bits(E4M3_VALUES[p8] * 2.0 ** -p_exp), g, m, v, s)
    seeds = 4000
    acc = np.zeros(n)
    lo = np.full(n, np.inf)
    hi = np.full(n, -np.inf)
    for sd in range(seeds):
        out = p8.copy()
        ref.sr_adamw_tensor_fp8p(out, g, m.copy(), v.copy(), 0, s, 3, sd, p_exp)
        val = E4M3_VALUES[out] * 2.0 ** -p_exp
        acc += val
        lo, hi = np.minimum(lo, val), np.maximum(hi, val)
    mean = acc / seeds
    delta = hi - lo
    assert (delta > 0).sum() > n // 2                                        # most elements sit between two grid values
    q = np.where(delta > 0, (y - lo) / np.where(delta > 0, delta, 1), 0.0)
    sigma = delta * np.sqrt(np.clip(q * (1 - q), 0, None) / seeds)
    assert np.all(np.abs(mean - y) <= 5 * sigma + 1e-12)


def test_fixed_points_range_rules_and_offsets():
    n, p_exp = 2048, 13
    p8, g, m, v = state(n, 4, p_exp)
    # no learning rate, no decay: every grid value stays where it is, whatever the draw
    s0 = ref.adamw_scalars(step=2, **dict(HYP, lr=0.0, weight_decay=0.0))
    for seed in (0, 1, 2):
        out = p8.copy()
        ref.sr_adamw_tensor_fp8p(out, g, m.copy(), v.copy(), 3, s0, 2, seed, p_exp)
        keep = (p8 & 0x7F) != 0                                               # -0 + 0 = +0 in y = p - 0
        assert np.array_equal(out[keep], p8[keep])
    # a NaN gradient gives the NaN code; a NaN code stays one
    s = ref.adamw_scalars(step=2, **HYP)
    g2 = g.copy(); g2[5] = 0x7FC0
    p2 = p8.copy(); p2[9] = 0x7F
    ref.sr_adamw_tensor_fp8p(p2, g2, m.copy(), v.copy(), 3, s, 2, 1, p_exp)
    assert p2[5] & 0x7F == 0x7F and p2[9] & 0x7F == 0x7F
    # a window with its element offset equals the slice of the whole tensor
    whole = p8.copy(); mw, vw = m.copy(), v.copy()
    ref.sr_adamw_tensor_fp8p(whole, g, mw, vw, 3, s, 2, 1, p_exp, elem_offset=8)
    part = p8[100:900].copy(); mp, vp = m[100:900].copy(), v[100:900].copy()
    ref.sr_adamw_tensor_fp8p(part, g[100:900].copy(), mp, vp, 3, s, 2, 1, p_exp, elem_offset=108)
    assert np.array_equal(part, whole[100:900]) and np.array_equal(mp, mw[100:900]) and np.array_equal(vp, vw[100:900])
    # the multi-tensor entry point routes on the flag and the dtypes
    t = dict(p=p8.copy(), g=g, m=m.copy(), v=v.copy(), p_exp=p_exp, tensor_id=3, elem_offset=8)
    ref.sr_adamw_step([t], HYP, 2, 1, ref.FLAG_FP8_PARAMS)
    assert np.array_equal(t["p"], whole) and np.array_equal(t["m"], mw)


def test_with_8_bit_moments_too_the_moment_write_back_is_the_fp8_moment_path():
    """All of the optimizer state in 8 bits: the moments must come out as ref_sr_adamw_tensor_fp8m
    writes them for the same parameter values held in BF16."""
    n, p_exp, m_exp, v_exp = 3000, 13, 12, 30
    rng = np.random.default_rng(8)
    p8, g, _, _ = state(n, 5, p_exp)
    fin5 = np.flatnonzero(np.isfinite(E5M2_VALUES) & (np.arange(256) < 128))
    m8 = FINITE[rng.integers(0, FINITE.size, n)].astype(np.uint8)
    v8 = fin5[rng.integers(0, fin5.size, n)].astype(np.uint8)
    gv = rng.standard_normal(n) * 2.0 ** -m_exp * 4
    gv[::50] = 4.0                                       # spikes: the scaled moments leave both formats' ranges
    g = trunc_bits(gv)
    s = ref.adamw_scalars(step=4, **HYP)
    ma, va, mb, vb = m8.copy(), v8.copy(), m8.copy(), v8.copy()
    pa = p8.copy()
    ref.sr_adamw_tensor_fp8p(pa, g, ma, va, 2, s, 4, 5, p_exp, 0, m_exp, v_exp, elem_offset=16)
    ref.sr_adamw_tensor_fp8m(trunc_bits(E4M3_VALUES[p8] * 2.0 ** -p_exp), g, mb, vb, 2, s, 4, 5, m_exp, v_exp, elem_offset=16)
    assert np.array_equal(ma, mb) and np.array_equal(va, vb)
    assert (va[::50] == 0x7B).all() and ((ma[::50] & 0x7F) == 0x7E).all()    # saturated, never infinite
    # and the parameter as with BF16 moments holding the same moment values
    pb = p8.copy()
    ref.sr_adamw_tensor_fp8p(pb, g, trunc_bits(E4M3_VALUES[m8] * 2.0 ** -m_exp), trunc_bits(E5M2_VALUES[v8] * 2.0 ** -v_exp),
                             2, s, 4, 5, p_exp, elem_offset=16)
    assert np.array_equal(pa, pb)
