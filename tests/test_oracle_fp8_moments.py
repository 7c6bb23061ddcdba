"""Pins of the oracle's update with 8-bit moments (an extension: the paper's conclusion names FP8 as
the next target of SR; m is kept as E4M3 codes and v as E5M2 codes, each with a power-of-two scale).
The decode and the update arithmetic are pinned to the BF16-moment path (already pinned to
torch.optim.AdamW and to exact rationals) on moment values both formats can hold, with torch's float8
decoders supplying the values; the write-back to exact-rational thresholds on neighbours found by
search in torch's decoded grids, with the draws read from the Philox stream directly."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref

torch = pytest.importorskip("torch")

HYP = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
E4M3_VALUES = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy().astype(np.float64)
E5M2_VALUES = torch.arange(256, dtype=torch.uint8).view(torch.float8_e5m2).float().numpy().astype(np.float64)


def trunc_bits(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def finite_codes(rng, n, values, signed):
    ok = np.flatnonzero(np.isfinite(values) & ((np.arange(256) < 128) | signed))
    return ok[rng.integers(0, ok.size, n)].astype(np.uint8)


def state(n, seed, m_exp, v_exp):
    rng = np.random.default_rng(seed)
    p = trunc_bits(rng.standard_normal(n) * 0.02)
    g = trunc_bits(rng.standard_normal(n) * 2.0 ** -m_exp * 4)
    m8 = finite_codes(rng, n, E4M3_VALUES, True)
    v8 = finite_codes(rng, n, E5M2_VALUES, False)
    return p, g, m8, v8


@pytest.mark.parametrize("m_exp,v_exp", [(0, 0), (12, 30), (-3, 7), (16, 40)])
def test_decode_and_arithmetic_equal_the_bf16_moment_path(m_exp, v_exp):
    """Every E4M3 / E5M2 value times a power of two is a BF16 value: the same state held in BF16
    moments must give bit-identical unrounded results, and (same stream-0 draws) the same new
    parameter."""
    n = 5000
    p, g, m8, v8 = state(n, 1, m_exp, v_exp)
    m_bf = trunc_bits(E4M3_VALUES[m8] * 2.0 ** -m_exp)
    v_bf = trunc_bits(E5M2_VALUES[v8] * 2.0 ** -v_exp)
    assert np.array_equal(ref.bf16_bits_to_f32(m_bf).astype(np.float64), E4M3_VALUES[m8] * 2.0 ** -m_exp)
    assert np.array_equal(ref.bf16_bits_to_f32(v_bf).astype(np.float64), E5M2_VALUES[v8] * 2.0 ** -v_exp)
    for t, flags in ((1, 0), (7, ref.FLAG_EPS_IN_ROOT), (300, ref.FLAG_DIV_BIAS)):
        s = ref.adamw_scalars(step=t, norm=3.0, max_norm=1.0, **HYP)
        want = ref.adamw_unrounded(p, g, m_bf, v_bf, s, flags)
        got = ref.adamw_unrounded_fp8m(p, g, m8, v8, s, m_exp, v_exp, flags)
        for a, b in zip(got, want):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
        for pflag in (0, ref.FLAG_RNE_PARAMS):
            p1, p2 = p.copy(), p.copy()
            ref.sr_adamw_tensor_fp8m(p1, g, m8.copy(), v8.copy(), 5, s, t, 99, m_exp, v_exp, flags | pflag, elem_offset=16)
            ref.sr_adamw_tensor(p2, g, m_bf.copy(), v_bf.copy(), 5, s, t, 99, flags | pflag, elem_offset=16)
            assert np.array_equal(p1, p2)


def neighbours(a: Fraction, values, top):
    """lo <= a < hi among the finite non-negative grid values (with their codes); `top` is the value
    the code after the last finite one would have."""
    grid = sorted((Fraction(float(values[c])), c) for c in range(128) if np.isfinite(values[c]))
    lo = max(x for x in grid if x[0] <= a)
    above = [x for x in grid if x[0] > a]
    return lo, (min(above) if above else (Fraction(top), None))


@pytest.mark.parametrize("m_exp,v_exp", [(12, 30), (15, 36)])
def test_write_back_is_sr_with_the_16_bit_draws_of_streams_1_and_2(m_exp, v_exp):
    n, tid, step, seed, off = 3000, 9, 4, 0xFEEDFACE, 40
    p, g, m8, v8 = state(n, 2, m_exp, v_exp)
    s = ref.adamw_scalars(step=step, **HYP)
    _, m1, v1 = ref.adamw_unrounded_fp8m(p, g, m8, v8, s, m_exp, v_exp)
    mo, vo = m8.copy(), v8.copy()
    ref.sr_adamw_tensor_fp8m(p.copy(), g, mo, vo, tid, s, step, seed, m_exp, v_exp, elem_offset=off)
    moved = {0: 0, 1: 0}
    for which, (x1, e, out, values, top, inf_code, stream) in enumerate((
            (m1, m_exp, mo, E4M3_VALUES, 512, None, 1), (v1, v_exp, vo, E5M2_VALUES, 65536, 0x7C, 2))):
        r16 = ref.r16_many(seed, step, tid, off, n, stream)
        for i in range(n):
            a = Fraction(float(x1[i])) * Fraction(2) ** e
            sign = 0x80 if a < 0 else 0
            a = abs(a)
            assert a < Fraction(float(values[0x7E if which == 0 else 0x7B]))      # inside the finite range here
            (lo, clo), (hi, chi) = neighbours(a, values, top)
            k16 = (a - lo) * 65536 // (hi - lo)
            up = int(r16[i]) + k16 >= 65536
            want = (chi if chi is not None else inf_code) if up else clo
            assert out[i] == sign | want, (which, i, float(a), int(r16[i]), int(k16))
            moved[which] += int(up)
    assert moved[0] > 300 and moved[1] > 300


def test_written_moments_are_unbiased_over_seeds():
    n, m_exp, v_exp = 64, 12, 30
    p, g, m8, v8 = state(n, 3, m_exp, v_exp)
    s = ref.adamw_scalars(step=2, **HYP)
    _, m1, v1 = ref.adamw_unrounded_fp8m(p, g, m8, v8, s, m_exp, v_exp)
    seeds = 4000
    ms, vs = np.zeros(n), np.zeros(n)
    for seed in range(seeds):
        mo, vo = m8.copy(), v8.copy()
        ref.sr_adamw_tensor_fp8m(p.copy(), g, mo, vo, 0, s, 2, seed, m_exp, v_exp)
        ms += E4M3_VALUES[mo]
        vs += E5M2_VALUES[vo]
    ma, va = np.abs(m1.astype(np.float64)) * 2.0 ** m_exp, v1.astype(np.float64) * 2.0 ** v_exp
    cell_m = 2.0 ** (np.floor(np.log2(np.maximum(ma, 2.0 ** -6))) - 3)
    cell_v = 2.0 ** (np.floor(np.log2(np.maximum(va, 2.0 ** -14))) - 2)
    assert np.all(np.abs(ms / seeds - m1 * 2.0 ** m_exp) <= 5 * 0.5 * cell_m / np.sqrt(seeds) + cell_m * 2.0 ** -15)
    assert np.all(np.abs(vs / seeds - va) <= 5 * 0.5 * cell_v / np.sqrt(seeds) + cell_v * 2.0 ** -15)


def test_range_rules_and_nan():
    s = ref.adamw_scalars(step=1, **HYP)
    p = trunc_bits(np.full(4, 0.5))
    # g = 1.0 at step 1: m1 = 0.1 g = 0.1 (as float32 products), v1 = 0.05
    g = trunc_bits(np.array([1.0, -1.0, 1.0, np.nan]))
    m8, v8 = np.zeros(4, np.uint8), np.zeros(4, np.uint8)
    ref.sr_adamw_tensor_fp8m(p.copy(), g, m8, v8, 0, s, 1, 0, 13, 21)      # 0.1 * 2^13 = 819 > 448; 0.05 * 2^21 > 65536
    assert list(m8[:3]) == [0x7E, 0xFE, 0x7E]            # E4M3 saturates, sign kept
    assert list(v8[:3]) == [0x7B, 0x7B, 0x7B]            # and so does E5M2 here: 57344, not infinity
    assert m8[3] & 0x7F == 0x7F and v8[3] & 0x7F == 0x7F  # NaN gradient: NaN codes
    # an infinity that came in with v8 leaves as the largest finite value, a NaN code in m8 stays a NaN
    m8, v8 = np.array([0x7F, 0x08], np.uint8), np.array([0x10, 0x7C], np.uint8)
    pp = p[:2].copy()
    ref.sr_adamw_tensor_fp8m(pp, g[:2], m8, v8, 0, s, 1, 0, 0, 0)
    assert m8[0] & 0x7F == 0x7F and v8[1] == 0x7B
    # just below the top: 57344 stays, and a value between 57344 and 65536 goes to 57344 whatever the draw
    # (g = 2^8 at step 1: v1 = (1 - beta2) 2^16 = 3276.8 (as binary32 products); times 2^4 = 52428.8, times 2^5 > 65536)
    g2 = trunc_bits(np.full(64, 256.0))
    for v_exp, allowed in ((4, {0x7A, 0x7B}), (5, {0x7B})):
        codes = set()
        for seed in range(40):
            m8, v8 = np.zeros(64, np.uint8), np.zeros(64, np.uint8)
            ref.sr_adamw_tensor_fp8m(trunc_bits(np.full(64, 0.5)), g2, m8, v8, 0, s, 1, seed, 0, v_exp)
            codes |= set(v8.tolist())
        assert codes == allowed


def test_slices_with_element_offsets_reproduce_the_whole():
    n, m_exp, v_exp = 1000, 12, 30
    p, g, m8, v8 = state(n, 4, m_exp, v_exp)
    s = ref.adamw_scalars(step=3, **HYP)
    whole = [p.copy(), m8.copy(), v8.copy()]
    ref.sr_adamw_tensor_fp8m(whole[0], g, whole[1], whole[2], 2, s, 3, 11, m_exp, v_exp, elem_offset=5)
    for a, b in ((0, 333), (333, 1000)):
        part = [p[a:b].copy(), m8[a:b].copy(), v8[a:b].copy()]
        ref.sr_adamw_tensor_fp8m(part[0], g[a:b].copy(), part[1], part[2], 2, s, 3, 11, m_exp, v_exp, elem_offset=5 + a)
        for x, y in zip(part, whole):
            assert np.array_equal(x, y[a:b])


def test_constant_gradient_drives_the_moments_to_g_and_g_squared():
    """m -> g and v -> g^2 in the mean, through 8-bit storage (the EMA's fixed point)."""
    n, g0, m_exp, v_exp = 2000, 3e-4, 14, 33
    p = trunc_bits(np.zeros(n))
    g = trunc_bits(np.full(n, g0))
    gv = float(ref.bf16_bits_to_f32(g)[0])
    m8, v8 = np.zeros(n, np.uint8), np.zeros(n, np.uint8)
    for t in range(1, 201):
        s = ref.adamw_scalars(step=t, **HYP)
        ref.sr_adamw_tensor_fp8m(p, g, m8, v8, 0, s, t, 5, m_exp, v_exp)
    m = E4M3_VALUES[m8] * 2.0 ** -m_exp
    v = E5M2_VALUES[v8] * 2.0 ** -v_exp
    assert abs(m.mean() / gv - 1) < 0.01 and abs(v.mean() / gv ** 2 - 1) < 0.02
