"""Pins of the oracle's stochastic rounding to the two OCP 8-bit formats (an extension: the paper's
conclusion names FP8 as the next target and specifies nothing; Eq.(2) of Section 2.1 is applied to
those grids).  The grids are pinned to torch's float8 decoders, the rounding law to exact rational
arithmetic on neighbours found by brute force in the decoded table, the nearest-rounding special
case to torch's own conversion, the random-word layout to the Philox block function."""
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ref

FMTS = {ref.E4M3: (torch.float8_e4m3fn, 448.0), ref.E5M2: (torch.float8_e5m2, 57344.0)}
TWO32 = 1 << 32
DRAW_BITS = {ref.E4M3: 20, ref.E5M2: 21}          # binary32's 23 fraction bits minus the format's 3 / 2
MIN_NORMAL = {ref.E4M3: Fraction(1, 1 << 6), ref.E5M2: Fraction(1, 1 << 14)}


def word(draw, fmt, low_ones=False):
    """A 32-bit random word whose top D bits are `draw`; the bits below are not part of the draw."""
    low = 32 - DRAW_BITS[fmt]
    return (draw << low) | (((1 << low) - 1) if low_ones else 0)


def table(fmt):
    """Sorted finite non-negative grid values with their codes, from the oracle's decoder."""
    vals = [(ref.fp8_decode(c, fmt), c) for c in range(128)]
    return sorted((v, c) for v, c in vals if np.isfinite(v))


@pytest.mark.parametrize("fmt", [ref.E4M3, ref.E5M2])
def test_decode_equals_torch_float8(fmt):
    dt, _ = FMTS[fmt]
    want = torch.arange(256, dtype=torch.uint8).view(dt).float().numpy()
    got = np.array([ref.fp8_decode(c, fmt) for c in range(256)], dtype=np.float64)
    assert np.array_equal(np.isnan(want), np.isnan(got))
    ok = ~np.isnan(want)
    assert np.array_equal(want[ok].astype(np.float64), got[ok])
    assert np.array_equal(np.signbit(want[ok]), np.signbit(got[ok]))


@pytest.mark.parametrize("fmt", [ref.E4M3, ref.E5M2])
def test_grid_values_never_move(fmt):
    for c in range(256):
        v = ref.fp8_decode(c, fmt)
        if not np.isfinite(v):
            continue
        for r in (0, 1, 1 << 31, TWO32 - 1):
            assert ref.sr_round_fp8(v, r, fmt) == c, (c, r)


def neighbours(a: Fraction, fmt):
    """lo <= a < hi among the grid magnitudes, by linear search; hi of the last cell is the value the
    next code would have (2^9 = 512 does not exist in E4M3, 2^16 is E5M2's infinity)."""
    t = table(fmt)
    lo = max((Fraction(v), c) for v, c in t if Fraction(v) <= a)
    above = [(Fraction(v), c) for v, c in t if Fraction(v) > a]
    return lo, (min(above) if above else None)


@pytest.mark.parametrize("fmt", [ref.E4M3, ref.E5M2])
def test_rounding_law_is_exact_at_the_threshold_draw(fmt):
    """For y in a cell [lo, hi): k = floor(2^D (|y|-lo)/(hi-lo)) with D draw bits (the top D bits of
    the word); draw 2^D-k-1 keeps lo, draw 2^D-k gives hi, whatever the word's lower bits hold.  At or
    above the smallest normal the fraction has at most D bits (the probability is Eq.(2)'s exactly);
    below it the fraction is truncated.  Values span the subnormal range, binade edges, the top cell."""
    _, maxfin = FMTS[fmt]
    D = DRAW_BITS[fmt]
    rng = np.random.default_rng(8 + fmt)
    tiny = 2.0 ** (-9 if fmt == ref.E4M3 else -16)
    ys = np.concatenate([
        rng.uniform(-maxfin, maxfin, 300), rng.normal(0, 1, 300), rng.normal(0, 8 * tiny, 300),
        rng.normal(0, tiny / 64, 100),
        np.array([v * s for v, _ in table(fmt)[1:] for s in (1 - 2.0 ** -24, 1 + 2.0 ** -23)]),
    ]).astype(np.float32)
    ys = ys[np.abs(ys) < maxfin]
    checked_up = checked_dn = exact = truncated = 0
    for y in ys:
        a = Fraction(float(abs(y)))
        (lo, clo), hi = neighbours(a, fmt)
        sign = 0x80 if np.signbit(y) else 0
        assert hi is not None
        k = (a - lo) * (1 << D) // (hi[0] - lo)
        assert 0 <= k < (1 << D)
        if k > 0:
            assert ref.sr_round_fp8(y, word((1 << D) - k, fmt), fmt) == sign | hi[1]
            assert ref.sr_round_fp8(y, word((1 << D) - k, fmt, True), fmt) == sign | hi[1]
            checked_up += 1
        assert ref.sr_round_fp8(y, word((1 << D) - k - 1, fmt, True), fmt) == sign | clo
        assert ref.sr_round_fp8(y, word((1 << D) - k - 1, fmt), fmt) == sign | clo
        assert ref.sr_round_fp8(y, 0, fmt) == sign | clo
        checked_dn += 1
        rem = (a - lo) * (1 << D) % (hi[0] - lo)
        if a >= MIN_NORMAL[fmt]:                               # probability exact: E[Q(y)] = y
            assert rem == 0 and lo + (hi[0] - lo) * Fraction(k, 1 << D) == a
            exact += 1
        elif rem != 0:                                         # truncated: short by less than 2^-D of a cell
            assert 0 < a - (lo + (hi[0] - lo) * Fraction(k, 1 << D)) < (hi[0] - lo) * Fraction(1, 1 << D)
            truncated += 1
    assert checked_up > 1000 and checked_dn > 1000 and exact > 800 and truncated > 50


def test_top_cell_and_out_of_range():
    # E5M2: above 57344 the upper neighbour is 2^16, emitted as infinity
    y = np.float32(60000.0)
    k = (Fraction(60000) - 57344) * (1 << 21) // (65536 - 57344)
    assert ref.sr_round_fp8(y, word((1 << 21) - k, ref.E5M2), ref.E5M2) == 0x7C
    assert ref.sr_round_fp8(y, word((1 << 21) - k - 1, ref.E5M2, True), ref.E5M2) == 0x7B
    assert ref.sr_round_fp8(-y, word((1 << 21) - k, ref.E5M2), ref.E5M2) == 0xFC
    assert ref.sr_round_fp8(np.float32(1e30), 0, ref.E5M2) == 0x7C          # beyond 2^16: infinity
    assert ref.sr_round_fp8(np.float32(np.inf), 0, ref.E5M2) == 0x7C
    assert ref.sr_round_fp8(np.float32(-np.inf), 7, ref.E5M2) == 0xFC
    # E4M3 saturates: no infinity in the format
    for y, r in ((448.0, TWO32 - 1), (449.0, 0), (460.0, TWO32 - 1), (511.9, TWO32 - 1), (1e30, 5), (np.inf, 9)):
        assert ref.sr_round_fp8(np.float32(y), r, ref.E4M3) == 0x7E
        assert ref.sr_round_fp8(np.float32(-y), r, ref.E4M3) == 0xFE
    # the cell below the top is an ordinary cell
    assert ref.sr_round_fp8(np.float32(447.0), TWO32 - 1, ref.E4M3) == 0x7E
    assert ref.sr_round_fp8(np.float32(447.0), 0, ref.E4M3) == 0x7D
    for fmt in (ref.E4M3, ref.E5M2):
        assert ref.sr_round_fp8(np.float32(np.nan), 3, fmt) & 0x7F == 0x7F
        assert ref.sr_round_fp8(np.float32(0.0), TWO32 - 1, fmt) == 0x00
        assert ref.sr_round_fp8(np.float32(-0.0), TWO32 - 1, fmt) == 0x80


@pytest.mark.parametrize("fmt", [ref.E4M3, ref.E5M2])
def test_half_draw_is_round_to_nearest_like_torch(fmt):
    """With r = 2^31 the magnitude goes up iff the fraction is >= 1/2: round to nearest, ties away.
    Off the ties this is the conversion torch does (nearest, ties to even)."""
    dt, maxfin = FMTS[fmt]
    rng = np.random.default_rng(21 + fmt)
    tiny = 2.0 ** (-9 if fmt == ref.E4M3 else -16)
    y = np.concatenate([rng.uniform(-0.9 * maxfin, 0.9 * maxfin, 4000), rng.normal(0, 1, 4000),
                        rng.normal(0, 16 * tiny, 4000)]).astype(np.float32)
    want = torch.from_numpy(y).to(dt).view(torch.uint8).numpy()
    got = np.array([ref.sr_round_fp8(v, 1 << 31, fmt) for v in y], dtype=np.uint8)
    t = [Fraction(v) for v, _ in table(fmt)]
    mids = {(a + b) / 2 for a, b in zip(t, t[1:])}
    tie = np.array([Fraction(float(abs(v))) in mids for v in y])
    zero = (want & 0x7F) == 0                                # -0 vs +0 of a vanishing value: compare magnitudes
    assert np.array_equal(got[~tie & ~zero], want[~tie & ~zero])
    assert np.array_equal(got[zero] & 0x7F, want[zero] & 0x7F)
    assert tie.sum() < 10


@pytest.mark.parametrize("fmt", [ref.E4M3, ref.E5M2])
def test_mean_over_stratified_draws_is_the_input(fmt):
    rng = np.random.default_rng(3 + fmt)
    draws = (np.arange(1 << 12, dtype=np.uint64) << np.uint64(20)) + np.uint64(1 << 19)
    for y in rng.normal(0, 1, 12).astype(np.float32):
        codes = [ref.sr_round_fp8(y, int(r), fmt) for r in draws]
        vals = np.array([ref.fp8_decode(c, fmt) for c in codes])
        cell = np.ptp(vals) if np.ptp(vals) > 0 else 1.0
        assert abs(vals.mean() - float(y)) <= cell * 2.0 ** -12


def test_random_word_layout_and_cast():
    seed, step, tid = 0x0123456789ABCDEF, 77, 5
    for i in (0, 1, 2, 3, 4, 7, (1 << 34) + 5, (1 << 40) + 2):
        blk = i >> 2
        w = ref.philox4x32_10([blk & 0xFFFFFFFF, (5 << 29) | (blk >> 32), tid, step],
                              [seed & 0xFFFFFFFF, seed >> 32])
        assert ref.r32(seed, step, tid, i, 5) == int(w[i & 3])
    rng = np.random.default_rng(0)
    src = rng.normal(0, 2, 1003).astype(np.float32)
    for fmt in (ref.E4M3, ref.E5M2):
        for off in (0, 6, (1 << 33) + 1):
            got = ref.sr_cast_f32_fp8(src, fmt, seed, step, tid, elem_offset=off, nthreads=2)
            want = [ref.sr_round_fp8(v, ref.r32(seed, step, tid, off + i, 5), fmt) for i, v in enumerate(src)]
            assert np.array_equal(got, np.array(want, dtype=np.uint8))
