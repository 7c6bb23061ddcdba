"""Pins of the CPU oracle's RNG and stochastic rounding (CPU only).

Each test checks the oracle against something fixed outside it: the
published Philox known-answer vectors, Eq.(2)'s probabilities counted over
ALL 2^16 draws with the expected count known by construction of the input,
the exact identities E[Q_SR(x)] = x and E[r^2] = Delta^2 q(1-q) (Section 2.1
and the Lemma on the SR perturbation, Appendix B), the random-walk example of
Section 2.2, and the add-noise-then-truncate form of Section 3 written
independently in numpy.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f32_from_int_scaled(n: int, q: int) -> np.float32:
    """n * 2^q as float32; caller guarantees exact representability."""
    v = np.float32(np.ldexp(np.float64(n), q))
    assert Fraction(float(v)) == Fraction(n) * Fraction(2) ** q
    return v


def bits_of(x: np.float32) -> int:
    return int(np.array([x], np.float32).view(np.uint32)[0])


def bf16_value(bits16) -> np.ndarray:
    return ref.bf16_bits_to_f32(np.asarray(bits16, dtype=np.uint16)).astype(np.float64)


# ------------------------------------------------------------------ Philox

def test_philox_known_answer_vectors():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = ref.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_r16_counter_layout():
    # element i -> block i>>3, 16-bit slice i&7 of the four output words; the stream sits in
    # the top three bits of counter word 1, above the high part of the block index.
    seed, step, tid = 0x0123456789ABCDEF, 77, 5
    for i in [0, 1, 7, 8, 9, 1000003, (1 << 35) + 13, (1 << 40) + 6]:
        for stream in range(4):
            blk = i >> 3
            w = ref.philox4x32_10([blk & 0xFFFFFFFF, (stream << 29) | (blk >> 32), tid, step],
                                  [seed & 0xFFFFFFFF, seed >> 32])
            j = i & 7
            expect = (int(w[j >> 1]) >> (16 * (j & 1))) & 0xFFFF
            assert ref.r16(seed, step, tid, i, stream) == expect
    # eight consecutive elements use the 128 output bits exactly once each
    w = ref.philox4x32_10([5, 0, tid, step], [seed & 0xFFFFFFFF, seed >> 32])
    got = ref.r16_many(seed, step, tid, 40, 8, 0)
    packed = sum(int(g) << (16 * j) for j, g in enumerate(got))
    assert packed == sum(int(x) << (32 * j) for j, x in enumerate(w))


def test_r16_streams_steps_tensors_seeds_are_distinct():
    base = ref.r16_many(1, 1, 0, 0, 4096, 0)
    for other in [ref.r16_many(1, 1, 0, 0, 4096, 1), ref.r16_many(1, 1, 0, 0, 4096, 2),
                  ref.r16_many(1, 1, 0, 0, 4096, 3), ref.r16_many(1, 2, 0, 0, 4096, 0),
                  ref.r16_many(1, 1, 1, 0, 4096, 0), ref.r16_many(2, 1, 0, 0, 4096, 0),
                  ref.r16_many(1 + (1 << 32), 1, 0, 0, 4096, 0),
                  ref.r16_many(1, 1, 0, 1 << 35, 4096, 0)]:
        # two independent 16-bit sequences agree in about 4096/65536 places
        assert int((base == other).sum()) < 16


def test_r16_uniformity_chi_square():
    n = 1 << 24
    draws = ref.r16_many(12345, 3, 7, 0, n, 0)
    counts = np.bincount(draws, minlength=65536).astype(np.float64)
    expected = n / 65536.0
    chi2 = float(((counts - expected) ** 2 / expected).sum())
    dof = 65535.0
    # chi-square with 65535 dof: mean dof, sd sqrt(2 dof) ~ 362; accept 6 sd
    assert abs(chi2 - dof) < 6.0 * np.sqrt(2.0 * dof)
    # each bit is balanced
    for b in range(16):
        ones = int(((draws >> b) & 1).sum())
        assert abs(ones - n / 2) < 6.0 * np.sqrt(n / 4)


# ------------------------------------------------- exhaustive SR (Eq. (2))

# (n, q): lo = n * 2^q is a BF16 magnitude (n < 256 with n >= 128 for normal numbers, any
# n < 128 at q = -133 for BF16 subnormals), hi = (n + 1) * 2^q the next one.
GRID_NQ = [
    (128, -7), (129, -7), (200, -7), (255, -7),          # one binade around 1.0, both edges
    (128, -13), (173, -20), (255, 0), (128, 10),
    (128, -133), (255, -133),                            # smallest normal binade
    (0, -133), (1, -133), (64, -133), (127, -133),       # BF16 subnormal range, incl. across to normal
    (128, 120), (254, 120),                              # largest binade
]
GRID_K = [0, 1, 2, 255, 256, 32767, 32768, 32769, 65534, 65535, 12345, 54321]


@pytest.mark.parametrize("n,q", GRID_NQ)
def test_sr_exhaustive_counts_mean_and_second_moment(n, q):
    lo = Fraction(n) * Fraction(2) ** q
    hi = Fraction(n + 1) * Fraction(2) ** q
    unit = Fraction(2) ** (q - 16)                      # spacing of binary32 inside [lo, hi)
    for k in GRID_K:
        x = f32_from_int_scaled(n * 65536 + k, q - 16)   # x = lo + k/65536 (hi - lo), by construction
        for sign in (+1, -1):
            xs = np.float32(sign) * x
            out = ref.sr_round_all_draws(bits_of(xs))
            vals = bf16_value(out)
            mags = np.abs(vals)
            up = mags == float(hi)
            down = mags == float(lo)
            assert bool(np.all(up | down))                       # outputs are the two neighbours
            assert int(up.sum()) == k                             # P(away from zero) = k/65536
            if not (n == 0 and k == 0):
                assert bool(np.all(np.sign(vals[mags > 0]) == sign))
            assert bool(np.all((out >> 15) == (0 if sign > 0 else 1)))   # sign bit kept, also on zero
            # unbiasedness as an identity: sum over all draws = 65536 x
            total = Fraction(int(down.sum())) * lo + Fraction(int(up.sum())) * hi
            assert total == 65536 * (Fraction(float(x)))
            # second moment: mean of (out - x)^2 = Delta^2 q (1 - q), q = k/65536
            err_up = hi - Fraction(float(x))
            err_dn = lo - Fraction(float(x))
            second = (int(up.sum()) * err_up ** 2 + int(down.sum()) * err_dn ** 2) / 65536
            qq = Fraction(k, 65536)
            assert second == (hi - lo) ** 2 * qq * (1 - qq)
            assert err_up == (65536 - k) * unit and err_dn == -k * unit


def test_sr_threshold_is_r_plus_k_ge_65536():
    # the coupling of draw to outcome: away from zero exactly for the k largest draws
    x = f32_from_int_scaled(128 * 65536 + 1000, -7 - 16)
    out = ref.sr_round_all_draws(bits_of(x))
    up = bf16_value(out) > 1.0
    assert bool(np.all(up[65536 - 1000:])) and not bool(np.any(up[:65536 - 1000]))


def test_sr_overflow_to_infinity():
    flt_max = np.finfo(np.float32).max
    for sign in (1.0, -1.0):
        out = ref.sr_round_all_draws(bits_of(np.float32(sign * flt_max)))
        vals = bf16_value(out)
        assert int(np.isinf(vals).sum()) == 65535          # k = 65535 for +-FLT_MAX
        assert bool(np.all(np.sign(vals) == sign))
        largest_bf16 = float(Fraction(255) * Fraction(2) ** 120)
        assert bool(np.all((np.abs(vals) == largest_bf16) | np.isinf(vals)))


def test_sr_special_values():
    for bits, expect in [(0x00000000, 0x0000), (0x80000000, 0x8000),
                         (0x7F800000, 0x7F80), (0xFF800000, 0xFF80)]:
        out = ref.sr_round_all_draws(bits)
        assert bool(np.all(out == expect))
    # NaNs: quiet, sign and upper payload kept, for every draw
    for bits in [0x7FC00000, 0xFFC00000, 0x7F800001, 0xFF80FFFF, 0x7FFFFFFF, 0x7FA12345]:
        out = ref.sr_round_all_draws(bits)
        assert bool(np.all(out == ((bits >> 16) | 0x40)))
        assert bool(np.all(np.isnan(bf16_value(out))))


def test_sr_exact_bf16_values_never_move():
    rng = np.random.default_rng(1)
    hi16 = rng.integers(0, 1 << 16, size=4096, dtype=np.uint32)
    y = (hi16 << np.uint32(16)).view(np.float32)
    finite = np.isfinite(y)
    r = rng.integers(0, 1 << 16, size=4096, dtype=np.uint32)
    out = ref.sr_round_many(y, r)
    assert bool(np.all(out[finite] == hi16[finite].astype(np.uint16)))


def test_sr_matches_add_noise_then_truncate():
    """Section 3's dithering form -- add 16 uniform bits below the kept mantissa, drop the low
    half -- is the same function of (y, draw) as the interval definition, for all finite y."""
    rng = np.random.default_rng(2)
    n = 1 << 22
    ybits = rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32)
    # add structured cases: every exponent with extreme low halves
    exps = np.arange(0, 255, dtype=np.uint32)
    extra = []
    for lowhalf in (0x0000, 0x0001, 0x7FFF, 0x8000, 0xFFFF):
        for top in (0x00, 0x7F):
            extra.append((exps << np.uint32(23)) | np.uint32(top << 16) | np.uint32(lowhalf))
    ybits = np.concatenate([ybits] + extra + [ybits[:1024] | np.uint32(0x80000000)])
    y = ybits.view(np.float32)
    finite = np.isfinite(y)
    r = rng.integers(0, 1 << 16, size=y.size, dtype=np.uint32)
    r[:64] = 0
    r[64:128] = 65535
    out = ref.sr_round_many(y, r)
    trick = ((ybits.astype(np.uint64) + r.astype(np.uint64)) >> np.uint64(16)).astype(np.uint16)
    assert bool(np.all(out[finite] == trick[finite]))


# ---------------------------------------------- SR and RNG together (E[Q]=x)

def test_sr_unbiased_over_ten_thousand_seeds():
    # x at several positions inside BF16 cells of different binades and signs
    cases = [(128, -7, 1), (128, -7, 32768), (200, -7, 65535), (173, -20, 12345),
             (255, 3, 40000), (5, -133, 20000), (128, -133, 999), (129, -13, 3)]
    xs, ks, spacings = [], [], []
    for n, q, k in cases:
        for sign in (1, -1):
            xs.append(np.float32(sign) * f32_from_int_scaled(n * 65536 + k, q - 16))
            ks.append(k)
            spacings.append(2.0 ** q)
    xs = np.array(xs, dtype=np.float32)
    n_seeds = 10000
    acc = np.zeros(xs.size, dtype=np.float64)
    for seed in range(n_seeds):
        out = ref.sr_cast_f32_bf16(xs, seed=seed, step=1, tensor_id=0, nthreads=1)
        acc += bf16_value(out)
    mean = acc / n_seeds
    for i in range(xs.size):
        q = ks[i] / 65536.0
        bound = 5.0 * spacings[i] * np.sqrt(q * (1.0 - q) / n_seeds)
        assert abs(mean[i] - float(xs[i])) <= bound, (i, mean[i], xs[i], bound)
    # a biased rule would fail: the tested deviations are far inside one spacing
    assert max(5.0 * np.sqrt(0.25 / n_seeds), 0.0) < 0.03


# ------------------------------------------- worked example of Section 2.2

def _golden_fraction(name):
    for l in open(os.path.join(GOLDEN, "random_walk_example.txt")):
        if l.startswith(name):
            _, a, b = l.split()
            return Fraction(int(a), int(b))
    raise KeyError(name)


def test_random_walk_example_exact():
    """Level x0 = 1.0, next level 1 + 2^-7.  A half-spacing update reaches the next level for
    exactly half of all draws; within two such updates for 3/4 of all draw pairs; an update
    of k/65536 of a spacing succeeds for exactly k draws (the geometric tail)."""
    x0 = np.float32(1.0)
    spacing = 2.0 ** -7
    nxt = 1.0 + spacing
    first = bf16_value(ref.sr_round_all_draws(bits_of(np.float32(x0 + np.float32(spacing / 2)))))
    assert set(np.unique(first)) == {1.0, nxt}
    n_up1 = int((first == nxt).sum())
    assert Fraction(n_up1, 65536) == _golden_fraction("p_single_half_update")
    # second update from each of the two possible states (draws independent of the first)
    reached = 0
    for state, count in ((1.0, 65536 - n_up1), (nxt, n_up1)):
        second = bf16_value(ref.sr_round_all_draws(
            bits_of(np.float32(np.float32(state) + np.float32(spacing / 2)))))
        reached += count * int((second >= nxt).sum())
    assert Fraction(reached, 65536 * 65536) == _golden_fraction("p_within_two_updates")
    # tail: per-update success probability equals the update size in units of the spacing
    for k in (1, 17, 4096, 40000):
        eps_update = np.float32(k * spacing / 65536.0)
        res = bf16_value(ref.sr_round_all_draws(bits_of(np.float32(x0 + eps_update))))
        assert int((res == nxt).sum()) == k


def test_random_walk_example_with_the_counter_rng():
    # same example driven by r16(seed, ...): fraction reaching the next level within two
    # updates over 40000 independent walks is 3/4 within 5 sigma
    n = 40000
    spacing = np.float32(2.0 ** -7)
    x = np.ones(n, dtype=np.float32)
    for step in (1, 2):
        y = (x + spacing / np.float32(2)).astype(np.float32)
        x = bf16_value(ref.sr_cast_f32_bf16(y, seed=99, step=step, tensor_id=0)).astype(np.float32)
    frac = float((x >= 1.0 + 2.0 ** -7).mean())
    assert abs(frac - 0.75) < 5.0 * np.sqrt(0.75 * 0.25 / n)


# ---------------------------------------------------------- nearest rounding

def test_rne_round_matches_torch_bfloat16_cast():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    ybits = rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32)
    ties = (rng.integers(0, 1 << 16, size=4096, dtype=np.uint32) << np.uint32(16)) | np.uint32(0x8000)
    ybits = np.concatenate([ybits, ties])
    y = ybits.view(np.float32)
    keep = ~np.isnan(y)
    y = y[keep]
    want = torch.from_numpy(y.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([ref.rne_round(v) for v in y[:20000]], dtype=np.uint16)
    assert bool(np.all(got == want[:20000]))
    got_ties = np.array([ref.rne_round(v) for v in y[-2000:]], dtype=np.uint16)
    assert bool(np.all(got_ties == want[-2000:]))


def test_cast_workload_properties():
    """Config-1 cast input: outputs are one of the two BF16 neighbours, values already on the
    grid stay, subnormals are not flushed, and windows with an element offset equal slices."""
    torch = pytest.importorskip("torch")
    from paper_2502_20566_amd import workloads as W
    x = W.make_cast_input(1 << 16, "cpu", W.data_seed(1, 0)).numpy()
    out = ref.sr_cast_f32_bf16(x, seed=0, step=1, tensor_id=0)
    xb = x.view(np.uint32)
    lo = (xb >> np.uint32(16)).astype(np.uint16)
    assert bool(np.all((out == lo) | (out == lo + 1)))
    on_grid = (xb & np.uint32(0xFFFF)) == 0
    assert on_grid.sum() > 300 and bool(np.all(out[on_grid] == lo[on_grid]))
    sub = ((xb >> np.uint32(23)) & np.uint32(0xFF)) == 0
    assert sub.sum() > 300 and bool(np.any(out[sub] & 0x7FFF))
    win = ref.sr_cast_f32_bf16(x[1001:5003], seed=0, step=1, tensor_id=0, elem_offset=1001)
    assert bool(np.all(win == out[1001:5003]))
    other = ref.sr_cast_f32_bf16(x, seed=1, step=1, tensor_id=0)
    assert 0.2 < float((other != out).mean()) < 0.8
