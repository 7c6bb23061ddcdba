"""GPU parity of sr_cast_f32_fp8 (extension: Eq.(2) of Section 2.1 on the OCP 8-bit grids) against the
CPU oracle, bit for bit, through the C ABI.  The kernel works on encodings (the chip's conversion
instruction for waves that hold nothing near the top of the format's range, else a split of the
significand and the carry of an add); the oracle on values (frexp/floor/ldexp and a search of the
decoded grid): they share nothing but the published formats and the Philox layout."""
import os

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2502_20566_amd import binding as B
from paper_2502_20566_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"
FMTS = [(B.SR_FP8_E4M3, ref.E4M3), (B.SR_FP8_E5M2, ref.E5M2)]


def gpu_cast(x: torch.Tensor, fmt, seed, step, tid) -> np.ndarray:
    out = torch.empty(x.numel(), dtype=torch.uint8, device=DEV)
    B.sr_cast_f32_fp8(x, out, fmt, seed, step, tid)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def from_bits(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.astype(np.uint32).view(np.int32)).to(DEV).view(torch.float32)


@pytest.mark.parametrize("gfmt,ofmt", FMTS)
def test_fp8_cast_value_mix_bit_exact(gfmt, ofmt):
    n = (1 << 20) + 3
    gen = torch.Generator(device=DEV).manual_seed(W.data_seed(1, 40 + gfmt))
    scale = torch.tensor([1.0, 1e-3, 60.0, 2.0 ** -8, 2.0 ** -15, 3e4, 1e-7, 500.0], device=DEV)
    x = torch.randn(n, device=DEV, generator=gen) * scale[torch.arange(n, device=DEV) % 8]
    for seed, step, tid in ((0, 1, 0), (0xDEADBEEFCAFE, 4000000000, 77)):
        got = gpu_cast(x, gfmt, seed, step, tid)
        want = ref.sr_cast_f32_fp8(x.cpu().numpy(), ofmt, seed, step, tid)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (bad[:5], got[bad[:5]], want[bad[:5]], x.cpu().numpy()[bad[:5]])
    other = gpu_cast(x, gfmt, 1, 1, 0)
    assert 0.1 < float((other != gpu_cast(x, gfmt, 0, 1, 0)).mean()) < 0.6      # a different seed draws differently


@pytest.mark.parametrize("gfmt,ofmt", FMTS)
def test_fp8_cast_every_grid_value_and_special_encodings(gfmt, ofmt):
    grid = np.array([ref.fp8_decode(c, ofmt) for c in range(256)], dtype=np.float32)
    finite = grid[np.isfinite(grid)]
    specials = np.array([0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00000, 0xFFC00000, 0x7F800001,
                         0xFFFFFFFF, 0x7F7FFFFF, 0xFF7FFFFF, 0x00000001, 0x807FFFFF, 0x00800000,
                         0x43E00000, 0x43DFFFFF, 0x43E00001, 0x43F00000, 0x477FE000, 0x47600000, 0x47600001,
                         0x477FFFFF, 0x47800000, 0x3C000000, 0x3BFFFFFF, 0x38800000, 0x387FFFFF, 0x37800000,
                         0x3A800000, 0x3A7FFFFF, 0x2F800000, 0x1F800000], dtype=np.uint32)
    vals = np.concatenate([finite, np.nextafter(finite, np.float32(np.inf)), np.nextafter(finite, np.float32(-np.inf)),
                           specials.view(np.float32)])
    bits = np.tile(vals.view(np.uint32), 64)
    x = from_bits(bits)
    for seed in (0, 5):
        got = gpu_cast(x, gfmt, seed, 2, 1)
        want = ref.sr_cast_f32_fp8(bits.view(np.float32), ofmt, seed, 2, 1)
        bad = np.flatnonzero(got != want)
        assert bad.size == 0, (hex(int(bits[bad[0]])), got[bad[0]], want[bad[0]])
    # grid values are fixed points whatever the draw
    m = finite.size
    assert np.array_equal(got[:m], np.array([c for c in range(256) if np.isfinite(grid[c])], dtype=np.uint8))


@pytest.mark.parametrize("gfmt,ofmt", FMTS)
@pytest.mark.parametrize("n", [1, 3, 4, 5, 255, 256, 257, 1021, 4 * 64 * 5 + 2])
def test_fp8_cast_ragged_sizes_and_views(gfmt, ofmt, n):
    base = torch.randn(n + 8, device=DEV, generator=torch.Generator(device=DEV).manual_seed(n)) * 3.0
    for off in (0, 1, 3):
        x = base[off:off + n]
        out_base = torch.zeros(n + 16, dtype=torch.uint8, device=DEV)
        for ooff in (0, 1, 2):
            out_base.zero_()
            dst = out_base[ooff:ooff + n]
            B.sr_cast_f32_fp8(x, dst, gfmt, 9, 3, 2)
            torch.cuda.synchronize()
            want = ref.sr_cast_f32_fp8(x.cpu().numpy(), ofmt, 9, 3, 2)
            whole = out_base.cpu().numpy()
            assert np.array_equal(whole[ooff:ooff + n], want)
            assert not whole[:ooff].any() and not whole[ooff + n:].any()


@pytest.mark.parametrize("gfmt,ofmt", FMTS)
def test_fp8_cast_strided_sweep_of_all_encodings(gfmt, ofmt):
    """Every 61st binary32 encoding (7.0e7 values over the whole range, both signs, NaNs and
    subnormals included) and every encoding of two narrow bands: around the smallest normal of
    the format and around its largest finite value."""
    sweep = np.arange(0, 1 << 32, 61, dtype=np.uint64).astype(np.uint32)
    lo_band = np.float32(2.0 ** (-6 if ofmt == ref.E4M3 else -14)).view(np.uint32)
    hi_band = np.float32(448.0 if ofmt == ref.E4M3 else 57344.0).view(np.uint32)
    bands = [np.arange(int(c) - (1 << 18), int(c) + (1 << 18), dtype=np.uint64).astype(np.uint32)
             for c in (lo_band, hi_band)]
    bits = np.concatenate([sweep] + bands)
    got = gpu_cast(from_bits(bits), gfmt, 3, 8, 6)
    want = ref.sr_cast_f32_fp8(bits.view(np.float32), ofmt, 3, 8, 6)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, (hex(int(bits[bad[0]])), got[bad[0]], want[bad[0]])


@pytest.mark.parametrize("gfmt,ofmt", FMTS)
def test_fp8_cast_wave_with_a_value_near_the_top_of_the_range(gfmt, ofmt):
    """A wave takes the integer path as a whole when one of its 256 values lies in the format's top
    binade or above, is infinite or a NaN.  Plant one such value in every wave of a sweep over all
    exponents (every 251st encoding and the band around the smallest normal), so that the integer
    path meets subnormal results, binade edges and zeros too, and must agree with the oracle there
    as the conversion instruction does in the other tests."""
    sweep = np.arange(0, 1 << 32, 251, dtype=np.uint64).astype(np.uint32)
    c = int(np.float32(2.0 ** (-6 if ofmt == ref.E4M3 else -14)).view(np.uint32))
    band = np.arange(c - (1 << 18), c + (1 << 18), dtype=np.uint64).astype(np.uint32)
    bits = np.concatenate([sweep, band])
    top = np.array([300.0, -447.0, np.inf, np.nan] if ofmt == ref.E4M3 else [40000.0, -57000.0, -np.inf, np.nan],
                   dtype=np.float32).view(np.uint32)
    where = np.arange(7, bits.size, 256)
    bits[where] = top[np.arange(where.size) % 4]
    got = gpu_cast(from_bits(bits), gfmt, 12, 9, 4)
    want = ref.sr_cast_f32_fp8(bits.view(np.float32), ofmt, 12, 9, 4)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, (hex(int(bits[bad[0]])), got[bad[0]], want[bad[0]])


STRIDE = int(os.environ.get("SR_TEST_FP8_STRIDE", "5"))       # 1 = every encoding (three minutes of oracle time)


@pytest.mark.parametrize("gfmt,ofmt", FMTS)
def test_fp8_cast_sweep_of_all_encodings_through_both_paths(gfmt, ofmt):
    """Every STRIDE-th of the 2^32 binary32 encodings (an odd stride meets every pattern of the low
    bits), in 32 pieces, converted twice: by the library as it runs (waves of neighbouring
    encodings share an exponent, so all below the format's top binade take the chip's conversion
    instruction and all above it the integer path) and with the test switch that sends every wave
    down the integer path.  The by-value oracle is computed once per piece and both must equal it:
    the instruction and the integer path are two implementations of the rule the oracle defines."""
    piece = 1 << 27
    try:
        for c in range(32):
            bits = torch.arange(c * piece, (c + 1) * piece, STRIDE, dtype=torch.int64, device=DEV).to(torch.int32)
            x = bits.view(torch.float32)
            want = ref.sr_cast_f32_fp8(x.cpu().numpy(), ofmt, 0xABCDEF, 5 + c, 2)
            for integer_path in (0, 1):
                B.lib().sr_debug_set(B.SR_DEBUG_FP8_INTEGER, integer_path)
                got = gpu_cast(x, gfmt, 0xABCDEF, 5 + c, 2)
                bad = np.flatnonzero(got != want)
                assert bad.size == 0, (integer_path, c, hex(c * piece + STRIDE * int(bad[0])), got[bad[0]], want[bad[0]])
    finally:
        B.lib().sr_debug_set(B.SR_DEBUG_FP8_INTEGER, 0)


@pytest.mark.parametrize("gfmt,ofmt", FMTS)
def test_fp8_cast_unbiased_on_device(gfmt, ofmt):
    y = 1.0 + 0.3 * 2.0 ** (-3 if ofmt == ref.E4M3 else -2)
    x = torch.full((1 << 16,), y, dtype=torch.float32, device=DEV)
    got = gpu_cast(x, gfmt, 11, 5, 3)
    vals = np.array([ref.fp8_decode(int(c), ofmt) for c in range(256)])[got]
    cell = 2.0 ** (-3 if ofmt == ref.E4M3 else -2)
    assert set(np.unique(vals)) == {1.0, 1.0 + cell}
    assert abs(vals.mean() - float(x[0])) <= 5 * cell * np.sqrt(0.3 * 0.7 / vals.size)


def test_fp8_cast_arguments():
    x = torch.zeros(8, dtype=torch.float32, device=DEV)
    out = torch.zeros(8, dtype=torch.uint8, device=DEV)
    with pytest.raises(B.SrError):
        B.sr_cast_f32_fp8(x, out, 2, 0, 1)
    e = torch.empty(0, dtype=torch.float32, device=DEV)
    B.sr_cast_f32_fp8(e, torch.empty(0, dtype=torch.uint8, device=DEV), B.SR_FP8_E5M2, 0, 1)
    f8 = torch.empty(8, dtype=torch.float8_e4m3fn, device=DEV)      # a torch float8 tensor as destination
    B.sr_cast_f32_fp8(torch.full((8,), 1.0, device=DEV), f8, B.SR_FP8_E4M3, 0, 1)
    torch.cuda.synchronize()
    assert bool((f8.float() == 1.0).all())
