"""Pins of the oracle's BF16 gradient accumulation with stochastic rounding (CPU only):
outputs are neighbours of the exact sum, the mean over seeds is the exact sum (Section 2.1,
E[Q_SR(x)] = x), nearest rounding equals torch's cast and stagnates once the accumulator dwarfs the
micro-gradient while SR keeps accumulating in expectation (Section 2.1's x + u example)."""
import numpy as np
import pytest

from oracle import ref

torch = pytest.importorskip("torch")


def trunc_bits(x):
    return (np.asarray(x, np.float32).view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def val(b):
    return ref.bf16_bits_to_f32(np.asarray(b, np.uint16))


def torch_rne_bits(x):
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_accumulate_rounds_the_exact_binary32_sum():
    n = 8192
    rng = np.random.default_rng(0)
    acc0 = trunc_bits(rng.standard_normal(n) * 1e-3)
    g = trunc_bits(rng.standard_normal(n) * 1e-4)
    scale = np.float32(0.25)
    s = (val(acc0) + (scale * val(g)).astype(np.float32)).astype(np.float32)     # scale*g exact here (power of two)
    lo = (s.view(np.uint32) >> np.uint32(16)).astype(np.uint16)
    for seed in (0, 1):
        acc = acc0.copy()
        ref.grad_accumulate(acc, g, float(scale), 7, seed, tensor_id=3)
        assert bool(np.all((acc == lo) | (acc == lo + 1)))
        # the draw is r16(seed, micro_step, tensor, index, stream 4): away from zero iff r + k >= 65536
        k = (s.view(np.uint32) & np.uint32(0xFFFF)).astype(np.int64)
        r = ref.r16_many(seed, 7, 3, 0, n, ref.STREAM_ACC).astype(np.int64)
        assert bool(np.all((acc == lo + 1) == (r + k >= 65536)))
    # nearest rounding = torch's cast; first micro-batch ignores the old accumulator
    acc = acc0.copy()
    ref.grad_accumulate(acc, g, float(scale), 7, 0, flags=ref.ACC_RNE)
    assert bool(np.all(acc == torch_rne_bits(s)))
    acc = acc0.copy()
    ref.grad_accumulate(acc, g, 3.0, 7, 0, flags=ref.ACC_RNE | ref.ACC_FIRST)
    assert bool(np.all(acc == torch_rne_bits((np.float32(3.0) * val(g)).astype(np.float32))))
    # element offset = window
    whole = acc0.copy(); ref.grad_accumulate(whole, g, 0.3, 2, 9, tensor_id=1)
    win = acc0[100:900].copy(); ref.grad_accumulate(win, g[100:900], 0.3, 2, 9, tensor_id=1, elem_offset=100)
    assert bool(np.all(win == whole[100:900]))


def test_accumulate_is_unbiased_over_seeds():
    n = 64
    rng = np.random.default_rng(1)
    acc0 = trunc_bits(rng.standard_normal(n) * 1e-2)
    g = trunc_bits(rng.standard_normal(n) * 1e-4)
    s = (val(acc0) + (np.float32(0.5) * val(g)).astype(np.float32)).astype(np.float32).astype(np.float64)
    n_seeds = 10000
    tot = np.zeros(n)
    for seed in range(n_seeds):
        acc = acc0.copy()
        ref.grad_accumulate(acc, g, 0.5, 1, seed, nthreads=1)
        tot += val(acc).astype(np.float64)
    spacing = 2.0 ** (np.floor(np.log2(np.abs(s))) - 7)
    assert bool(np.all(np.abs(tot / n_seeds - s) <= 5 * spacing * 0.5 / np.sqrt(n_seeds)))


def test_accumulation_of_many_small_micro_gradients():
    """64 micro-batches of gradients 1/256 the size of the running sum's spacing region:
    nearest rounding stops accumulating, SR's sum is right in the mean."""
    n, K = 4096, 64
    g = trunc_bits(np.full(n, 2.0 ** -12, np.float32))
    acc_sr = trunc_bits(np.full(n, 1.0, np.float32))
    acc_nr = acc_sr.copy()
    for k in range(K):
        ref.grad_accumulate(acc_sr, g, 1.0, k + 1, 5)
        ref.grad_accumulate(acc_nr, g, 1.0, k + 1, 5, flags=ref.ACC_RNE)
    exact = 1.0 + K * 2.0 ** -12
    assert bool(np.all(val(acc_nr) == 1.0))                        # 2^-12 < half a spacing (2^-8): stagnates
    mean = float(val(acc_sr).astype(np.float64).mean())
    # per element the sum of K Bernoulli(2^-12/2^-7) moves of 2^-7: sd = 2^-7 sqrt(K q (1-q))
    q = 2.0 ** -5
    sd = 2.0 ** -7 * np.sqrt(K * q * (1 - q)) / np.sqrt(n)
    assert abs(mean - exact) <= 5 * sd
