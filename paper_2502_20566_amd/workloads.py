"""Seeded synthetic inputs for the SR-AdamW update path.

This module only GENERATES data (shapes, random values, special-value masks).
It holds none of the method's arithmetic -- no rounding rule, no RNG of the
method, no optimizer formula -- so both the CPU checker and the GPU library
can be fed from it.  It does not import the HIP binding.

The parameter sets stand in for the GPT-2 / GPT-Neo models the paper trains
(Section 5.1, Table 1): only tensor shapes and value distributions matter to
the optimizer update, so weights are N(0, 0.02) noise (the GPT-2 initialisation
scale), LayerNorm gains are 1, biases are 0, and gradients are zero-mean noise
of a stated standard deviation with an optional fraction of large outliers.
No dataset, checkpoint or benchmark item is involved.
"""
from dataclasses import dataclass
from typing import List, Optional, Tuple

import torch

SEED_BASE = 0x5EED0000


def data_seed(config: int, step: int) -> int:
    return SEED_BASE + 1000 * config + step


# ------------------------------------------------------------------- shapes

def gpt_shapes(d: int, n_layer: int, ffn: int, vocab: int, ctx: int) -> List[Tuple[str, Tuple[int, ...], str]]:
    """(name, shape, kind) for a GPT-2-style decoder; kind in {'weight','gain','bias'}."""
    out = [("wte", (vocab, d), "weight"), ("wpe", (ctx, d), "weight")]
    for l in range(n_layer):
        pre = f"h{l}."
        out += [
            (pre + "ln1.w", (d,), "gain"), (pre + "ln1.b", (d,), "bias"),
            (pre + "qkv.w", (d, 3 * d), "weight"), (pre + "qkv.b", (3 * d,), "bias"),
            (pre + "proj.w", (d, d), "weight"), (pre + "proj.b", (d,), "bias"),
            (pre + "ln2.w", (d,), "gain"), (pre + "ln2.b", (d,), "bias"),
            (pre + "fc.w", (d, ffn), "weight"), (pre + "fc.b", (ffn,), "bias"),
            (pre + "fcproj.w", (ffn, d), "weight"), (pre + "fcproj.b", (d,), "bias"),
        ]
    out += [("lnf.w", (d,), "gain"), ("lnf.b", (d,), "bias")]
    return out


def numel_of(shape) -> int:
    n = 1
    for s in shape:
        n *= s
    return n


def total_numel(shapes) -> int:
    return sum(numel_of(s) for _, s, _ in shapes)


@dataclass
class Config:
    """One benchmark / parity configuration (hyper-parameters follow Section 5.1:
    beta = (0.9, 0.95), eps = 1e-8, weight decay 0.1 unless the config says otherwise)."""
    index: int
    name: str
    shapes: list                      # list of (name, shape, kind); a flat buffer is one 'weight'
    lr: float
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1
    steps: int = 1
    param_std: float = 0.02
    grad_std: float = 1e-4
    outlier_frac: float = 0.0
    outlier_std: float = 1.0
    clip: Optional[float] = None      # max_norm, None = no clipping
    fp32_moments: bool = False
    warm_steps: int = 0               # moments warm-started by this many seeded steps
    seed: int = 0                     # SR seed

    @property
    def hyper(self):
        return dict(lr=self.lr, beta1=self.beta1, beta2=self.beta2, eps=self.eps,
                    weight_decay=self.weight_decay)

    @property
    def numel(self):
        return total_numel(self.shapes)


def config(index: int) -> Config:
    if index == 1:
        return Config(1, "flat-2^20", [("flat", (1 << 20,), "weight")], lr=1e-3, beta2=0.999,
                      grad_std=1e-3, steps=1)
    if index == 2:
        return Config(2, "gpt2-small-124M", gpt_shapes(768, 12, 3072, 50257, 1024), lr=6e-4,
                      grad_std=1e-4, steps=10)
    if index == 3:
        return Config(3, "gpt2-350M", gpt_shapes(1024, 24, 4096, 50257, 1024), lr=3e-3,
                      grad_std=1e-3, outlier_frac=1e-3, outlier_std=1.0, clip=1.0, steps=10)
    if index == 4:
        return Config(4, "gpt-2.7B-fp32-moments", gpt_shapes(2560, 32, 10240, 50272, 2048),
                      lr=1.6e-4, grad_std=1e-4, clip=1.0, fp32_moments=True, steps=5)
    if index == 5:
        n = total_numel(gpt_shapes(4096, 32, 16384, 50272, 2048))
        return Config(5, "gpt-6.7B-flat", [("flat", (n,), "weight")], lr=1.2e-4, grad_std=1e-4,
                      warm_steps=100, steps=1)
    raise ValueError(f"no config {index}")


def scaled_down(cfg: Config, d: int, n_layer: int, ffn: int, vocab: int, ctx: int) -> Config:
    """Same recipe on a smaller GPT shape list (CPU-sized parity cases)."""
    import copy
    c = copy.copy(cfg)
    c.shapes = gpt_shapes(d, n_layer, ffn, vocab, ctx)
    c.name = cfg.name + f"-scaled(d={d},L={n_layer})"
    return c


# --------------------------------------------------------------- generators

_CHUNK = 1 << 26   # elements generated per call, bounds the FP32 temporaries


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _fill_normal_bf16(out: torch.Tensor, std: float, gen) -> None:
    flat = out.view(-1)
    n = flat.numel()
    for s in range(0, n, _CHUNK):
        e = min(n, s + _CHUNK)
        tmp = torch.randn(e - s, device=out.device, dtype=torch.float32, generator=gen)
        flat[s:e] = (tmp * std).to(torch.bfloat16)


def make_params(shapes, device, seed: int, std: float = 0.02) -> List[torch.Tensor]:
    """BF16 parameters, one flat tensor per entry: weights ~ N(0, std), gains = 1, biases = 0."""
    gen = _gen(device, seed)
    out = []
    for _, shape, kind in shapes:
        t = torch.empty(numel_of(shape), device=device, dtype=torch.bfloat16)
        if kind == "weight":
            _fill_normal_bf16(t, std, gen)
        elif kind == "gain":
            t.fill_(1.0)
        else:
            t.zero_()
        out.append(t)
    return out


def fill_grads(grads: List[torch.Tensor], seed: int, std: float, outlier_frac: float = 0.0,
               outlier_std: float = 1.0) -> None:
    """Overwrite `grads` with BF16 N(0, std); a seeded fraction replaced by N(0, outlier_std)."""
    if not grads:
        return
    gen = _gen(grads[0].device, seed)
    for t in grads:
        flat = t.view(-1)
        n = flat.numel()
        for s in range(0, n, _CHUNK):
            e = min(n, s + _CHUNK)
            tmp = torch.randn(e - s, device=t.device, dtype=torch.float32, generator=gen) * std
            if outlier_frac > 0.0:
                mask = torch.rand(e - s, device=t.device, generator=gen) < outlier_frac
                big = torch.randn(e - s, device=t.device, dtype=torch.float32, generator=gen) * outlier_std
                tmp = torch.where(mask, big, tmp)
            flat[s:e] = tmp.to(torch.bfloat16)


def make_grads(shapes, device, seed: int, std: float, outlier_frac: float = 0.0,
               outlier_std: float = 1.0) -> List[torch.Tensor]:
    grads = [torch.empty(numel_of(s), device=device, dtype=torch.bfloat16) for _, s, _ in shapes]
    fill_grads(grads, seed, std, outlier_frac, outlier_std)
    return grads


def make_moments(shapes, device, fp32: bool) -> Tuple[List[torch.Tensor], List[torch.Tensor]]:
    dt = torch.float32 if fp32 else torch.bfloat16
    m = [torch.zeros(numel_of(s), device=device, dtype=dt) for _, s, _ in shapes]
    v = [torch.zeros(numel_of(s), device=device, dtype=dt) for _, s, _ in shapes]
    return m, v


def make_cast_input(n: int, device, seed: int) -> torch.Tensor:
    """FP32 values uniform in [-4, 4]; a seeded 1% overwritten by their own value with the
    low 16 encoding bits cleared (values that already are BF16 values), another seeded 1%
    by FP32 subnormals (random sign, zero exponent field, random non-zero mantissa)."""
    gen = _gen(device, seed)
    x = (torch.rand(n, device=device, dtype=torch.float32, generator=gen) * 8.0) - 4.0
    sel = torch.rand(n, device=device, generator=gen)
    bits = x.view(torch.int32)
    exact = sel < 0.01
    bits[exact] = bits[exact] & ~0xFFFF
    sub = (sel >= 0.01) & (sel < 0.02)
    k = int(sub.sum().item())
    mant = torch.randint(1, 1 << 23, (k,), device=device, dtype=torch.int32, generator=gen)
    sign = torch.randint(0, 2, (k,), device=device, dtype=torch.int32, generator=gen)
    bits[sub] = mant | (sign << 31)
    return x


# ------------------------------------------------------------ host plumbing

def bf16_to_u16_numpy(t: torch.Tensor):
    """BF16 tensor -> numpy uint16 array of its bit patterns (host copy)."""
    import numpy as np
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16).copy()


def u16_numpy_to_bf16(a, device) -> torch.Tensor:
    import numpy as np
    return torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16).to(device)
