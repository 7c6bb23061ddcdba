"""A small optimizer object over the C ABI: keeps the marshalled tensor list, the moments, the
step counter and the norm workspace, and issues grad_global_norm + sr_adamw_step once per step.
Argument bookkeeping only -- every arithmetic step runs in the HIP library.

    opt = SRAdamW(model.parameters(), lr=6e-4, max_norm=1.0, seed=0)
    loss.backward(); opt.step(); opt.zero_grad()

Parameters must be contiguous BF16 device tensors; gradients are read from `.grad` (BF16) or from
the tensors given to `step(grads=...)`.  All replicas of a data-parallel job must use the same
`seed` and the same parameter order (Algorithm 1, lines 9 and 11: shared randomness): tensor i of
the list gets RNG tensor id i.
"""
from typing import Iterable, List, Optional, Sequence

import torch

from . import binding as B

_STRATEGIES = {
    "sr": 0,                                                     # SR on p, m, v
    "sr_param": B.SR_FLAG_RNE_MOMENTS,                            # the paper's setting: SR on p only
    "nearest": B.SR_FLAG_RNE_PARAMS | B.SR_FLAG_RNE_MOMENTS,      # plain BF16
    "fp32_moments": B.SR_FLAG_FP32_MOMENTS,
    "kahan": B.SR_FLAG_KAHAN,
    "master": B.SR_FLAG_MASTER_FP32 | B.SR_FLAG_FP32_MOMENTS,
}


class SRAdamW:
    def __init__(self, params: Iterable[torch.Tensor], lr: float = 1e-3, betas=(0.9, 0.95), eps: float = 1e-8,
                 weight_decay: float = 0.1, max_norm: Optional[float] = None, seed: int = 0,
                 strategy: str = "sr", eps_in_root: bool = False, divide_bias_correction: bool = False):
        self.params: List[torch.Tensor] = [p for p in params]
        if strategy not in _STRATEGIES:
            raise ValueError(f"strategy must be one of {sorted(_STRATEGIES)}")
        self.flags = _STRATEGIES[strategy]
        if eps_in_root:
            self.flags |= B.SR_FLAG_EPS_IN_ROOT
        if divide_bias_correction:
            self.flags |= B.SR_FLAG_DIV_BIAS
        self.fp32_moments = bool(self.flags & B.SR_FLAG_FP32_MOMENTS)
        self.hyper = dict(lr=lr, beta1=betas[0], beta2=betas[1], eps=eps, weight_decay=weight_decay)
        self.max_norm = max_norm
        self.seed = seed
        self.t = 0
        mdt = torch.float32 if self.fp32_moments else torch.bfloat16
        flat = [p.detach().view(-1) for p in self.params]
        self.m = [torch.zeros(p.numel(), dtype=mdt, device=p.device) for p in flat]
        self.v = [torch.zeros(p.numel(), dtype=mdt, device=p.device) for p in flat]
        self.aux = None
        if strategy == "kahan":
            self.aux = [torch.zeros_like(p) for p in flat]
        elif strategy == "master":
            self.aux = [p.float() for p in flat]
        self._flat = flat
        self._tl = None
        self._grad_ptrs = None
        dev = flat[0].device if flat else torch.device("cuda")
        self.norm = torch.zeros(1, dtype=torch.float32, device=dev)
        self._ws = None

    def _list_for(self, grads: Sequence[torch.Tensor]) -> B.TensorList:
        ptrs = tuple(g.data_ptr() for g in grads)
        if self._tl is None or ptrs != self._grad_ptrs:        # rebuilt only when gradient buffers move
            self._tl = B.TensorList(self._flat, [g.view(-1) for g in grads], self.m, self.v,
                                    self.fp32_moments, aux=self.aux)
            self._grad_ptrs = ptrs
            if self.max_norm is not None:
                need = max(self._tl.workspace_bytes(), 256)
                if self._ws is None or self._ws.numel() < need:
                    self._ws = torch.empty(need, dtype=torch.uint8, device=self.norm.device)
        return self._tl

    def step(self, grads: Optional[Sequence[torch.Tensor]] = None, lr: Optional[float] = None) -> None:
        """One update (Algorithm 1 lines 5-10) on the current stream.  `lr` overrides the stored
        learning rate for this and later steps (schedules)."""
        if grads is None:
            grads = [p.grad for p in self.params]
            if any(g is None for g in grads):
                raise ValueError("every parameter needs a gradient (pass grads=... otherwise)")
        if lr is not None:
            self.hyper["lr"] = lr
        tl = self._list_for(grads)
        self.t += 1
        if self.max_norm is not None:
            B.grad_global_norm(tl, self.norm, self._ws)
            B.sr_adamw_step(tl, self.hyper, self.t, self.seed, self.flags, self.norm, self.max_norm)
        else:
            B.sr_adamw_step(tl, self.hyper, self.t, self.seed, self.flags)

    def zero_grad(self) -> None:
        for p in self.params:
            p.grad = None

    def state_dict(self) -> dict:
        """Everything a resume needs: the RNG is stateless, so (seed, step) and the tensors."""
        return dict(t=self.t, seed=self.seed, hyper=dict(self.hyper), m=self.m, v=self.v, aux=self.aux)

    def load_state_dict(self, sd: dict) -> None:
        self.t, self.seed = sd["t"], sd["seed"]
        self.hyper.update(sd["hyper"])
        for dst, src in zip(self.m, sd["m"]):
            dst.copy_(src)
        for dst, src in zip(self.v, sd["v"]):
            dst.copy_(src)
        if self.aux is not None:
            for dst, src in zip(self.aux, sd["aux"]):
                dst.copy_(src)
