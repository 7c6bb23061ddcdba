"""SRAdamW: a torch.optim.Optimizer over the C ABI.

Bookkeeping only -- parameter groups, the moments, the step counter, the marshalled tensor lists and
the norm workspace; every arithmetic step runs in the HIP library (grad_global_norm, sr_adamw_step).

    opt = SRAdamW(model.parameters(), lr=6e-4, max_norm=1.0, seed=0)
    opt = SRAdamW([{"params": decay}, {"params": no_decay, "weight_decay": 0.0}], lr=6e-4)
    loss.backward(); opt.step(); opt.zero_grad()

Parameters must be contiguous BF16 device tensors; gradients are read from `.grad` (BF16) or from the
tensors given to `step(grads=...)` (one per parameter, in group order).  Groups may differ in lr,
betas, eps and weight_decay (learning-rate schedulers of torch work on `param_groups` as usual); the
rounding strategy, the clip and the seed belong to the optimizer.  All replicas of a data-parallel
job must use the same `seed` and the same parameter order (Algorithm 1, lines 9 and 11: shared
randomness): the k-th parameter over all groups gets RNG tensor id k.
"""
from typing import List, Optional, Sequence, Tuple

import torch

from . import binding as B

_STRATEGIES = {
    "sr": 0,                                                     # SR on p, m, v
    "sr_param": B.SR_FLAG_RNE_MOMENTS,                            # the paper's setting: SR on p only
    "nearest": B.SR_FLAG_RNE_PARAMS | B.SR_FLAG_RNE_MOMENTS,      # plain BF16
    "fp32_moments": B.SR_FLAG_FP32_MOMENTS,
    "kahan": B.SR_FLAG_KAHAN,
    "master": B.SR_FLAG_MASTER_FP32 | B.SR_FLAG_FP32_MOMENTS,
    "fp8_moments": B.SR_FLAG_FP8_MOMENTS,                         # extension: m as E4M3, v as E5M2 codes
}


class SRAdamW(torch.optim.Optimizer):
    def __init__(self, params, lr: float = 1e-3, betas=(0.9, 0.95), eps: float = 1e-8,
                 weight_decay: float = 0.1, max_norm: Optional[float] = None, seed: int = 0,
                 strategy: str = "sr", eps_in_root: bool = False, divide_bias_correction: bool = False,
                 fp8_exponents: Optional[Tuple[int, int]] = None):
        """fp8_exponents = (m_exp, v_exp): with strategy "fp8_moments" the moments are stored as
        Q_SR(m 2^m_exp) in E4M3 and Q_SR(v 2^v_exp) in E5M2 (one byte each); choose the exponents so
        that the largest |m| 2^m_exp stays below 448 and the largest v 2^v_exp below 57344 (larger
        values saturate or become infinite)."""
        if strategy not in _STRATEGIES:
            raise ValueError(f"strategy must be one of {sorted(_STRATEGIES)}")
        if (strategy == "fp8_moments") != (fp8_exponents is not None):
            raise ValueError('fp8_exponents goes with strategy "fp8_moments" (and is required by it)')
        super().__init__(params, dict(lr=lr, betas=tuple(betas), eps=eps, weight_decay=weight_decay))
        self.strategy = strategy
        self.flags = _STRATEGIES[strategy]
        if eps_in_root:
            self.flags |= B.SR_FLAG_EPS_IN_ROOT
        if divide_bias_correction:
            self.flags |= B.SR_FLAG_DIV_BIAS
        self.fp32_moments = bool(self.flags & B.SR_FLAG_FP32_MOMENTS)
        self.fp8_exponents = None if fp8_exponents is None else (int(fp8_exponents[0]), int(fp8_exponents[1]))
        self.max_norm = max_norm
        self.seed = seed
        self.t = 0
        mdt = torch.float32 if self.fp32_moments else torch.uint8 if self.fp8_exponents else torch.bfloat16
        self._flat: List[List[torch.Tensor]] = []                 # per group: flat views of the parameters
        dev = None
        for group in self.param_groups:
            flat = [p.detach().view(-1) for p in group["params"]]
            self._flat.append(flat)
            for p, f in zip(group["params"], flat):
                dev = f.device
                st = self.state[p]
                st["exp_avg"] = torch.zeros(f.numel(), dtype=mdt, device=f.device)
                st["exp_avg_sq"] = torch.zeros(f.numel(), dtype=mdt, device=f.device)
                if strategy == "kahan":
                    st["aux"] = torch.zeros_like(f)               # BF16 compensation
                elif strategy == "master":
                    st["aux"] = f.float()                         # binary32 master copy
        self.norm = torch.zeros(1, dtype=torch.float32, device=dev or torch.device("cuda"))
        self._lists = None                                        # (per-group TensorLists, list of all tensors)
        self._grad_ptrs = None
        self._ws = None

    # ------------------------------------------------------------------ marshalling

    def _all_params(self) -> List[torch.Tensor]:
        return [p for group in self.param_groups for p in group["params"]]

    def _lists_for(self, grads: Sequence[torch.Tensor]):
        ptrs = tuple(g.data_ptr() for g in grads)
        if self._lists is None or ptrs != self._grad_ptrs:        # rebuilt only when gradient buffers move
            per_group, k = [], 0
            for group, flat in zip(self.param_groups, self._flat):
                n = len(flat)
                st = [self.state[p] for p in group["params"]]
                aux = [s["aux"] for s in st] if (n and "aux" in st[0]) else None
                per_group.append(B.TensorList(flat, [g.view(-1) for g in grads[k:k + n]],
                                              [s["exp_avg"] for s in st], [s["exp_avg_sq"] for s in st],
                                              self.fp32_moments, tensor_ids=list(range(k, k + n)), aux=aux,
                                              fp8_exponents=None if self.fp8_exponents is None
                                              else [self.fp8_exponents] * n))
                k += n
            everything = None
            if self.max_norm is not None:                         # the norm runs over all groups at once
                flat_all = [f for flat in self._flat for f in flat]
                g_all = [g.view(-1) for g in grads]
                everything = B.TensorList(flat_all, g_all, g_all, g_all)      # only .g and .numel are read
                need = max(everything.workspace_bytes(), 256)
                if self._ws is None or self._ws.numel() < need:
                    self._ws = torch.empty(need, dtype=torch.uint8, device=self.norm.device)
            # the lists hold the gradients' addresses, not the tensors: a gradient buffer that the
            # framework frees after the step (zero_grad(set_to_none=True)) must not be kept alive here
            for tl in per_group + ([everything] if everything is not None else []):
                tl.keep = (tl.keep[0], None, tl.keep[2] if tl is not everything else None,
                           tl.keep[3] if tl is not everything else None, tl.keep[4])
            self._lists = (per_group, everything)
            self._grad_ptrs = ptrs
        return self._lists

    # ------------------------------------------------------------------ the step

    @torch.no_grad()
    def step(self, closure=None, grads: Optional[Sequence[torch.Tensor]] = None, lr: Optional[float] = None):
        """One update (Algorithm 1 lines 5-10) on the current stream.  `lr` sets the learning rate of
        every group for this and later steps; `grads` replaces the parameters' `.grad`."""
        loss = None
        if closure is not None:
            with torch.enable_grad():
                loss = closure()
        if grads is None:
            grads = [p.grad for p in self._all_params()]
            if any(g is None for g in grads):
                raise ValueError("every parameter needs a gradient (pass grads=... otherwise)")
        if lr is not None:
            for group in self.param_groups:
                group["lr"] = lr
        per_group, everything = self._lists_for(grads)
        self.t += 1
        if self.max_norm is not None:
            B.grad_global_norm(everything, self.norm, self._ws)
        for group, tl in zip(self.param_groups, per_group):
            hyper = dict(lr=group["lr"], beta1=group["betas"][0], beta2=group["betas"][1], eps=group["eps"],
                         weight_decay=group["weight_decay"])
            if self.max_norm is not None:
                B.sr_adamw_step(tl, hyper, self.t, self.seed, self.flags, self.norm, self.max_norm)
            else:
                B.sr_adamw_step(tl, hyper, self.t, self.seed, self.flags)
        return loss

    # ------------------------------------------------------------------ checkpoints

    def state_dict(self) -> dict:
        """Everything a resume needs: the RNG is stateless, so (seed, step), the groups' settings and
        the state tensors, in parameter order.  (torch's own packing would cast binary32 moments of
        BF16 parameters to BF16 on load, so the format is ours.)"""
        params = self._all_params()
        return dict(t=self.t, seed=self.seed, strategy=self.strategy, fp8_exponents=self.fp8_exponents,
                    param_groups=[{k: v for k, v in g.items() if k != "params"} for g in self.param_groups],
                    state=[dict(self.state[p]) for p in params])

    def load_state_dict(self, sd: dict) -> None:
        if sd.get("strategy", self.strategy) != self.strategy:
            raise ValueError(f"checkpoint was written with strategy {sd['strategy']!r}, this optimizer uses {self.strategy!r}")
        if sd.get("fp8_exponents") is not None and tuple(sd["fp8_exponents"]) != self.fp8_exponents:
            raise ValueError(f"checkpoint uses fp8 scale exponents {sd['fp8_exponents']}, this optimizer {self.fp8_exponents}")
        self.t, self.seed = sd["t"], sd["seed"]
        for group, saved in zip(self.param_groups, sd["param_groups"]):
            group.update(saved)
        for p, saved in zip(self._all_params(), sd["state"]):
            for k, dst in self.state[p].items():
                dst.copy_(saved[k])
