"""MI355X-native SR-AdamW update path (arXiv 2502.20566, Algorithm 1).

The compute lives in the HIP library built from csrc/ (C ABI declared in
include/sradamw.h); `binding` marshals arguments to it, `workloads` generates
seeded synthetic inputs, `optimizer.SRAdamW` (also `paper_2502_20566_amd.SRAdamW`)
keeps the step's bookkeeping.  Nothing here computes on the CPU.
"""
__all__ = ["workloads", "binding", "optimizer", "SRAdamW"]


def __getattr__(name):
    if name == "SRAdamW":                      # imported on first use: it pulls in torch
        from .optimizer import SRAdamW
        return SRAdamW
    raise AttributeError(name)
