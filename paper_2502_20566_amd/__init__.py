"""MI355X-native SR-AdamW update path (arXiv 2502.20566, Algorithm 1).

The compute lives in the HIP library built from csrc/ (C ABI declared in
include/sradamw.h); `binding` marshals arguments to it and `workloads`
generates seeded synthetic inputs; `optimizer.SRAdamW` keeps the step's bookkeeping.  Nothing here computes on the CPU.
"""
__all__ = ["workloads", "binding", "optimizer"]
