"""The entry point that allocates nothing, grad_global_norm_static, against grad_global_norm:
same bits, on two calls in a row, the second on a smaller list (the static scratch keeps the first
call's partial sums), then on a list that does not fit (rejected, nothing enqueued)."""
import ctypes as C

import pytest
import torch

from paper_2502_20566_amd import binding as B
from paper_2502_20566_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


def norms(shapes, seed, std):
    """(norm through the caller's workspace, norm through the static scratch) of one seeded list."""
    grads = W.make_grads(shapes, DEV, seed, std, 1e-3, 1.0)
    tl = B.TensorList(grads, grads, grads, grads)            # only .g and .numel are read
    ws = torch.empty(max(tl.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    want = torch.zeros(1, dtype=torch.float32, device=DEV)
    got = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
    B.grad_global_norm(tl, want, ws)
    B.grad_global_norm_static(tl, got)
    torch.cuda.synchronize()
    return want, got


def test_static_scratch_norm_equals_workspace_norm_twice_then_smaller():
    big = W.gpt_shapes(256, 3, 1024, 5003, 64) + [("ragged", (3 * 65536 + 77,), "weight")]
    small = W.gpt_shapes(48, 1, 192, 301, 16) + [("tail", (5,), "weight")]
    for shapes, seed, std in ((big, 11, 1e-3), (small, 12, 3e-2), (big, 13, 1e-4), (small[:3], 14, 1.0)):
        want, got = norms(shapes, seed, std)
        assert want.item() > 0.0
        # same kernels, same summation tree: identical binary32 encodings
        assert want.view(torch.int32).item() == got.view(torch.int32).item(), (want.item(), got.item())


def test_static_scratch_empty_list_and_limit():
    out = torch.full((1,), 7.0, dtype=torch.float32, device=DEV)
    rc = B.lib().grad_global_norm_static(None, 0, out.data_ptr(), None)
    torch.cuda.synchronize()
    assert rc == B.SR_OK and out.item() == 0.0
    # one partial sum per 65536 elements: a list of 2^17 + 1 tensors of one chunk each does not fit
    # in 2^20 bytes.  The pointers are never dereferenced: the size is rejected on the host.
    n = (1 << 17) + 1
    g = torch.zeros(8, dtype=torch.bfloat16, device=DEV)
    arr = (B.SrTensor * n)()
    for i in range(n):
        arr[i].g, arr[i].numel = g.data_ptr(), 8
    out.fill_(7.0)
    rc = B.lib().grad_global_norm_static(arr, n, out.data_ptr(), None)
    torch.cuda.synchronize()
    assert rc == B.SR_ERR_SIZE and out.item() == 7.0
    assert b"static scratch" in B.lib().sr_strerror(rc)


def test_static_scratch_norm_under_graph_capture():
    """What the entry point is for: after one call outside a capture (which looks the scratch
    address up), norm + clipped step are captured with no workspace in sight and replayed three
    times, with eager work and synchronisations between the replays; the result equals three eager
    calls through the workspace entry point."""
    from oracle import ref  # noqa: F401  (same import order as the other GPU tests)
    import numpy as np
    cfg = W.config(3)
    shapes = W.gpt_shapes(48, 2, 192, 1001, 32)

    def fresh():
        p = W.make_params(shapes, DEV, 61, cfg.param_std)
        m, v = W.make_moments(shapes, DEV, False)
        g = W.make_grads(shapes, DEV, 62, cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
        return p, m, v, B.TensorList(p, g, m, v), torch.zeros(1, dtype=torch.float32, device=DEV)

    p, m, v, tl, norm = fresh()
    ws = torch.empty(max(tl.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    for _ in range(3):
        B.grad_global_norm(tl, norm, ws)
        B.sr_adamw_step(tl, cfg.hyper, 5, 8, 0, norm, cfg.clip)
    torch.cuda.synchronize()
    eager = [W.bf16_to_u16_numpy(x) for x in p + m + v]

    p2, m2, v2, tl2, norm2 = fresh()
    B.grad_global_norm_static(tl2, norm2)                    # first call on the device: outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            B.grad_global_norm_static(tl2, norm2)
            B.sr_adamw_step(tl2, cfg.hyper, 5, 8, 0, norm2, cfg.clip)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    other = torch.zeros(1024, device=DEV)
    for _ in range(3):
        graph.replay()
        other += 1.0
        torch.cuda.synchronize()
    for a, b in zip(eager, [W.bf16_to_u16_numpy(x) for x in p2 + m2 + v2]):
        assert bool(np.all(a == b))
