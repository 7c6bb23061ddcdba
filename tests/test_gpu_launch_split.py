"""Jobs larger than one dispatch (2^32 - 1 work-items) are cut into several launches, tensors into
pieces at counter-block boundaries.  The hardware limit needs tens of billions of elements to
reach; sr_debug_set(SR_DEBUG_LAUNCH_LIMIT, n) lowers it so that small inputs take the same host paths.  Every
entry point must give the bits it gives in one launch -- which the other tests pin to the oracle."""
import numpy as np
import pytest
import torch

import test_gpu_fp8_moments as F8
import test_gpu_parity as P
from oracle import ref
from paper_2502_20566_amd import binding as B
from paper_2502_20566_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.fixture
def limit():
    yield lambda n: B.lib().sr_debug_set(B.SR_DEBUG_LAUNCH_LIMIT, n)
    B.lib().sr_debug_set(B.SR_DEBUG_LAUNCH_LIMIT, 0)


@pytest.mark.parametrize("mode", ["sr", "fp32", "kahan", "master"])
@pytest.mark.parametrize("wgs", [1, 3, 10])
def test_update_and_norm_cut_into_many_launches_match_the_oracle(limit, mode, wgs):
    limit(wgs)
    P.test_adamw_ragged_misaligned_and_offset_tensors(mode)


@pytest.mark.parametrize("wgs", [1, 4])
def test_update_with_8_bit_moments_cut_into_many_launches(limit, wgs):
    limit(wgs)
    F8.test_fp8_moments_many_steps_with_clip_and_offsets()
    F8.test_fp8_moments_every_code_as_input(0)


@pytest.mark.parametrize("wgs", [1, 5])
def test_accumulate_with_norm_cut_into_many_launches(limit, wgs):
    limit(wgs)
    P.test_grad_accumulate_micro_batches_bit_exact_with_fused_norm()


@pytest.mark.parametrize("wgs", [1, 2, 7])
def test_casts_and_probe_cut_into_many_launches(limit, wgs):
    n = 5003
    x = W.make_cast_input(n, DEV, 31)
    host = x.cpu().numpy()
    want16 = ref.sr_cast_f32_bf16(host, 4, 2, 9)
    want8 = [ref.sr_cast_f32_fp8(host, f, 4, 2, 9) for f in (ref.E4M3, ref.E5M2)]
    limit(wgs)
    out16 = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    B.sr_cast_f32_bf16(x, out16, 4, 2, 9)
    assert np.array_equal(P.to_np(out16), want16)
    for f, w in zip((B.SR_FP8_E4M3, B.SR_FP8_E5M2), want8):
        out8 = torch.zeros(n, dtype=torch.uint8, device=DEV)
        B.sr_cast_f32_fp8(x, out8, f, 4, 2, 9)
        torch.cuda.synchronize()
        assert np.array_equal(out8.cpu().numpy(), w)
    ts = [(torch.randn(n, device=DEV) * 0.01).to(torch.bfloat16) for _ in range(4)]
    before = [P.to_np(t) for t in ts]
    B.sr_stream_probe(*ts)
    torch.cuda.synchronize()
    assert all(np.array_equal(P.to_np(t), b) for t, b in zip(ts, before))


def test_norm_bits_do_not_depend_on_the_cut(limit):
    grads = W.make_grads(W.gpt_shapes(48, 2, 192, 1001, 32) + [("big", (3 * 65536 + 17,), "weight")], DEV, 5, 1e-3)
    tl = B.TensorList(grads, grads, grads, grads)
    ws = torch.empty(max(tl.workspace_bytes(), 256), dtype=torch.uint8, device=DEV)
    got = []
    for wgs in (0, 1, 2):
        limit(wgs)
        norm = torch.zeros(1, dtype=torch.float32, device=DEV)
        B.grad_global_norm(tl, norm, ws)
        torch.cuda.synchronize()
        got.append(norm.cpu().numpy().view(np.uint32)[0])
    assert got[0] == got[1] == got[2]
