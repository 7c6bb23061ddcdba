"""The C-ABI library loads, exports what include/sradamw.h declares, and rejects bad arguments
on the host before anything is launched (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest
import torch

from paper_2502_20566_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HAVE_GPU = torch.cuda.is_available()
_keep = []


def buf(nbytes: int, misalign: int = 0) -> int:
    """An address for a tensor argument.  On a GPU machine it is real device memory (so that a
    validation bug could not turn into a wild access); without a GPU nothing can be launched
    and a made-up aligned address serves."""
    if HAVE_GPU:
        t = torch.zeros(nbytes + 64, dtype=torch.uint8, device="cuda")
        _keep.append(t)
        return t.data_ptr() + misalign
    return 0x7F0000001000 + 0x100000 * len(_keep) + misalign


def tensor(numel=64, **kw):
    t = B.SrTensor()
    t.p, t.g, t.m, t.v = buf(2 * numel), buf(2 * numel), buf(4 * numel), buf(4 * numel)
    t.aux = None
    t.numel, t.elem_offset, t.tensor_id, t.m_exp, t.v_exp, t.p_exp, t.reserved = numel, 0, 0, 0, 0, 0, 0
    for k, v in kw.items():
        setattr(t, k, v)
    return t


def step(tensors, hyper=None, step=1, seed=0, flags=0, norm=None, max_norm=0.0):
    arr = (B.SrTensor * max(len(tensors), 1))(*tensors)
    h = B.SrHyper(*(hyper or (1e-3, 0.9, 0.95, 1e-8, 0.1)))
    return B.lib().sr_adamw_step(arr, len(tensors), C.byref(h), step, seed, flags, norm, max_norm, None)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sradamw.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name)
    assert L.sr_version() >= 100
    assert C.sizeof(B.SrTensor) == 64 and C.sizeof(B.SrHyper) == 20


def test_header_is_plain_c_and_struct_layouts_match_the_binding(tmp_path):
    """include/sradamw.h compiles as C99 on its own, and the struct layouts the C compiler derives
    from it are the ones the ctypes binding uses."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no host C compiler")
    fields = {"sr_tensor_t": ["p", "g", "m", "v", "aux", "numel", "elem_offset", "tensor_id", "m_exp", "v_exp", "p_exp", "reserved"],
              "sr_accum_t": ["acc", "grad", "numel", "elem_offset", "tensor_id", "reserved"],
              "sr_hyper_t": ["lr", "beta1", "beta2", "eps", "weight_decay"]}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "sradamw.h"', 'int main(void) {']
    for st, fs in fields.items():
        lines.append(f'printf("{st} %zu", sizeof({st}));')
        for f in fs:
            lines.append(f'printf(" %zu", offsetof({st}, {f}));')
        lines.append('printf("\\n");')
    lines += ['return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    ct = {"sr_tensor_t": B.SrTensor, "sr_accum_t": B.SrAccum, "sr_hyper_t": B.SrHyper}
    for line in filter(None, out):
        name, size, *offs = line.split()
        assert int(size) == C.sizeof(ct[name])
        assert [int(o) for o in offs] == [getattr(ct[name], f).offset for f in fields[name]]


def test_strerror_covers_all_codes():
    L = B.lib()
    msgs = {c: L.sr_strerror(c).decode() for c in (0, -1, -2, -3, -4, -5, -6, -99)}
    assert len(set(msgs.values())) == 8 and msgs[0] == "ok"


def test_workspace_bytes_bounds_the_partials():
    L = B.lib()
    chunk = 512 * 8 * 16
    for n_t, numel in [(0, 0), (1, 1), (3, chunk), (388, 2651591680), (1, 6658465792)]:
        w = L.sr_workspace_bytes(n_t, numel)
        assert w % 256 == 0 and w >= 8 * (numel // chunk + n_t)


def test_adamw_argument_errors():
    t = tensor()
    assert step([t], step=0) == B.SR_ERR_ARG
    assert step([t], hyper=(1e-3, 1.0, 0.95, 1e-8, 0.1)) == B.SR_ERR_ARG
    assert step([t], hyper=(1e-3, 0.9, -0.1, 1e-8, 0.1)) == B.SR_ERR_ARG
    assert step([t], hyper=(1e-3, 0.9, 0.95, -1e-8, 0.1)) == B.SR_ERR_ARG
    assert step([t], hyper=(float("nan"), 0.9, 0.95, 1e-8, 0.1)) == B.SR_ERR_ARG
    assert step([t], hyper=(1e-3, 0.9, 0.95, float("inf"), 0.1)) == B.SR_ERR_ARG
    assert step([t], hyper=(1e-3, 0.9, 0.95, 1e-8, float("nan"))) == B.SR_ERR_ARG
    assert step([t], flags=1024) == B.SR_ERR_ARG
    # the 8-bit parameter combines with 8-bit moments and the arithmetic variants only
    for bad in (512 | 1, 512 | 2, 512 | 4, 512 | 16, 512 | 8 | 1):
        assert step([t], flags=bad) == B.SR_ERR_ARG
    assert step([tensor(p_exp=101)], flags=512) == B.SR_ERR_ARG
    assert step([tensor(p_exp=-101)], flags=512 | 128) == B.SR_ERR_ARG
    assert step([tensor(p_exp=3)]) == B.SR_ERR_ARG                           # zero without the flag
    assert step([tensor(elem_offset=2 ** 63)], flags=512) == B.SR_ERR_ARG    # the 32-bit-word stream's index range
    for bad in (128 | 1, 128 | 2, 128 | 8 | 1, 128 | 16):        # 8-bit moments combine with few flags
        assert step([t], flags=bad) == B.SR_ERR_ARG
    assert step([tensor(reserved=1)], flags=128) == B.SR_ERR_ARG
    assert step([tensor(m_exp=101)], flags=128) == B.SR_ERR_ARG              # scale exponents lie in [-100, 100]
    assert step([tensor(v_exp=-101)], flags=128) == B.SR_ERR_ARG
    assert step([tensor(m_exp=1)]) == B.SR_ERR_ARG                           # and are zero without 8-bit moments
    assert step([tensor(v_exp=-1)], flags=B.SR_FLAG_RNE_MOMENTS) == B.SR_ERR_ARG
    # comparison strategies: exact flag combinations and an aux tensor are required
    assert step([t], flags=B.SR_FLAG_MASTER_FP32) == B.SR_ERR_ARG
    assert step([t], flags=B.SR_FLAG_KAHAN | B.SR_FLAG_FP32_MOMENTS) == B.SR_ERR_ARG
    assert step([t], flags=B.SR_FLAG_KAHAN | B.SR_FLAG_MASTER_FP32 | B.SR_FLAG_FP32_MOMENTS) == B.SR_ERR_ARG
    assert step([t], flags=B.SR_FLAG_KAHAN) == B.SR_ERR_NULL
    assert step([t], flags=B.SR_FLAG_MASTER_FP32 | B.SR_FLAG_FP32_MOMENTS) == B.SR_ERR_NULL
    assert step([tensor(aux=t.m + 1)], flags=B.SR_FLAG_KAHAN) == B.SR_ERR_ALIGN
    assert step([tensor(aux=t.m + 2)], flags=B.SR_FLAG_MASTER_FP32 | B.SR_FLAG_FP32_MOMENTS) == B.SR_ERR_ALIGN
    assert step([tensor(reserved=1)]) == B.SR_ERR_ARG
    assert step([tensor(elem_offset=2 ** 64 - 8)]) == B.SR_ERR_ARG
    nrm = buf(4)
    assert step([t], norm=nrm, max_norm=0.0) == B.SR_ERR_ARG
    assert step([t], norm=nrm, max_norm=float("nan")) == B.SR_ERR_ARG
    assert step([t], norm=nrm + 2, max_norm=1.0) == B.SR_ERR_ALIGN


def test_adamw_null_and_alignment_errors():
    assert step([tensor(p=None)]) == B.SR_ERR_NULL
    assert step([tensor(v=None)]) == B.SR_ERR_NULL
    t = tensor()
    assert step([tensor(g=t.g + 1)]) == B.SR_ERR_ALIGN
    assert step([tensor(m=t.m + 2)], flags=B.SR_FLAG_FP32_MOMENTS) == B.SR_ERR_ALIGN
    L = B.lib()
    h = B.SrHyper(1e-3, 0.9, 0.95, 1e-8, 0.1)
    assert L.sr_adamw_step(None, 1, C.byref(h), 1, 0, 0, None, 0.0, None) == B.SR_ERR_NULL
    arr = (B.SrTensor * 1)(t)
    assert L.sr_adamw_step(arr, 1, None, 1, 0, 0, None, 0.0, None) == B.SR_ERR_NULL
    # a bad entry anywhere in the list rejects the whole call
    assert step([tensor(), tensor(), tensor(g=None)]) == B.SR_ERR_NULL


def test_adamw_empty_inputs_are_no_ops():
    assert step([]) == B.SR_OK
    assert step([tensor(numel=0, p=None, g=None, m=None, v=None)]) == B.SR_OK


def test_cast_argument_errors():
    L = B.lib()
    assert L.sr_cast_f32_bf16(None, None, 0, 0, 1, 0, None) == B.SR_OK
    assert L.sr_cast_f32_bf16(None, buf(16), 8, 0, 1, 0, None) == B.SR_ERR_NULL
    assert L.sr_cast_f32_bf16(buf(32), None, 8, 0, 1, 0, None) == B.SR_ERR_NULL
    assert L.sr_cast_f32_bf16(buf(32, 2), buf(16), 4, 0, 1, 0, None) == B.SR_ERR_ALIGN
    assert L.sr_cast_f32_bf16(buf(32), buf(16, 1), 4, 0, 1, 0, None) == B.SR_ERR_ALIGN


def test_fp8_cast_argument_errors():
    L = B.lib()
    assert L.sr_cast_f32_fp8(None, None, 0, B.SR_FP8_E4M3, 0, 1, 0, None) == B.SR_OK
    assert L.sr_cast_f32_fp8(buf(32), buf(8), 8, 2, 0, 1, 0, None) == B.SR_ERR_ARG          # unknown format
    assert L.sr_cast_f32_fp8(None, buf(8), 8, B.SR_FP8_E5M2, 0, 1, 0, None) == B.SR_ERR_NULL
    assert L.sr_cast_f32_fp8(buf(32), None, 8, B.SR_FP8_E5M2, 0, 1, 0, None) == B.SR_ERR_NULL
    assert L.sr_cast_f32_fp8(buf(32, 2), buf(8), 4, B.SR_FP8_E4M3, 0, 1, 0, None) == B.SR_ERR_ALIGN
    assert L.sr_cast_f32_fp8(buf(32), buf(8), (1 << 61) + 1, B.SR_FP8_E4M3, 0, 1, 0, None) == B.SR_ERR_ARG


def test_norm_argument_errors():
    L = B.lib()
    t = tensor(numel=100000)
    arr = (B.SrTensor * 1)(t)
    out, ws = buf(4), buf(4096)
    assert L.grad_global_norm(arr, 1, None, ws, 4096, None) == B.SR_ERR_NULL
    assert L.grad_global_norm(None, 1, out, ws, 4096, None) == B.SR_ERR_NULL
    assert L.grad_global_norm(arr, 1, out, None, 4096, None) == B.SR_ERR_WORKSPACE
    assert L.grad_global_norm(arr, 1, out, ws, 8, None) == B.SR_ERR_WORKSPACE       # 2 chunks need 16 bytes
    assert L.grad_global_norm(arr, 1, out, ws + 4, 4096, None) == B.SR_ERR_WORKSPACE
    assert L.grad_global_norm(arr, 1, out + 2, ws, 4096, None) == B.SR_ERR_ALIGN
    arr[0].g = None
    assert L.grad_global_norm(arr, 1, out, ws, 4096, None) == B.SR_ERR_NULL


def test_sum_of_squares_argument_errors():
    L = B.lib()
    arr = (B.SrTensor * 1)(tensor(numel=100000))
    ws = buf(4096)
    assert L.grad_sum_of_squares(arr, 1, None, ws, 4096, None) == B.SR_ERR_NULL
    assert L.grad_sum_of_squares(arr, 1, buf(16, 4), ws, 4096, None) == B.SR_ERR_ALIGN
    assert L.grad_sum_of_squares(arr, 1, buf(16), None, 0, None) == B.SR_ERR_WORKSPACE
    assert L.grad_sum_of_squares(arr, 1, buf(16), ws, 8, None) == B.SR_ERR_WORKSPACE


def test_binding_rejects_host_tensors_and_wrong_dtypes():
    x = torch.zeros(8, dtype=torch.float32)
    y = torch.zeros(8, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        B.sr_cast_f32_bf16(x, y, 0, 1)
    with pytest.raises(ValueError):
        B.TensorList([y], [y], [y], [y])


def test_accumulate_argument_errors():
    L = B.lib()
    a = B.SrAccum()
    a.acc, a.grad, a.numel, a.elem_offset, a.tensor_id, a.reserved = buf(2 * 100000), buf(2 * 100000), 100000, 0, 0, 0
    arr = (B.SrAccum * 1)(a)
    out, ws = buf(4), buf(4096)

    def call(arr=arr, n=1, scale=1.0, flags=0, out=None, ws=None, wsb=0):
        return L.sr_grad_accumulate(arr, n, scale, 1, 0, flags, out, ws, wsb, None)
    assert call(arr=None) == B.SR_ERR_NULL
    assert call(flags=4) == B.SR_ERR_ARG
    assert call(scale=float("nan")) == B.SR_ERR_ARG
    assert call(out=out + 2, ws=ws, wsb=4096) == B.SR_ERR_ALIGN
    assert call(out=out, ws=None, wsb=4096) == B.SR_ERR_WORKSPACE
    assert call(out=out, ws=ws, wsb=8) == B.SR_ERR_WORKSPACE            # 196 chunks need 1568 bytes
    assert call(out=out, ws=ws + 4, wsb=4096) == B.SR_ERR_WORKSPACE
    arr[0].reserved = 1
    assert call() == B.SR_ERR_ARG
    arr[0].reserved = 0
    arr[0].grad = None
    assert call() == B.SR_ERR_NULL
    arr[0].grad = a.grad + 1
    assert call() == B.SR_ERR_ALIGN
    arr[0].grad = a.grad
    arr[0].elem_offset = 2 ** 64 - 5
    assert call() == B.SR_ERR_ARG
    assert call(n=0) == B.SR_OK
    assert L.sr_accumulate_workspace_bytes(3, 10 ** 9) >= 8 * (10 ** 9 // 512 + 3)


def test_accumulate_workspace_bound_covers_ragged_tensors_at_odd_offsets():
    """Many tensors just under a chunk, each starting mid-block in the counter, span two chunks
    each: the documented bound must cover the partial sums they need (one per chunk of 512
    elements, counted from the counter block that holds the tensor's first element), and on a GPU
    box a workspace of exactly that size must be accepted."""
    L = B.lib()
    n, numel, off = 177, 506, 7
    blocks = ((off + numel - 1) >> 3) - (off >> 3) + 1
    chunks = n * ((blocks + 63) // 64)
    assert chunks == 2 * n
    need = L.sr_accumulate_workspace_bytes(n, n * numel)
    assert need >= 8 * chunks
    if not HAVE_GPU:
        return
    arr = (B.SrAccum * n)()
    for i in range(n):
        arr[i].acc, arr[i].grad, arr[i].numel = buf(2 * 512), buf(2 * 512), numel
        arr[i].elem_offset, arr[i].tensor_id, arr[i].reserved = off, i, 0
    out, ws = buf(4), buf(need)
    assert L.sr_grad_accumulate(arr, n, 1.0, 1, 0, 0, out, ws, need, None) == B.SR_OK
    torch.cuda.synchronize()
    assert L.sr_grad_accumulate(arr, n, 1.0, 1, 0, 0, out, ws, 8 * chunks - 8, None) == B.SR_ERR_WORKSPACE


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No CPU fallback anywhere: when the built library is not there, the binding raises and says
    how to build it; nothing else is tried."""
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libsradamw.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.lib()
    src = open(os.path.join(ROOT, "paper_2502_20566_amd", "binding.py")).read()
    assert "oracle" not in src                              # the product path never reaches for the checker
