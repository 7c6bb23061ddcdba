"""ctypes binding of libsradamw.so (C ABI in include/sradamw.h).

Argument marshalling only: every step of the update runs in the HIP kernels.
PyTorch supplies device memory and streams.  There is no CPU fallback: if the
library is missing or a call fails, an exception is raised.
"""
import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import torch  # imported before the library so that one HIP runtime serves both

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsradamw.so")

SR_OK = 0
SR_ERR_NULL, SR_ERR_ARG, SR_ERR_WORKSPACE, SR_ERR_ALIGN, SR_ERR_HIP, SR_ERR_SIZE = -1, -2, -3, -4, -5, -6
SR_FLAG_FP32_MOMENTS = 1
SR_FLAG_RNE_MOMENTS = 2
SR_FLAG_RNE_PARAMS = 4
SR_FLAG_MASTER_FP32 = 8
SR_FLAG_KAHAN = 16
SR_FLAG_EPS_IN_ROOT = 32
SR_FLAG_DIV_BIAS = 64
SR_FLAG_FP8_MOMENTS = 128
SR_FLAG_SKIP_NONFINITE_NORM = 256
SR_FLAG_FP8_PARAMS = 512

SR_DEBUG_LAUNCH_LIMIT, SR_DEBUG_FP8_INTEGER, SR_DEBUG_RESIDENT_WAVES = 0, 1, 2

SR_ACC_RNE = 1
SR_ACC_FIRST = 2

SR_FP8_E4M3, SR_FP8_E5M2 = 0, 1

EXPORTS = ("sr_cast_f32_bf16", "sr_cast_f32_fp8", "grad_global_norm", "grad_global_norm_static", "grad_sum_of_squares", "sr_adamw_step", "sr_workspace_bytes",
           "sr_grad_accumulate", "sr_accumulate_workspace_bytes", "sr_stream_probe", "sr_stream_probe_fp8m",
           "sr_strerror", "sr_last_hip_error", "sr_version", "sr_debug_set")


class SrTensor(C.Structure):
    _fields_ = [("p", C.c_void_p), ("g", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("aux", C.c_void_p), ("numel", C.c_uint64), ("elem_offset", C.c_uint64),
                ("tensor_id", C.c_uint32), ("m_exp", C.c_int8), ("v_exp", C.c_int8), ("p_exp", C.c_int8), ("reserved", C.c_uint8)]


class SrAccum(C.Structure):
    _fields_ = [("acc", C.c_void_p), ("grad", C.c_void_p), ("numel", C.c_uint64),
                ("elem_offset", C.c_uint64), ("tensor_id", C.c_uint32), ("reserved", C.c_uint32)]


class SrHyper(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float)]


class SrError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().sr_strerror(code).decode()
        if code == SR_ERR_HIP:
            msg += f" [hipError {lib().sr_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({code})")


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2502_20566_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -c 'import __graft_entry__ as g; g.build()'`; "
                               "there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        L.sr_cast_f32_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint32,
                                       C.c_uint32, C.c_void_p]
        L.sr_cast_f32_bf16.restype = C.c_int
        L.sr_cast_f32_fp8.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32,
                                      C.c_uint32, C.c_void_p]
        L.sr_cast_f32_fp8.restype = C.c_int
        L.grad_global_norm.argtypes = [C.POINTER(SrTensor), C.c_uint32, C.c_void_p, C.c_void_p,
                                       C.c_uint64, C.c_void_p]
        L.grad_global_norm.restype = C.c_int
        L.grad_global_norm_static.argtypes = [C.POINTER(SrTensor), C.c_uint32, C.c_void_p, C.c_void_p]
        L.grad_global_norm_static.restype = C.c_int
        L.grad_sum_of_squares.argtypes = L.grad_global_norm.argtypes
        L.grad_sum_of_squares.restype = C.c_int
        L.sr_adamw_step.argtypes = [C.POINTER(SrTensor), C.c_uint32, C.POINTER(SrHyper), C.c_uint32,
                                    C.c_uint64, C.c_uint32, C.c_void_p, C.c_float, C.c_void_p]
        L.sr_adamw_step.restype = C.c_int
        L.sr_grad_accumulate.argtypes = [C.POINTER(SrAccum), C.c_uint32, C.c_float, C.c_uint32, C.c_uint64,
                                         C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        L.sr_grad_accumulate.restype = C.c_int
        L.sr_accumulate_workspace_bytes.argtypes = [C.c_uint32, C.c_uint64]
        L.sr_accumulate_workspace_bytes.restype = C.c_uint64
        L.sr_stream_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        L.sr_stream_probe.restype = C.c_int
        L.sr_stream_probe_fp8m.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p]
        L.sr_stream_probe_fp8m.restype = C.c_int
        L.sr_workspace_bytes.argtypes = [C.c_uint32, C.c_uint64]
        L.sr_workspace_bytes.restype = C.c_uint64
        L.sr_strerror.argtypes = [C.c_int]
        L.sr_strerror.restype = C.c_char_p
        L.sr_last_hip_error.argtypes = []
        L.sr_last_hip_error.restype = C.c_int
        L.sr_debug_set.argtypes = [C.c_uint32, C.c_uint32]
        L.sr_debug_set.restype = None
        L.sr_version.argtypes = []
        L.sr_version.restype = C.c_int
        _lib = L
    return _lib


def _stream_handle(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _check_dev(t: torch.Tensor, dtype, name: str):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if t.device.index != torch.cuda.current_device():
        # kernels are launched on the current device's stream with plain pointers
        raise ValueError(f"{name} lives on {t.device}, the current device is cuda:{torch.cuda.current_device()}")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


class TensorList:
    """A marshalled multi-tensor list (host array of sr_tensor_t).  Build once, reuse every
    step; it keeps the torch tensors alive."""

    def __init__(self, params: Sequence[torch.Tensor], grads: Sequence[torch.Tensor],
                 ms: Sequence[torch.Tensor], vs: Sequence[torch.Tensor], fp32_moments: bool = False,
                 tensor_ids: Optional[Sequence[int]] = None,
                 elem_offsets: Optional[Sequence[int]] = None,
                 aux: Optional[Sequence[torch.Tensor]] = None,
                 fp8_exponents: Optional[Sequence[Tuple[int, int]]] = None,
                 fp8_param_exponents: Optional[Sequence[int]] = None):
        """aux: per-tensor auxiliary arrays for the comparison strategies -- float32 master
        parameters (SR_FLAG_MASTER_FP32) or bfloat16 Kahan compensation (SR_FLAG_KAHAN).
        fp8_exponents: per-tensor (m_exp, v_exp) for SR_FLAG_FP8_MOMENTS; ms and vs are then one
        byte per element (uint8 or a torch float8 dtype).
        fp8_param_exponents: per-tensor p_exp for SR_FLAG_FP8_PARAMS; params are then one byte per
        element too."""
        n = len(params)
        if not (len(grads) == len(ms) == len(vs) == n):
            raise ValueError("params, grads, ms, vs must have the same length")
        mdt = torch.float32 if fp32_moments else torch.bfloat16
        if fp8_exponents is not None:
            if fp32_moments or len(fp8_exponents) != n:
                raise ValueError("fp8_exponents: one (m_exp, v_exp) per tensor, not with fp32_moments")
            mdt = None                                        # any one-byte dtype
        self.fp32_moments = fp32_moments
        self.fp8_moments = fp8_exponents is not None
        self.fp8_params = fp8_param_exponents is not None
        if self.fp8_params and (fp32_moments or aux is not None or len(fp8_param_exponents) != n):
            raise ValueError("fp8_param_exponents: one p_exp per tensor, not with fp32_moments or aux tensors")
        self.n = n
        self.array = (SrTensor * max(n, 1))()
        self.keep = (list(params), list(grads), list(ms), list(vs), None if aux is None else list(aux))
        self.aux_dtype = None if aux is None else aux[0].dtype if len(aux) else None
        if aux is not None and len(aux) != n:
            raise ValueError("aux must have one entry per tensor")
        self.total_numel = 0
        for i in range(n):
            p, g, m, v = params[i], grads[i], ms[i], vs[i]
            if self.fp8_params and p.element_size() != 1:
                raise ValueError(f"params[{i}] must hold one byte per element")
            _check_dev(p, p.dtype if self.fp8_params else torch.bfloat16, f"params[{i}]")
            _check_dev(g, torch.bfloat16, f"grads[{i}]")
            for name, x in (("ms", m), ("vs", v)):
                if mdt is None and x.element_size() != 1:
                    raise ValueError(f"{name}[{i}] must hold one byte per element")
                _check_dev(x, x.dtype if mdt is None else mdt, f"{name}[{i}]")
            if not (p.numel() == g.numel() == m.numel() == v.numel()):
                raise ValueError(f"tensor {i}: p, g, m, v differ in size")
            e = self.array[i]
            e.p, e.g, e.m, e.v = p.data_ptr(), g.data_ptr(), m.data_ptr(), v.data_ptr()
            e.aux = None
            if aux is not None:
                a = aux[i]
                if a.dtype not in (torch.float32, torch.bfloat16):
                    raise ValueError(f"aux[{i}] must be float32 or bfloat16")
                _check_dev(a, a.dtype, f"aux[{i}]")
                if a.numel() != p.numel() or a.dtype != aux[0].dtype:
                    raise ValueError(f"aux[{i}] differs in size or dtype")
                e.aux = a.data_ptr()
            e.numel = p.numel()
            e.elem_offset = 0 if elem_offsets is None else int(elem_offsets[i])
            e.tensor_id = i if tensor_ids is None else int(tensor_ids[i])
            e.m_exp, e.v_exp, e.p_exp, e.reserved = 0, 0, 0, 0
            if self.fp8_params:
                if not -100 <= int(fp8_param_exponents[i]) <= 100:
                    raise ValueError("fp8 scale exponents must lie in [-100, 100]")
                e.p_exp = int(fp8_param_exponents[i])
            if fp8_exponents is not None:
                m_exp, v_exp = (int(x) for x in fp8_exponents[i])
                if not (-100 <= m_exp <= 100 and -100 <= v_exp <= 100):
                    raise ValueError("fp8 scale exponents must lie in [-100, 100]")
                e.m_exp, e.v_exp = m_exp, v_exp
            self.total_numel += p.numel()

    def workspace_bytes(self) -> int:
        return int(lib().sr_workspace_bytes(self.n, self.total_numel))


def sr_workspace_bytes(n_tensors: int, total_numel: int) -> int:
    return int(lib().sr_workspace_bytes(n_tensors, total_numel))


def sr_cast_f32_bf16(src: torch.Tensor, dst: torch.Tensor, seed: int, step: int, tensor_id: int = 0,
                     stream=None) -> None:
    _check_dev(src, torch.float32, "src")
    _check_dev(dst, torch.bfloat16, "dst")
    if src.numel() != dst.numel():
        raise ValueError("src and dst differ in size")
    rc = lib().sr_cast_f32_bf16(src.data_ptr(), dst.data_ptr(), src.numel(), seed, step, tensor_id,
                                _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "sr_cast_f32_bf16")


def sr_cast_f32_fp8(src: torch.Tensor, dst: torch.Tensor, fmt: int, seed: int, step: int, tensor_id: int = 0,
                    stream=None) -> None:
    """dst (uint8 or a torch float8 dtype, one byte per element) <- Q_SR(src) on the grid of
    SR_FP8_E4M3 or SR_FP8_E5M2."""
    _check_dev(src, torch.float32, "src")
    if not dst.is_cuda or not dst.is_contiguous() or dst.element_size() != 1:
        raise ValueError("dst must be a contiguous one-byte device tensor")
    if src.numel() != dst.numel():
        raise ValueError("src and dst differ in size")
    rc = lib().sr_cast_f32_fp8(src.data_ptr(), dst.data_ptr(), src.numel(), fmt, seed, step, tensor_id,
                               _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "sr_cast_f32_fp8")


def grad_global_norm(tl: TensorList, norm_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """norm_out: float32 device tensor with one element; workspace: device tensor (any dtype) of
    at least tl.workspace_bytes() bytes."""
    _check_dev(norm_out, torch.float32, "norm_out")
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")
    rc = lib().grad_global_norm(tl.array, tl.n, norm_out.data_ptr(), workspace.data_ptr(),
                                workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "grad_global_norm")


def grad_global_norm_static(tl: TensorList, norm_out: torch.Tensor, stream=None) -> None:
    """grad_global_norm with the library's static scratch instead of a workspace (allocates nothing)."""
    _check_dev(norm_out, torch.float32, "norm_out")
    rc = lib().grad_global_norm_static(tl.array, tl.n, norm_out.data_ptr(), _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "grad_global_norm_static")


def grad_sum_of_squares(tl: TensorList, sumsq_out: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """sumsq_out: float64 device tensor with one element (the sum of squares, not its root)."""
    _check_dev(sumsq_out, torch.float64, "sumsq_out")
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous device tensor")
    rc = lib().grad_sum_of_squares(tl.array, tl.n, sumsq_out.data_ptr(), workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "grad_sum_of_squares")


def sr_adamw_step(tl: TensorList, hyper: dict, step: int, seed: int, flags: int = 0,
                  grad_norm: Optional[torch.Tensor] = None, max_norm: float = 0.0, stream=None) -> None:
    """hyper = dict(lr, beta1, beta2, eps, weight_decay).  grad_norm: float32 device scalar from
    grad_global_norm, or None for no clipping."""
    if bool(flags & SR_FLAG_FP32_MOMENTS) != tl.fp32_moments:
        raise ValueError("SR_FLAG_FP32_MOMENTS does not match the moment dtype of the list")
    if bool(flags & SR_FLAG_FP8_MOMENTS) != tl.fp8_moments:
        raise ValueError("SR_FLAG_FP8_MOMENTS needs a list built with fp8_exponents (and only such a list)")
    if bool(flags & SR_FLAG_FP8_PARAMS) != tl.fp8_params:
        raise ValueError("SR_FLAG_FP8_PARAMS needs a list built with fp8_param_exponents (and only such a list)")
    if (flags & SR_FLAG_MASTER_FP32) and tl.n and tl.aux_dtype != torch.float32:
        raise ValueError("SR_FLAG_MASTER_FP32 needs float32 aux tensors in the list")
    if (flags & SR_FLAG_KAHAN) and tl.n and tl.aux_dtype != torch.bfloat16:
        raise ValueError("SR_FLAG_KAHAN needs bfloat16 aux tensors in the list")
    h = SrHyper(hyper["lr"], hyper["beta1"], hyper["beta2"], hyper["eps"], hyper["weight_decay"])
    nptr = None
    if grad_norm is not None:
        _check_dev(grad_norm, torch.float32, "grad_norm")
        nptr = grad_norm.data_ptr()
    rc = lib().sr_adamw_step(tl.array, tl.n, C.byref(h), step, seed, flags, nptr, max_norm,
                             _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "sr_adamw_step")


def sr_stream_probe_fp8m(p: torch.Tensor, g: torch.Tensor, m8: torch.Tensor, v8: torch.Tensor, stream=None) -> None:
    """6-read/4-write pass over BF16 p, g and one-byte m8, v8 that leaves the data unchanged (measurement aid)."""
    for name, t in (("p", p), ("g", g)):
        _check_dev(t, torch.bfloat16, name)
    for name, t in (("m8", m8), ("v8", v8)):
        if t.element_size() != 1:
            raise ValueError(f"{name} must hold one byte per element")
        _check_dev(t, t.dtype, name)
    if not (p.numel() == g.numel() == m8.numel() == v8.numel()):
        raise ValueError("p, g, m8, v8 differ in size")
    rc = lib().sr_stream_probe_fp8m(p.data_ptr(), g.data_ptr(), m8.data_ptr(), v8.data_ptr(), p.numel(),
                                    _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "sr_stream_probe_fp8m")


def sr_stream_probe(p: torch.Tensor, g: torch.Tensor, m: torch.Tensor, v: torch.Tensor, stream=None) -> None:
    """4-read/3-write pass over BF16 p, g, m, v that leaves the data unchanged (measurement aid)."""
    for name, t in (("p", p), ("g", g), ("m", m), ("v", v)):
        _check_dev(t, torch.bfloat16, name)
        if t.numel() != p.numel():
            raise ValueError("p, g, m, v differ in size")
    rc = lib().sr_stream_probe(p.data_ptr(), g.data_ptr(), m.data_ptr(), v.data_ptr(), p.numel(),
                               _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "sr_stream_probe")


class AccumList:
    """A marshalled list of (accumulator, micro-batch gradient) pairs for sr_grad_accumulate."""

    def __init__(self, accs: Sequence[torch.Tensor], grads: Sequence[torch.Tensor],
                 tensor_ids: Optional[Sequence[int]] = None, elem_offsets: Optional[Sequence[int]] = None):
        n = len(accs)
        if len(grads) != n:
            raise ValueError("accs and grads must have the same length")
        self.n = n
        self.array = (SrAccum * max(n, 1))()
        self.keep = (list(accs), list(grads))
        self.total_numel = 0
        for i in range(n):
            _check_dev(accs[i], torch.bfloat16, f"accs[{i}]")
            _check_dev(grads[i], torch.bfloat16, f"grads[{i}]")
            if accs[i].numel() != grads[i].numel():
                raise ValueError(f"pair {i} differs in size")
            e = self.array[i]
            e.acc, e.grad, e.numel = accs[i].data_ptr(), grads[i].data_ptr(), accs[i].numel()
            e.elem_offset = 0 if elem_offsets is None else int(elem_offsets[i])
            e.tensor_id = i if tensor_ids is None else int(tensor_ids[i])
            e.reserved = 0
            self.total_numel += accs[i].numel()

    def workspace_bytes(self) -> int:
        return int(lib().sr_accumulate_workspace_bytes(self.n, self.total_numel))


def sr_grad_accumulate(al: AccumList, scale: float, micro_step: int, seed: int, flags: int = 0,
                       norm_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                       stream=None) -> None:
    """acc <- Q(acc + scale*grad) for every pair; with norm_out (float32 device scalar) and a
    workspace of al.workspace_bytes() bytes also the global norm of the result."""
    nptr, wptr, wbytes = None, None, 0
    if norm_out is not None:
        _check_dev(norm_out, torch.float32, "norm_out")
        if workspace is None or not workspace.is_cuda or not workspace.is_contiguous():
            raise ValueError("a contiguous device workspace is needed with norm_out")
        nptr, wptr = norm_out.data_ptr(), workspace.data_ptr()
        wbytes = workspace.numel() * workspace.element_size()
    rc = lib().sr_grad_accumulate(al.array, al.n, scale, micro_step, seed, flags, nptr, wptr, wbytes,
                                  _stream_handle(stream))
    if rc != SR_OK:
        raise SrError(rc, "sr_grad_accumulate")
