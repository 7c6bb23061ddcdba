"""ctypes front end of the CPU oracle (oracle/sr_oracle.c).

TEST INFRASTRUCTURE: only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import this module.  It shares no code with
the HIP library and imports nothing from the product package.

BF16 data are numpy uint16 arrays holding the bit patterns; FP32 data are
numpy float32 arrays.  All arrays must be C-contiguous.
"""
import ctypes as C

import numpy as np

from . import build as _build

FLAG_FP32_MOMENTS = 1
FLAG_RNE_MOMENTS = 2
FLAG_RNE_PARAMS = 4
FLAG_MASTER_FP32 = 8
FLAG_KAHAN = 16
FLAG_EPS_IN_ROOT = 32
FLAG_DIV_BIAS = 64
FLAG_FP8_MOMENTS = 128
FLAG_SKIP_NONFINITE_NORM = 256
FLAG_FP8_PARAMS = 512

STREAM_PARAM, STREAM_M, STREAM_V, STREAM_CAST, STREAM_ACC = 0, 1, 2, 3, 4
ACC_RNE = 1
ACC_FIRST = 2


class Scalars(C.Structure):
    _fields_ = [(n, C.c_float) for n in
                ("beta1", "beta2", "omb1", "omb2", "rbc1", "rbc2", "lr", "eps", "lw", "clip",
                 "bc1", "bc2")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        u16p, u32p, f32p = (C.POINTER(C.c_uint16), C.POINTER(C.c_uint32), C.POINTER(C.c_float))
        L.ref_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.ref_philox4x32_10.restype = None
        L.ref_r16.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint32]
        L.ref_r16.restype = C.c_uint32
        L.ref_r16_many.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64,
                                   C.c_uint32, u16p]
        L.ref_r16_many.restype = None
        L.ref_sr_round.argtypes = [C.c_float, C.c_uint32]
        L.ref_sr_round.restype = C.c_uint16
        L.ref_rne_round.argtypes = [C.c_float]
        L.ref_rne_round.restype = C.c_uint16
        L.ref_sr_round_many.argtypes = [f32p, u32p, C.c_uint64, u16p]
        L.ref_sr_round_many.restype = None
        L.ref_sr_round_all_draws.argtypes = [f32p, u16p]
        L.ref_sr_round_all_draws.restype = None
        L.ref_sr_cast_f32_bf16.argtypes = [f32p, u16p, C.c_uint64, C.c_uint64, C.c_uint32,
                                           C.c_uint32, C.c_uint64, C.c_int]
        L.ref_sr_cast_f32_bf16.restype = None
        L.ref_fp8_decode.argtypes = [C.c_uint32, C.c_int]
        L.ref_fp8_decode.restype = C.c_double
        L.ref_r32.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint32]
        L.ref_r32.restype = C.c_uint32
        L.ref_sr_round_fp8.argtypes = [C.c_float, C.c_uint32, C.c_int]
        L.ref_sr_round_fp8.restype = C.c_uint8
        L.ref_sr_cast_f32_fp8.argtypes = [f32p, C.POINTER(C.c_uint8), C.c_uint64, C.c_int, C.c_uint64,
                                          C.c_uint32, C.c_uint32, C.c_uint64, C.c_int]
        L.ref_sr_cast_f32_fp8.restype = None
        L.ref_adamw_scalars.argtypes = [C.c_float] * 5 + [C.c_uint32, f32p, C.c_float,
                                                          C.POINTER(Scalars)]
        L.ref_adamw_scalars.restype = None
        L.ref_adamw_unrounded.argtypes = [u16p, u16p, C.c_void_p, C.c_void_p, C.c_uint64,
                                          C.POINTER(Scalars), C.c_uint32, f32p, f32p, f32p]
        L.ref_adamw_unrounded.restype = None
        L.ref_sr_adamw_tensor.argtypes = [u16p, u16p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_uint64,
                                          C.c_uint32, C.c_uint64, C.POINTER(Scalars),
                                          C.c_uint32, C.c_uint64, C.c_uint32, C.c_int]
        L.ref_sr_adamw_tensor.restype = None
        u8p = C.POINTER(C.c_uint8)
        L.ref_sr_adamw_tensor_fp8m.argtypes = [u16p, u16p, u8p, u8p, C.c_uint64, C.c_uint32, C.c_uint64,
                                               C.POINTER(Scalars), C.c_uint32, C.c_uint64, C.c_uint32,
                                               C.c_int, C.c_int, C.c_int]
        L.ref_sr_adamw_tensor_fp8m.restype = None
        L.ref_sr_adamw_tensor_fp8p.argtypes = [u8p, u16p, u16p, u16p, u8p, u8p, C.c_uint64, C.c_uint32, C.c_uint64,
                                               C.POINTER(Scalars), C.c_uint32, C.c_uint64, C.c_uint32,
                                               C.c_int, C.c_int, C.c_int, C.c_int]
        L.ref_sr_adamw_tensor_fp8p.restype = None
        L.ref_adamw_unrounded_fp8m.argtypes = [u16p, u16p, u8p, u8p, C.c_uint64, C.POINTER(Scalars),
                                               C.c_uint32, C.c_int, C.c_int, f32p, f32p, f32p]
        L.ref_adamw_unrounded_fp8m.restype = None
        L.ref_grad_accumulate.argtypes = [u16p, u16p, C.c_uint64, C.c_float, C.c_uint32, C.c_uint64,
                                          C.c_uint32, C.c_uint64, C.c_uint32, C.c_int]
        L.ref_grad_accumulate.restype = None
        L.ref_grad_global_norm.argtypes = [C.POINTER(u16p), C.POINTER(C.c_uint64), C.c_uint32]
        L.ref_grad_global_norm.restype = C.c_float
        L.ref_max_threads.argtypes = []
        L.ref_max_threads.restype = C.c_int
        _lib = L
    return _lib


def _u16(a):
    assert a.dtype == np.uint16 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_uint16))


def _f32(a):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _u32(a):
    assert a.dtype == np.uint32 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_uint32))


# ------------------------------------------------------------------ plumbing

def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact decode of BF16 bit patterns (uint16) to float32 (format definition)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def max_threads() -> int:
    return int(lib().ref_max_threads())


# ----------------------------------------------------------------------- RNG

def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().ref_philox4x32_10(_u32(c), _u32(k), _u32(out))
    return out


def r16(seed, step, tensor_id, i, stream):
    return int(lib().ref_r16(seed, step, tensor_id, i, stream))


def r16_many(seed, step, tensor_id, i0, n, stream) -> np.ndarray:
    out = np.empty(n, dtype=np.uint16)
    lib().ref_r16_many(seed, step, tensor_id, i0, n, stream, _u16(out))
    return out


# ------------------------------------------------------------------ rounding

def sr_round(y, r):
    return int(lib().ref_sr_round(C.c_float(float(y)), int(r)))


def rne_round(y):
    return int(lib().ref_rne_round(C.c_float(float(y))))


def sr_round_many(y: np.ndarray, r: np.ndarray) -> np.ndarray:
    y = np.ascontiguousarray(y, dtype=np.float32)
    r = np.ascontiguousarray(r, dtype=np.uint32)
    out = np.empty(y.shape, dtype=np.uint16)
    lib().ref_sr_round_many(_f32(y), _u32(r), y.size, _u16(out))
    return out


def sr_round_all_draws(y_bits: int) -> np.ndarray:
    """Q_SR of the binary32 value with encoding `y_bits` for every draw 0..65535."""
    y = np.array([y_bits], dtype=np.uint32).view(np.float32)
    out = np.empty(65536, dtype=np.uint16)
    lib().ref_sr_round_all_draws(_f32(y), _u16(out))
    return out


def sr_cast_f32_bf16(src: np.ndarray, seed, step, tensor_id, elem_offset=0, nthreads=0):
    src = np.ascontiguousarray(src, dtype=np.float32)
    dst = np.empty(src.shape, dtype=np.uint16)
    lib().ref_sr_cast_f32_bf16(_f32(src), _u16(dst), src.size, seed, step, tensor_id,
                               elem_offset, nthreads)
    return dst


# ------------------------------------------------------ 8-bit formats (extension)

E4M3, E5M2 = 0, 1


def fp8_decode(code: int, fmt: int) -> float:
    return float(lib().ref_fp8_decode(code, fmt))


def r32(seed, step, tensor_id, i, stream) -> int:
    return int(lib().ref_r32(seed, step, tensor_id, i, stream))


def sr_round_fp8(y, r, fmt: int) -> int:
    """One value; y is converted to binary32 first (a NaN keeps its sign, not its payload)."""
    return int(lib().ref_sr_round_fp8(np.float32(y), r, fmt))


def sr_cast_f32_fp8(src: np.ndarray, fmt: int, seed, step, tensor_id, elem_offset=0, nthreads=0):
    src = np.ascontiguousarray(src, dtype=np.float32)
    dst = np.empty(src.shape, dtype=np.uint8)
    lib().ref_sr_cast_f32_fp8(_f32(src), dst.ctypes.data_as(C.POINTER(C.c_uint8)), src.size, fmt,
                              seed, step, tensor_id, elem_offset, nthreads)
    return dst


# --------------------------------------------------------------------- AdamW

def adamw_scalars(lr, beta1, beta2, eps, weight_decay, step, norm=None, max_norm=0.0) -> Scalars:
    s = Scalars()
    if norm is None:
        nptr = None
    else:
        nv = C.c_float(float(norm))
        nptr = C.pointer(nv)
    lib().ref_adamw_scalars(lr, beta1, beta2, eps, weight_decay, step, nptr, max_norm, C.byref(s))
    return s


def _moment_ptr(a, flags):
    if flags & FLAG_FP32_MOMENTS:
        assert a.dtype == np.float32 and a.flags.c_contiguous
    else:
        assert a.dtype == np.uint16 and a.flags.c_contiguous
    return a.ctypes.data_as(C.c_void_p)


def adamw_unrounded(p, g, m, v, scalars: Scalars, flags=0):
    n = p.size
    y = np.empty(n, np.float32)
    m1 = np.empty(n, np.float32)
    v1 = np.empty(n, np.float32)
    lib().ref_adamw_unrounded(_u16(p), _u16(g), _moment_ptr(m, flags), _moment_ptr(v, flags), n,
                              C.byref(scalars), flags, _f32(y), _f32(m1), _f32(v1))
    return y, m1, v1


def sr_adamw_tensor(p, g, m, v, tensor_id, scalars: Scalars, step, seed, flags=0,
                    elem_offset=0, nthreads=0, aux=None):
    """One tensor, in place over p, m, v (numpy arrays) and aux (binary32 master parameters with
    FLAG_MASTER_FP32, BF16 compensation bits with FLAG_KAHAN)."""
    assert p.size == g.size == m.size == v.size
    aptr = None
    if flags & FLAG_MASTER_FP32:
        assert flags & FLAG_FP32_MOMENTS
        assert aux is not None and aux.dtype == np.float32 and aux.flags.c_contiguous and aux.size == p.size
        aptr = aux.ctypes.data_as(C.c_void_p)
    elif flags & FLAG_KAHAN:
        assert not (flags & FLAG_FP32_MOMENTS)
        assert aux is not None and aux.dtype == np.uint16 and aux.flags.c_contiguous and aux.size == p.size
        aptr = aux.ctypes.data_as(C.c_void_p)
    lib().ref_sr_adamw_tensor(_u16(p), _u16(g), _moment_ptr(m, flags), _moment_ptr(v, flags), aptr,
                              p.size, tensor_id, elem_offset, C.byref(scalars), step, seed,
                              flags, nthreads)


def _u8(a):
    assert a.dtype == np.uint8 and a.flags.c_contiguous
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def sr_adamw_tensor_fp8m(p, g, m8, v8, tensor_id, scalars: Scalars, step, seed, m_exp, v_exp, flags=0,
                         elem_offset=0, nthreads=0):
    """One tensor with 8-bit moments (m8: E4M3 codes of m * 2^m_exp, v8: E5M2 codes of v * 2^v_exp),
    in place over p, m8, v8."""
    assert p.size == g.size == m8.size == v8.size and abs(m_exp) <= 100 and abs(v_exp) <= 100
    lib().ref_sr_adamw_tensor_fp8m(_u16(p), _u16(g), _u8(m8), _u8(v8), p.size, tensor_id, elem_offset,
                                   C.byref(scalars), step, seed, flags, m_exp, v_exp, nthreads)


def sr_adamw_tensor_fp8p(p8, g, m, v, tensor_id, scalars: Scalars, step, seed, p_exp, flags=0,
                         m_exp=0, v_exp=0, elem_offset=0, nthreads=0):
    """One tensor with the parameter held as E4M3 codes p8 (of p * 2^p_exp), in place over p8, m, v.
    m, v are BF16 bit patterns (uint16), or 8-bit codes (uint8: E4M3 m, E5M2 v, with m_exp, v_exp)."""
    assert p8.dtype == np.uint8 and p8.size == g.size == m.size == v.size
    assert abs(p_exp) <= 100 and abs(m_exp) <= 100 and abs(v_exp) <= 100
    if m.dtype == np.uint8:
        lib().ref_sr_adamw_tensor_fp8p(_u8(p8), _u16(g), None, None, _u8(m), _u8(v), p8.size, tensor_id, elem_offset,
                                       C.byref(scalars), step, seed, flags, p_exp, m_exp, v_exp, nthreads)
    else:
        lib().ref_sr_adamw_tensor_fp8p(_u8(p8), _u16(g), _u16(m), _u16(v), None, None, p8.size, tensor_id, elem_offset,
                                       C.byref(scalars), step, seed, flags, p_exp, 0, 0, nthreads)


def adamw_unrounded_fp8m(p, g, m8, v8, scalars: Scalars, m_exp, v_exp, flags=0):
    n = p.size
    y, m1, v1 = np.empty(n, np.float32), np.empty(n, np.float32), np.empty(n, np.float32)
    lib().ref_adamw_unrounded_fp8m(_u16(p), _u16(g), _u8(m8), _u8(v8), n, C.byref(scalars), flags,
                                   m_exp, v_exp, _f32(y), _f32(m1), _f32(v1))
    return y, m1, v1


def sr_adamw_step(tensors, hyper, step, seed, flags=0, norm=None, max_norm=0.0, nthreads=0):
    """Multi-tensor step: `tensors` is a list of dicts with numpy arrays p, g, m, v and
    optional tensor_id (default: list index) and elem_offset (default 0).
    hyper = dict(lr, beta1, beta2, eps, weight_decay)."""
    s = adamw_scalars(hyper["lr"], hyper["beta1"], hyper["beta2"], hyper["eps"],
                      hyper["weight_decay"], step, norm, max_norm)
    if flags & FLAG_SKIP_NONFINITE_NORM:
        # guard of a clipped step: a NaN or infinite gradient norm leaves every tensor as it is
        if norm is not None and not np.isfinite(np.float32(norm)):
            return s
        flags &= ~FLAG_SKIP_NONFINITE_NORM
    for idx, t in enumerate(tensors):
        if flags & FLAG_FP8_PARAMS:
            sr_adamw_tensor_fp8p(t["p"], t["g"], t["m"], t["v"], t.get("tensor_id", idx), s, step, seed, t["p_exp"],
                                 flags & ~(FLAG_FP8_PARAMS | FLAG_FP8_MOMENTS), t.get("m_exp", 0), t.get("v_exp", 0),
                                 t.get("elem_offset", 0), nthreads)
        elif flags & FLAG_FP8_MOMENTS:
            sr_adamw_tensor_fp8m(t["p"], t["g"], t["m"], t["v"], t.get("tensor_id", idx), s, step, seed,
                                 t["m_exp"], t["v_exp"], flags & ~FLAG_FP8_MOMENTS, t.get("elem_offset", 0), nthreads)
        else:
            sr_adamw_tensor(t["p"], t["g"], t["m"], t["v"], t.get("tensor_id", idx), s, step, seed,
                            flags, t.get("elem_offset", 0), nthreads, aux=t.get("aux"))
    return s


def grad_accumulate(acc, g, scale, micro_step, seed, tensor_id=0, elem_offset=0, flags=0, nthreads=0):
    """acc <- Q(acc + scale*g) in place (numpy uint16 BF16 bit patterns)."""
    assert acc.size == g.size
    lib().ref_grad_accumulate(_u16(acc), _u16(g), acc.size, scale, micro_step, seed, tensor_id,
                              elem_offset, flags, nthreads)


def grad_global_norm(grads) -> float:
    n = len(grads)
    ptrs = (C.POINTER(C.c_uint16) * max(n, 1))()
    sizes = (C.c_uint64 * max(n, 1))()
    for i, g in enumerate(grads):
        ptrs[i] = _u16(g)
        sizes[i] = g.size
    return float(lib().ref_grad_global_norm(ptrs, sizes, n))
