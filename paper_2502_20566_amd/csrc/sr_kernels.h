// Kernels of the SR-AdamW update path for gfx950 (wave64): the fused multi-tensor update
// (Algorithm 1 lines 5-10 of arXiv 2502.20566 with stochastically rounded write-backs), the
// standalone SR casts (to BF16; to the OCP 8-bit formats as an extension), the BF16 gradient
// accumulation with SR, the two-pass global gradient norm, and a no-arithmetic traffic probe.
//
// Work decomposition shared by all kernels: a tensor is cut into 8-element blocks aligned to the
// RNG counter (block index = element index >> 3, so one Philox call serves one 128-bit BF16
// vector); a lane owns whole blocks; a workgroup owns one chunk of consecutive blocks of ONE
// tensor; the chunk -> tensor map is a small prefix table that travels in the kernel argument
// segment (scalar loads, no device-side table to upload or keep alive).
#pragma once
#include "sr_device.h"

namespace sr {

// Update and cast kernels run as single-wave workgroups with one block per lane: measured on
// MI355X, 64-lane workgroups stream the 4-read/3-write pattern about 10% faster than 256-lane
// ones (finer interleaving of the seven streams in time), and more blocks per lane are slower.
// Rows of 4 elements per lane in the cast kernels.  Measured on 6.66e9 elements: BF16 cast 6.06 /
// 6.10 / 7.04 ms with 1 / 2 / 4 rows; 8-bit cast (integer path) 6.07 / 5.64 / 5.64 ms.
#ifndef SR_TUNE_CAST_ITERS
#define SR_TUNE_CAST_ITERS 1
#endif
#ifndef SR_TUNE_FP8_ITERS
#define SR_TUNE_FP8_ITERS 2
#endif
#ifndef SR_TUNE_THREADS
#define SR_TUNE_THREADS 64
#endif
// Tensors per update launch: the descriptors and the chunk table travel by value in the kernel
// argument segment (22 KiB at 320).  Measured on MI355X with 56 / 160 / 320 per launch: the
// 148-tensor list 0.282 / 0.273 / 0.273 ms, the 292-tensor list 0.786 / 0.772 / 0.770 ms, the
// 388-tensor list equal within noise: every launch boundary drains and refills the chip.
#ifndef SR_TUNE_MAXBATCH
#define SR_TUNE_MAXBATCH 320
#endif
// Waves allowed to reside per CU, by kernel class (0 = as many as fit, 32): see occupancy_lds in
// the host code; LDS is granted in units of 1280 bytes, so the settings that differ are 32, 24
// (23-24 measured), 20, 18 (17-18 measured), 16, 14, 12, 11, 10, 9, 8.  Measured on MI355X,
// 6.66e9 elements, one process, arrays as allocated, waves per CU 32 / 24 / 20 / 18 / 16 / 14 / 12 / 11:
//   BF16 update (SR)    14.51 / 14.44 / 14.24 / 14.25 / 14.36 / 14.54 / 14.98 / 15.49 ms
//   same, moments to nearest 14.63 / 14.43 / 14.16 / 14.02 / 14.04 / 14.19 / 14.69 / 15.41 ms
//   same, no arithmetic 14.64 / 14.70 / 14.54 / 14.22 / 14.08 / 13.98 / 13.89 / 13.92 ms
//   Kahan (18 B/el)     19.81 / 19.90 / 19.38 / 18.89 / 18.61 / 18.39 / 18.23 / 18.27 ms
//   master (28 B/el)    28.83 / 28.87 / 28.73 / 28.63 / 28.50 / 28.50 / 28.52 / 28.54 ms
//   8-bit moments       11.87 / 12.03 / 12.34 / 12.63 / 12.97 / 13.55 / 14.23 / 14.60 ms   (no cap)
// and in earlier runs: binary32 moments (2.65e9 el) best at 14-16 (9.09 -> 8.96-8.99 ms); the
// BF16 cast (half a block per lane) and the accumulation lose from any cap (6.16 -> 6.93,
// 6.20 -> 6.47 ms at 20); the 8-bit cast gains a little at 24 (4.94 -> 4.84 ms).
// The update's arithmetic keeps the vector ALUs busy for nearly the whole kernel (VALUBusy 90-103%
// with SR on all three outputs, 86-91% with the moments to nearest, in two runs), so it needs
// 16-20 waves to overlap with the memory stream, while the bare stream is fastest at 11-12.
// A read-only stream does not care (7.32 ms for 8, 16 and 32 waves): it is the mix of reads and
// writes that loses bandwidth when more requests than needed are in flight.
#ifndef SR_TUNE_WAVES_BF16
#define SR_TUNE_WAVES_BF16 18
#endif
#ifndef SR_TUNE_WAVES_KAHAN
#define SR_TUNE_WAVES_KAHAN 12
#endif
#ifndef SR_TUNE_WAVES_FP32
#define SR_TUNE_WAVES_FP32 16
#endif
#ifndef SR_TUNE_WAVES_FP8M
#define SR_TUNE_WAVES_FP8M 0
#endif
#ifndef SR_TUNE_WAVES_CAST
#define SR_TUNE_WAVES_CAST 0
#endif
#ifndef SR_TUNE_WAVES_CAST8
#define SR_TUNE_WAVES_CAST8 24
#endif
#ifndef SR_TUNE_WAVES_ACC
#define SR_TUNE_WAVES_ACC 0
#endif
constexpr int kThreads = SR_TUNE_THREADS;   // lanes per workgroup of the update and cast kernels
constexpr int kMaxBatch = SR_TUNE_MAXBATCH; // tensors per update launch
// Norm, first pass: measured on MI355X, 512-lane workgroups with 16 blocks per lane and
// nontemporal loads read at 7.1 TB/s (the read-only ceiling); plain loads reach 6.1 TB/s.
constexpr int kNormThreads = 512;      // lanes per workgroup of the norm's first pass
constexpr int kNormMaxBatch = 400;     // tensors per norm launch
constexpr int kNormIters = 16;         // blocks per lane in the norm's first pass
constexpr int kNormChunkElems = kNormThreads * 8 * kNormIters;
constexpr int kFinalThreads = 1024;
// Gradient accumulation (2 reads, 1 write): measured 6.0 ms on 6.66e9 elements with single-wave
// workgroups and one block per lane, 6.1-7.1 ms for every larger geometry; with the norm each
// wave leaves one partial sum (8 bytes per 512 elements), folded by sumsq_reduce_kernel.
constexpr int kAccThreads = 64;        // lanes per workgroup of the gradient accumulation
constexpr int kAccIters = 1;           // blocks per lane (one partial sum of squares per chunk)
constexpr int kReduceThreads = 256;    // partial-sum folding: each workgroup adds kReduceFan partials
constexpr int kReduceFan = 4096;
constexpr uint32_t kReduceAbove = 16384;   // fold while more partials than this remain
constexpr int kAccChunkElems = kAccThreads * 8 * kAccIters;
constexpr int kAccMaxBatch = 320;      // tensors per accumulation launch

typedef uint32_t v4u __attribute__((ext_vector_type(4)));
// Vector accesses are declared with the alignment of the ELEMENT type (2 bytes for BF16 arrays, 4 for
// binary32 arrays): global memory on this target takes dwordx4/x2 accesses at any such address, so
// tensors that are views starting anywhere in a larger buffer keep the vector path.
typedef v4u v4u_a2 __attribute__((aligned(2)));
typedef v4u v4u_a4 __attribute__((aligned(4)));

// DESC_VEC: elem_offset % 8 == 0, blocks of the RNG counter start at element 0.  With 8-bit moments
// bits 8-15 and 16-23 hold the scale exponents of m and v (two's complement, |e| <= 100).
// With an 8-bit parameter bits 24-31 hold its scale exponent.
enum : uint32_t { DESC_VEC = 1u, DESC_MEXP_SHIFT = 8u, DESC_VEXP_SHIFT = 16u, DESC_PEXP_SHIFT = 24u };

struct TensorDesc {
    uint16_t* p;
    const uint16_t* g;
    void* m;
    void* v;
    void* aux;
    uint64_t numel;
    uint64_t elem_offset;
    uint32_t tensor_id;
    uint32_t flags;
};

struct StepScalars {
    float beta1, beta2, omb1, omb2, rbc1, rbc2, lr, eps, lw, max_norm;
    float bc1, bc2;                        // 1 - beta^t (used by the divide-by-bias-correction variant)
    const float* d_norm;
    uint32_t seed_lo, seed_hi, step, n_tensors;
    uint32_t variant;                      // VARIANT_* bits: wave-uniform choices of the arithmetic
    uint32_t skip_nonfinite;               // with clipping: leave everything unchanged when the norm is NaN or infinite
};
// VARIANT_FP8_INTEGER (test switch): every wave writes its 8-bit moments through the integer path.
enum : uint32_t { VARIANT_EPS_IN_ROOT = 1u, VARIANT_DIV_BIAS = 2u, VARIANT_FP8_INTEGER = 4u };

struct AdamwBatch {
    StepScalars s;
    uint32_t chunk_start[kMaxBatch + 1];   // first chunk of tensor i; [n_tensors] = total
    uint32_t pad_;
    TensorDesc t[kMaxBatch];
};
static_assert(sizeof(AdamwBatch) <= 32768, "kernel argument segment");

struct NormDesc { const uint16_t* g; uint64_t numel; };
struct NormBatch {
    uint32_t n_tensors;
    uint32_t partial_base;                 // index of this launch's first partial sum
    uint32_t chunk_start[kNormMaxBatch + 1];
    uint32_t pad_;
    NormDesc t[kNormMaxBatch];
};
static_assert(sizeof(NormBatch) <= 32768, "kernel argument segment");

struct AccDesc {
    uint16_t* acc;
    const uint16_t* g;
    uint64_t numel;
    uint64_t elem_offset;
    uint32_t tensor_id;
    uint32_t pad_;
};
enum : uint32_t { ACC_RNE = 1u, ACC_FIRST = 2u, ACC_NORM = 4u };
struct AccBatch {
    float scale;
    uint32_t seed_lo, seed_hi, micro_step, n_tensors, partial_base, mode, pad_;
    uint32_t chunk_start[kAccMaxBatch + 1];
    uint32_t pad2_;
    AccDesc t[kAccMaxBatch];
};
static_assert(sizeof(AccBatch) <= 32768, "kernel argument segment");

// ------------------------------------------------------------------ memory access helpers

// A = alignment of the array's element type in bytes (2 or 4).
template <bool NT, int A>
__device__ __forceinline__ v4u load_v4(const void* ptr)
{
    if (A == 2) {
        if (NT) return __builtin_nontemporal_load(reinterpret_cast<const v4u_a2*>(ptr));
        return *reinterpret_cast<const v4u_a2*>(ptr);
    }
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const v4u_a4*>(ptr));
    return *reinterpret_cast<const v4u_a4*>(ptr);
}
template <bool NT, int A>
__device__ __forceinline__ void store_v4(void* ptr, v4u x)
{
    if (A == 2) {
        if (NT) __builtin_nontemporal_store(x, reinterpret_cast<v4u_a2*>(ptr));
        else *reinterpret_cast<v4u_a2*>(ptr) = x;
    } else {
        if (NT) __builtin_nontemporal_store(x, reinterpret_cast<v4u_a4*>(ptr));
        else *reinterpret_cast<v4u_a4*>(ptr) = x;
    }
}

typedef uint32_t v2u __attribute__((ext_vector_type(2)));
typedef v2u v2u_a2 __attribute__((aligned(2)));
template <bool NT>
__device__ __forceinline__ v2u load_v2(const void* ptr)
{
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const v2u_a2*>(ptr));
    return *reinterpret_cast<const v2u_a2*>(ptr);
}
template <bool NT>
__device__ __forceinline__ void store_v2(void* ptr, v2u x)
{
    if (NT) __builtin_nontemporal_store(x, reinterpret_cast<v2u_a2*>(ptr));
    else *reinterpret_cast<v2u_a2*>(ptr) = x;
}

// Buffer accesses of the fast paths.  A workgroup describes its own span of each array (base =
// first byte of the chunk, wave-uniform, in scalar registers; size = the chunk's bytes) and every
// lane adds a small byte offset: measured on MI355X the 4-read/3-write stream runs 4% faster with
// buffer instructions than with global ones (14.7 vs 15.3 ms on 6.66e9 elements), and the hardware
// range check confines every such access to the chunk.  Cache policy: nt (streaming).
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
template <bool NT> __device__ __forceinline__ v4u buf_load16(rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, NT ? 2 : 0);
}
template <bool NT> __device__ __forceinline__ void buf_store16(rsrc_t r, uint32_t off, v4u x)
{
    __builtin_amdgcn_raw_buffer_store_b128(x, r, (int)off, 0, NT ? 2 : 0);
}
template <bool NT> __device__ __forceinline__ v2u buf_load8(rsrc_t r, uint32_t off)
{
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, NT ? 2 : 0);
}
template <bool NT> __device__ __forceinline__ void buf_store8(rsrc_t r, uint32_t off, v2u x)
{
    __builtin_amdgcn_raw_buffer_store_b64(x, r, (int)off, 0, NT ? 2 : 0);
}

// Descriptor of n_elems elements of type E starting at element first_elem of `base`.
template <typename E>
__device__ __forceinline__ rsrc_t chunk_rsrc(const void* base, int64_t first_elem, uint32_t n_elems)
{
    return make_rsrc(reinterpret_cast<const char*>(base) + first_elem * (int64_t)sizeof(E),
                     n_elems * (uint32_t)sizeof(E));
}

// True when the 8-element block starting at element l0 lies inside [0, numel).
__device__ __forceinline__ bool block_inside(int64_t l0, uint64_t numel)
{
    return l0 >= 0 && (uint64_t)l0 + 8 <= numel;
}

// Eight BF16 values starting at element l0 of `base` as four packed pairs.  `full`: the block lies
// inside the tensor (one vector access).  Otherwise element-wise, with zeros outside [0, numel).
template <bool NT>
__device__ __forceinline__ v4u load8_bf16(const uint16_t* base, int64_t l0, uint64_t numel, bool full)
{
    if (full) return load_v4<NT, 2>(base + l0);
    uint32_t h[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t l = l0 + j;
        h[j] = (l >= 0 && (uint64_t)l < numel) ? (uint32_t)base[l] : 0u;
    }
    v4u r;
    r.x = h[0] | (h[1] << 16); r.y = h[2] | (h[3] << 16);
    r.z = h[4] | (h[5] << 16); r.w = h[6] | (h[7] << 16);
    return r;
}

template <bool NT>
__device__ __forceinline__ void store8_bf16(uint16_t* base, int64_t l0, uint64_t numel, bool full, v4u x)
{
    if (full) { store_v4<NT, 2>(base + l0, x); return; }
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t l = l0 + j;
        if (l >= 0 && (uint64_t)l < numel) base[l] = (uint16_t)(w[j >> 1] >> (16 * (j & 1)));
    }
}

template <bool NT>
__device__ __forceinline__ void load8_f32(const float* base, int64_t l0, uint64_t numel, bool full, float (&out)[8])
{
    if (full) {
        const v4u a = load_v4<NT, 4>(base + l0), b = load_v4<NT, 4>(base + l0 + 4);
        out[0] = __uint_as_float(a.x); out[1] = __uint_as_float(a.y);
        out[2] = __uint_as_float(a.z); out[3] = __uint_as_float(a.w);
        out[4] = __uint_as_float(b.x); out[5] = __uint_as_float(b.y);
        out[6] = __uint_as_float(b.z); out[7] = __uint_as_float(b.w);
        return;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t l = l0 + j;
        out[j] = (l >= 0 && (uint64_t)l < numel) ? base[l] : 0.0f;
    }
}

template <bool NT>
__device__ __forceinline__ void store8_f32(float* base, int64_t l0, uint64_t numel, bool full, const float (&x)[8])
{
    if (full) {
        v4u a, b;
        a.x = __float_as_uint(x[0]); a.y = __float_as_uint(x[1]);
        a.z = __float_as_uint(x[2]); a.w = __float_as_uint(x[3]);
        b.x = __float_as_uint(x[4]); b.y = __float_as_uint(x[5]);
        b.z = __float_as_uint(x[6]); b.w = __float_as_uint(x[7]);
        store_v4<NT, 4>(base + l0, a);
        store_v4<NT, 4>(base + l0 + 4, b);
        return;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t l = l0 + j;
        if (l >= 0 && (uint64_t)l < numel) base[l] = x[j];
    }
}

__device__ __forceinline__ void unpack8(v4u x, float (&out)[8])
{
    out[0] = bf16_lo(x.x); out[1] = bf16_hi(x.x);
    out[2] = bf16_lo(x.y); out[3] = bf16_hi(x.y);
    out[4] = bf16_lo(x.z); out[5] = bf16_hi(x.z);
    out[6] = bf16_lo(x.w); out[7] = bf16_hi(x.w);
}

// Eight stochastic roundings with the 128 bits of one Philox block.
template <bool NAN_SAFE>
__device__ __forceinline__ v4u sr8(const float (&y)[8], const u32x4& r)
{
    v4u o;
    if (NAN_SAFE) {
        o.x = sr_pair_nan_safe(y[0], y[1], r.w[0]); o.y = sr_pair_nan_safe(y[2], y[3], r.w[1]);
        o.z = sr_pair_nan_safe(y[4], y[5], r.w[2]); o.w = sr_pair_nan_safe(y[6], y[7], r.w[3]);
    } else {
        o.x = sr_pair(y[0], y[1], r.w[0]); o.y = sr_pair(y[2], y[3], r.w[1]);
        o.z = sr_pair(y[4], y[5], r.w[2]); o.w = sr_pair(y[6], y[7], r.w[3]);
    }
    return o;
}

// True in every active lane when any active lane holds a NaN among its eight values (wave-uniform, so
// that the guarded rounding is a branch and not a per-lane select).
__device__ __forceinline__ bool any_nan8(const float (&y)[8])
{
    bool n = false;
#pragma unroll
    for (int j = 0; j < 8; ++j) n |= (y[j] != y[j]);
    return __builtin_amdgcn_ballot_w64(n) != 0;
}

// Largest i in [0, n) with start[i] <= chunk (start[] ascending, start[0] = 0).  Wave-uniform.
__device__ __forceinline__ uint32_t find_tensor(const uint32_t* start, uint32_t n, uint32_t chunk)
{
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (start[mid] <= chunk) lo = mid; else hi = mid;
    }
    return lo;
}

// ---------------------------------------------------------------------- 8-bit formats

// FMT 0: E4M3, 1: E5M2 (the OCP 8-bit formats).
template <int FMT> struct Fp8 {
    static constexpr int mb = FMT == 0 ? 3 : 2;
    static constexpr int ef = FMT == 0 ? 121 : 113;              // exponent field of the smallest normal
    static constexpr uint32_t top = FMT == 0 ? 0x7Eu : 0x7Cu;
    static constexpr uint32_t efmax = FMT == 0 ? 127u + 8u : 127u + 15u;   // binade of the largest finite value
};

// One element on the integer path: every range and NaN rule applied.  TOP: the code that larger
// results collapse to (the format's own by default: E4M3's largest finite value, E5M2's infinity).
template <int FMT, uint32_t TOP = Fp8<FMT>::top>
__device__ __forceinline__ uint32_t fp8_code(uint32_t bits, uint32_t r32)
{
    using P = Fp8<FMT>;
    return fp8_sign(bits) | fp8_finish<TOP>(bits, sr_fp8_magnitude<P::mb, P::ef>(bits, r32));
}

// Four elements into one word.  `ranged`: some value of the wave lies in the format's top binade
// or above, is infinite or a NaN (wave-uniform): the integer path with the range rules; otherwise
// the chip's conversion instruction, which computes the same function of (value, random word)
// below the top binade: it adds the word's top 23 - mb bits to the dropped fraction cut to as
// many bits and keeps the carry, subnormal results included (checked against the by-value
// oracle on every binary32 encoding).
template <int FMT, uint32_t TOP = Fp8<FMT>::top>
__device__ __forceinline__ uint32_t fp8_encode4(const uint32_t (&b)[4], const uint32_t (&r)[4], bool ranged)
{
    if (ranged)
        return fp8_code<FMT, TOP>(b[0], r[0]) | (fp8_code<FMT, TOP>(b[1], r[1]) << 8) |
               (fp8_code<FMT, TOP>(b[2], r[2]) << 16) | (fp8_code<FMT, TOP>(b[3], r[3]) << 24);
    int w = 0;
    if (FMT == 0) {
        w = __builtin_amdgcn_cvt_sr_fp8_f32(__uint_as_float(b[0]), (int)r[0], w, 0);
        w = __builtin_amdgcn_cvt_sr_fp8_f32(__uint_as_float(b[1]), (int)r[1], w, 1);
        w = __builtin_amdgcn_cvt_sr_fp8_f32(__uint_as_float(b[2]), (int)r[2], w, 2);
        w = __builtin_amdgcn_cvt_sr_fp8_f32(__uint_as_float(b[3]), (int)r[3], w, 3);
    } else {
        w = __builtin_amdgcn_cvt_sr_bf8_f32(__uint_as_float(b[0]), (int)r[0], w, 0);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(__uint_as_float(b[1]), (int)r[1], w, 1);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(__uint_as_float(b[2]), (int)r[2], w, 2);
        w = __builtin_amdgcn_cvt_sr_bf8_f32(__uint_as_float(b[3]), (int)r[3], w, 3);
    }
    return (uint32_t)w;
}

// The largest magnitude among four encodings, as an encoding (NaNs compare above everything).
__device__ __forceinline__ uint32_t max_magnitude4(const uint32_t (&b)[4])
{
    return max(max(b[0] & 0x7FFFFFFFu, b[1] & 0x7FFFFFFFu), max(b[2] & 0x7FFFFFFFu, b[3] & 0x7FFFFFFFu));
}

// Eight codes (two words) to binary32, times the power of two `inv_scale`, in one instruction per
// pair: the chip's scaled conversion multiplies the decoded value by 2^floor(log2 inv_scale),
// exactly, and decodes every code of both formats as the OCP tables say (checked on all 256, with
// several scales); NaN codes give a quiet NaN.
template <int FMT>
__device__ __forceinline__ void fp8_decode8(v2u codes, float inv_scale, float (&out)[8])
{
    typedef float f2 __attribute__((ext_vector_type(2)));
    f2 q[4];
    if (FMT == 0) {
        q[0] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8((int)codes.x, inv_scale, false);
        q[1] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8((int)codes.x, inv_scale, true);
        q[2] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8((int)codes.y, inv_scale, false);
        q[3] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8((int)codes.y, inv_scale, true);
    } else {
        q[0] = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8((int)codes.x, inv_scale, false);
        q[1] = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8((int)codes.x, inv_scale, true);
        q[2] = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8((int)codes.y, inv_scale, false);
        q[3] = __builtin_amdgcn_cvt_scalef32_pk_f32_bf8((int)codes.y, inv_scale, true);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) { out[2 * j] = q[j].x; out[2 * j + 1] = q[j].y; }
}

// Four values times the power of two `scale` into one word of codes.  Not `ranged` (no scaled
// value of the wave reaches the format's top binade, none is a NaN): the chip's scaled conversion,
// which rounds x / 2^floor(log2 inv_scale) -- the exact product, binary32 subnormal inputs
// included -- by the rule of fp8_encode4 (checked against that rule on 4e6 values per scale).  The
// product as a binary32 multiplication, which is what the definition says, can differ from the
// exact one only where it underflows, and there both give a zero with the product's sign.
// `ranged`: the multiplication and the integer path, saturating: both formats collapse to their
// largest finite value (an optimizer state must not hold an infinity: it would stay one).
template <int FMT>
__device__ __forceinline__ uint32_t fp8_encode4_scaled(const float (&x)[4], const uint32_t (&r)[4], float scale,
                                                       float inv_scale, bool ranged)
{
    if (ranged) {
        const uint32_t b[4] = {__float_as_uint(x[0] * scale), __float_as_uint(x[1] * scale),
                               __float_as_uint(x[2] * scale), __float_as_uint(x[3] * scale)};
        return fp8_encode4<FMT, (FMT == 0 ? 0x7Eu : 0x7Bu)>(b, r, true);
    }
    int w = 0;
    if (FMT == 0) {
        w = __builtin_amdgcn_cvt_scalef32_sr_fp8_f32(w, x[0], r[0], inv_scale, 0);
        w = __builtin_amdgcn_cvt_scalef32_sr_fp8_f32(w, x[1], r[1], inv_scale, 1);
        w = __builtin_amdgcn_cvt_scalef32_sr_fp8_f32(w, x[2], r[2], inv_scale, 2);
        w = __builtin_amdgcn_cvt_scalef32_sr_fp8_f32(w, x[3], r[3], inv_scale, 3);
    } else {
        w = __builtin_amdgcn_cvt_scalef32_sr_bf8_f32(w, x[0], r[0], inv_scale, 0);
        w = __builtin_amdgcn_cvt_scalef32_sr_bf8_f32(w, x[1], r[1], inv_scale, 1);
        w = __builtin_amdgcn_cvt_scalef32_sr_bf8_f32(w, x[2], r[2], inv_scale, 2);
        w = __builtin_amdgcn_cvt_scalef32_sr_bf8_f32(w, x[3], r[3], inv_scale, 3);
    }
    return (uint32_t)w;
}

// Eight codes starting at element l0 of `base`, element-wise, zeros outside [0, numel).
__device__ __forceinline__ v2u load8_u8(const uint8_t* base, int64_t l0, uint64_t numel)
{
    uint32_t w[2] = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t l = l0 + j;
        const uint32_t c = (l >= 0 && (uint64_t)l < numel) ? base[l] : 0u;
        w[j >> 2] |= c << (8 * (j & 3));
    }
    v2u r; r.x = w[0]; r.y = w[1];
    return r;
}
__device__ __forceinline__ void store8_u8(uint8_t* base, int64_t l0, uint64_t numel, v2u codes)
{
    const uint32_t w[2] = {codes.x, codes.y};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int64_t l = l0 + j;
        if (l >= 0 && (uint64_t)l < numel) base[l] = (uint8_t)(w[j >> 2] >> (8 * (j & 3)));
    }
}

// The power of two 2^e as a binary32 value (|e| <= 126).
__device__ __forceinline__ float pow2f(int e) { return __uint_as_float((uint32_t)(127 + e) << 23); }

// The write-back of a lane's eight new moments as 8-bit codes: m * 2^m_exp to E4M3 and
// v * 2^v_exp to E5M2, each with the element's 16-bit draw of its stream (mw, vw: two draws per
// word, low half for the even element, as for BF16 moments) in the top half of the random word.
// `nan`: some value of the wave may be a NaN (wave-uniform; the maxima below skip NaNs).
__device__ __forceinline__ void fp8_moments_out(const float (&m)[8], const float (&v)[8], int m_exp, int v_exp,
                                                const uint32_t* mw, const uint32_t* vw, bool nan, v2u& mo, v2u& vo)
{
    uint32_t mr[8], vr[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        mr[j] = (j & 1) ? (mw[j >> 1] & 0xFFFF0000u) : (mw[j >> 1] << 16);
        vr[j] = (j & 1) ? (vw[j >> 1] & 0xFFFF0000u) : (vw[j >> 1] << 16);
    }
    // the range rules apply from the formats' top binades upwards: scaled magnitudes of 2^8 for
    // E4M3 and 2^15 for E5M2 (a negative v cannot arise from the update but may be loaded: its
    // magnitude counts)
    float mmax = 0.0f, vmax = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        mmax = __builtin_fmaxf(mmax, __builtin_fabsf(m[j]));
        vmax = __builtin_fmaxf(vmax, __builtin_fabsf(v[j]));
    }
    const bool lane_ranged = mmax >= pow2f(8 - m_exp) || vmax >= pow2f(15 - v_exp);
    const bool ranged = nan || __builtin_amdgcn_ballot_w64(lane_ranged) != 0;   // wave-uniform
    const float ml[4] = {m[0], m[1], m[2], m[3]}, mh[4] = {m[4], m[5], m[6], m[7]};
    const float vl[4] = {v[0], v[1], v[2], v[3]}, vh[4] = {v[4], v[5], v[6], v[7]};
    const uint32_t mrl[4] = {mr[0], mr[1], mr[2], mr[3]}, mrh[4] = {mr[4], mr[5], mr[6], mr[7]};
    const uint32_t vrl[4] = {vr[0], vr[1], vr[2], vr[3]}, vrh[4] = {vr[4], vr[5], vr[6], vr[7]};
    const float ms = pow2f(m_exp), mi = pow2f(-m_exp), vs = pow2f(v_exp), vi = pow2f(-v_exp);
    mo.x = fp8_encode4_scaled<0>(ml, mrl, ms, mi, ranged); mo.y = fp8_encode4_scaled<0>(mh, mrh, ms, mi, ranged);
    vo.x = fp8_encode4_scaled<1>(vl, vrl, vs, vi, ranged); vo.y = fp8_encode4_scaled<1>(vh, vrh, vs, vi, ranged);
}

// The write-back of a lane's eight new parameters as E4M3 codes of y * 2^p_exp, each with the top
// 20 bits of its own 32-bit random word (r0: elements 0-3, r1: elements 4-7); saturating at the
// format's largest finite value.  `nan`: some value of the wave may be a NaN (wave-uniform).
__device__ __forceinline__ v2u fp8_param_out(const float (&y)[8], int p_exp, const uint32_t (&r0)[4],
                                             const uint32_t (&r1)[4], bool nan)
{
    float ymax = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) ymax = __builtin_fmaxf(ymax, __builtin_fabsf(y[j]));
    const bool ranged = nan || __builtin_amdgcn_ballot_w64(ymax >= pow2f(8 - p_exp)) != 0;   // wave-uniform
    const float yl[4] = {y[0], y[1], y[2], y[3]}, yh[4] = {y[4], y[5], y[6], y[7]};
    const float ps = pow2f(p_exp), pi = pow2f(-p_exp);
    v2u o;
    o.x = fp8_encode4_scaled<0>(yl, r0, ps, pi, ranged);
    o.y = fp8_encode4_scaled<0>(yh, r1, ps, pi, ranged);
    return o;
}

// ---------------------------------------------------------------------------- fused update

// Variant of the step, from the ABI's flag bits (same values as SR_FLAG_* in sradamw.h).
template <uint32_t F>
struct Mode {
    static constexpr bool fp32m  = (F & 1u) != 0;                 // binary32 moments, stored unrounded
    static constexpr bool master = (F & 8u) != 0;                 // aux = binary32 master parameters
    static constexpr bool kahan  = (F & 16u) != 0;                // aux = BF16 Kahan compensation
    static constexpr bool fp8m   = (F & 128u) != 0;               // 8-bit moments: m E4M3, v E5M2, scaled
    static constexpr bool fp8p   = (F & 512u) != 0;               // 8-bit parameter: E4M3 codes, scaled, SR
    static constexpr bool rnem   = !fp32m && !fp8m && (kahan || (F & 2u)); // BF16 moments rounded to nearest
    static constexpr bool rnep   = master || kahan || (F & 4u);   // BF16 parameter rounded to nearest
    static constexpr bool srm    = !fp32m && !fp8m && !rnem;      // BF16 moments stochastically rounded
    static constexpr bool aux    = master || kahan;
    static constexpr bool half   = fp32m;                         // fast path: a lane owns half a block
};

// Correctly rounded square root of a binary32 value in [2^-96, +inf]: the hardware's approximation
// and one step down or up, decided by the exact residuals x - s_down*s and x - s_up*s (one fused
// multiply-add each).  This is the core of the compiler's own expansion of sqrtf, without its input
// scaling for arguments below 2^-96 and without its special-case select for zeros, infinities and
// NaNs: seven instructions instead of sixteen.  Equal to sqrtf on every encoding of that range
// (compared once on the GPU, all 1.9e9 of them).
__device__ __forceinline__ float sqrt_normal(float x)
{
    const float s = __builtin_amdgcn_sqrtf(x);
    const float sd = __uint_as_float(__float_as_uint(s) - 1u), su = __uint_as_float(__float_as_uint(s) + 1u);
    const float rd = __builtin_fmaf(-sd, s, x);
    const float ru = __builtin_fmaf(-su, s, x);
    float r = (rd <= 0.0f) ? sd : s;
    r = (ru > 0.0f) ? su : r;
    return r;
}
constexpr uint32_t kSqrtNormalLo = 0x0F800000u, kSqrtNormalHi = 0x7F800000u;   // encodings of 2^-96 and +inf

// Correctly rounded quotient n / d for 2^-40 <= |n| <= 2^40 and 2^-41 <= d <= 2^41: the reciprocal
// approximation, one refinement of it, and two refinements of the quotient -- the compiler's own
// expansion of the division with its v_div_scale / v_div_fmas scaling and v_div_fixup steps left
// out.  Inside that domain those steps do nothing (the exponents differ by less than 96, neither
// operand nor the reciprocal nor the quotient is subnormal, nothing is zero, infinite or a NaN), so
// the instruction sequence is the same one: 8 instructions instead of 11.  A NaN numerator gives a
// NaN, as the full form does.  Compared with the full form on 3.4e10 random pairs of the domain and
// on its edges: identical.
__device__ __forceinline__ float div_normal(float n, float d)
{
    const float r0 = __builtin_amdgcn_rcpf(d);
    const float e0 = __builtin_fmaf(-d, r0, 1.0f);
    const float r1 = __builtin_fmaf(e0, r0, r0);
    const float q0 = n * r1;
    const float e1 = __builtin_fmaf(-d, q0, n);
    const float q1 = __builtin_fmaf(e1, r1, q0);
    const float e2 = __builtin_fmaf(-d, q1, n);
    return __builtin_fmaf(e2, r1, q1);
}
// A wave takes the short forms when every root argument lies in [2^-80, 2^80] (so every root in
// [2^-40, 2^40], inside sqrt_normal's range), every |numerator| in [2^-40, 2^40] and eps <= 2^40.
constexpr uint32_t kShortRootLo = (127u - 80u) << 23, kShortRootHi = (127u + 80u) << 23;
constexpr float kShortNumLo = 0x1p-40f, kShortNumHi = 0x1p40f;

// Algorithm 1 lines 5-10 for one element, in two parts.  One rounding per operation, in this order
// (no contraction: the library is built with -ffp-contract=off; sqrt and divide are correctly
// rounded).  `variant` is 0 at compile time in the kernels of the default arithmetic (straight-line
// code) and a kernel argument in the others (wave-uniform branches).
// Part 1, lines 5-8.  In: g, m, v.  m and v are replaced by the unrounded new moments; mh is the
// bias-corrected first moment, root_arg what line 10 takes the root of: the bias-corrected second
// moment, plus eps in the variant that has eps inside the root (Appendix B).  Bias corrections as
// multiplications by host reciprocals, or (variant) the divisions of lines 7-8 as printed.
template <bool CLIP>
__device__ __forceinline__ void moments_elem(const StepScalars& S, uint32_t variant, float c, float g,
                                             float& m, float& v, float& mh, float& root_arg)
{
    const float g1 = CLIP ? g * c : g;
    const float t1 = S.beta1 * m;
    const float t2 = S.omb1 * g1;
    const float m1 = t1 + t2;
    const float gg = g1 * g1;
    const float t3 = S.beta2 * v;
    const float t4 = S.omb2 * gg;
    const float v1 = t3 + t4;
    float vh;
    if (variant & VARIANT_DIV_BIAS) { mh = m1 / S.bc1; vh = v1 / S.bc2; }
    else                            { mh = m1 * S.rbc1; vh = v1 * S.rbc2; }
    root_arg = (variant & VARIANT_EPS_IN_ROOT) ? vh + S.eps : vh;
    m = m1;
    v = v1;
}

// Part 2, line 10.  Out: sum = lr u + (lr wd) p and y = p - sum (the unrounded new parameter).
// SHORT: the wave's operands lie in the domains of sqrt_normal and div_normal (the caller has checked).
template <bool SHORT>
__device__ __forceinline__ void step_elem(const StepScalars& S, uint32_t variant, float p, float mh, float root_arg,
                                          float& y, float& sum)
{
    const float root = SHORT ? sqrt_normal(root_arg) : __builtin_sqrtf(root_arg);
    const float d = (variant & VARIANT_EPS_IN_ROOT) ? root : root + S.eps;
    const float q = SHORT ? div_normal(mh, d) : mh / d;
    const float a = S.lr * q;
    const float w = S.lw * p;
    sum = a + w;
    y = p - sum;
}

// The N (8 or 4) elements a lane owns, as binary32 values, and what it will store.
template <int N>
struct LaneRegs {
    float p[N], g[N], m[N], v[N], aux[N];      // in; m, v (binary32 moments) and aux (master) also out
    uint32_t po[N / 2], mo[N / 2], vo[N / 2], ao[N / 2];   // out: packed BF16 pairs (p; BF16 m, v; Kahan c)
};

// The update of a lane's N elements and the write-back roundings (8-bit moments are left unrounded
// in L.m, L.v for fp8_moments_out).  pw, mw, vw: the random words of
// the lane's elements for the three output streams (16 bits per element; only read where the mode
// rounds stochastically).
template <uint32_t F, bool CLIP, bool VAR, int N>
__device__ __forceinline__ bool update_lane(LaneRegs<N>& L, const StepScalars& S, float c,
                                            const uint32_t* pw, const uint32_t* mw, const uint32_t* vw)
{
    using M = Mode<F>;
    const uint32_t variant = VAR ? S.variant : 0u;
    float y[N], sum[N], mh[N], ra[N];
#pragma unroll
    for (int j = 0; j < N; ++j) moments_elem<CLIP>(S, variant, c, L.g[j], L.m[j], L.v[j], mh[j], ra[j]);
    // Where the arithmetic is not hidden behind the memory time (8-bit moments) the square roots and divisions
    // of a wave whose operands all lie in the short forms' domains take those forms; zeros, tiny,
    // huge, infinite and negative root arguments and NaNs send the whole wave through sqrtf and the
    // full division (a NaN numerator alone does not: it gives a NaN either way).
    bool short_root = false;
    if (M::fp8m) {
        uint32_t lo = __float_as_uint(ra[0]), hi = lo;
        float nlo = __builtin_fabsf(mh[0]), nhi = nlo;
#pragma unroll
        for (int j = 1; j < N; ++j) {
            lo = min(lo, __float_as_uint(ra[j])); hi = max(hi, __float_as_uint(ra[j]));
            nlo = __builtin_fminf(nlo, __builtin_fabsf(mh[j])); nhi = __builtin_fmaxf(nhi, __builtin_fabsf(mh[j]));
        }
        const bool lane_ok = lo >= kShortRootLo && hi <= kShortRootHi && nlo >= kShortNumLo && nhi <= kShortNumHi;
        short_root = S.eps <= kShortNumHi && __builtin_amdgcn_ballot_w64(!lane_ok) == 0;   // wave-uniform
    }
    if (short_root) {
#pragma unroll
        for (int j = 0; j < N; ++j) step_elem<true>(S, variant, M::master ? L.aux[j] : L.p[j], mh[j], ra[j], y[j], sum[j]);
    } else {
#pragma unroll
        for (int j = 0; j < N; ++j) step_elem<false>(S, variant, M::master ? L.aux[j] : L.p[j], mh[j], ra[j], y[j], sum[j]);
    }
    // A NaN in m' or v' always makes y NaN, so one test covers all three outputs; the test is
    // folded over the wave so that the guarded roundings are a branch no wave takes in practice
    // (as per-lane selects they were 100 of the 680 vector instructions of a wave).
    bool nan = false;
    if (!M::rnep || M::srm || M::fp8m) {
        bool lane_nan = false;
#pragma unroll
        for (int j = 0; j < N; ++j) lane_nan |= (y[j] != y[j]);
        nan = __builtin_amdgcn_ballot_w64(lane_nan) != 0;          // wave-uniform
    }
    if (M::fp8p) {
        // 8-bit parameter: the unrounded result goes back in L.aux (unused otherwise in this
        // mode) for fp8_param_out, which needs a 32-bit random word per element
#pragma unroll
        for (int j = 0; j < N; ++j) L.aux[j] = y[j];
    } else if (M::master) {
        // O2-style mixed precision: the master stays binary32, the model copy is RNE(master)
#pragma unroll
        for (int j = 0; j < N; ++j) L.aux[j] = y[j];
#pragma unroll
        for (int j = 0; j < N / 2; ++j) L.po[j] = rne_pair(y[2 * j], y[2 * j + 1]);
    } else if (M::kahan) {
        // Kahan summation on the parameter with BF16 sum and BF16 compensation c:
        // yk = (-s) - c;  t = p + yk;  p' = RNE(t);  c' = RNE((p' - p) - yk)
        uint32_t pn[N];
        float cn[N];
#pragma unroll
        for (int j = 0; j < N; ++j) {
            const float ns = -sum[j];
            const float yk = ns - L.aux[j];
            const float t = L.p[j] + yk;
            pn[j] = rne_one(t) & 0xFFFF0000u;
            const float d1 = __uint_as_float(pn[j]) - L.p[j];
            cn[j] = d1 - yk;
        }
#pragma unroll
        for (int j = 0; j < N / 2; ++j) {
            L.po[j] = pack_high_halves(pn[2 * j], pn[2 * j + 1]);
            L.ao[j] = rne_pair(cn[2 * j], cn[2 * j + 1]);
        }
    } else if (M::rnep) {
#pragma unroll
        for (int j = 0; j < N / 2; ++j) L.po[j] = rne_pair(y[2 * j], y[2 * j + 1]);
    } else if (nan) {
#pragma unroll
        for (int j = 0; j < N / 2; ++j) L.po[j] = sr_pair_nan_safe(y[2 * j], y[2 * j + 1], pw[j]);
    } else {
#pragma unroll
        for (int j = 0; j < N / 2; ++j) L.po[j] = sr_pair(y[2 * j], y[2 * j + 1], pw[j]);
    }
    if (M::rnem) {
#pragma unroll
        for (int j = 0; j < N / 2; ++j) {
            L.mo[j] = rne_pair(L.m[2 * j], L.m[2 * j + 1]);
            L.vo[j] = rne_pair(L.v[2 * j], L.v[2 * j + 1]);
        }
    } else if (M::srm) {
        if (nan) {
#pragma unroll
            for (int j = 0; j < N / 2; ++j) {
                L.mo[j] = sr_pair_nan_safe(L.m[2 * j], L.m[2 * j + 1], mw[j]);
                L.vo[j] = sr_pair_nan_safe(L.v[2 * j], L.v[2 * j + 1], vw[j]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < N / 2; ++j) {
                L.mo[j] = sr_pair(L.m[2 * j], L.m[2 * j + 1], mw[j]);
                L.vo[j] = sr_pair(L.v[2 * j], L.v[2 * j + 1], vw[j]);
            }
        }
    }
    return nan;      // wave-uniform: some lane's new parameter (hence possibly a new moment) is a NaN
}

__device__ __forceinline__ void unpack4(v2u x, float (&out)[4])
{
    out[0] = bf16_lo(x.x); out[1] = bf16_hi(x.x); out[2] = bf16_lo(x.y); out[3] = bf16_hi(x.y);
}
__device__ __forceinline__ void floats4(v4u x, float (&out)[4])
{
    out[0] = __uint_as_float(x.x); out[1] = __uint_as_float(x.y);
    out[2] = __uint_as_float(x.z); out[3] = __uint_as_float(x.w);
}
__device__ __forceinline__ v4u bits4(const float (&x)[4])
{
    v4u r;
    r.x = __float_as_uint(x[0]); r.y = __float_as_uint(x[1]);
    r.z = __float_as_uint(x[2]); r.w = __float_as_uint(x[3]);
    return r;
}
__device__ __forceinline__ void floats8(v4u a, v4u b, float (&out)[8])
{
    out[0] = __uint_as_float(a.x); out[1] = __uint_as_float(a.y);
    out[2] = __uint_as_float(a.z); out[3] = __uint_as_float(a.w);
    out[4] = __uint_as_float(b.x); out[5] = __uint_as_float(b.y);
    out[6] = __uint_as_float(b.z); out[7] = __uint_as_float(b.w);
}
__device__ __forceinline__ v4u bits4lo(const float (&x)[8])
{
    v4u r;
    r.x = __float_as_uint(x[0]); r.y = __float_as_uint(x[1]);
    r.z = __float_as_uint(x[2]); r.w = __float_as_uint(x[3]);
    return r;
}
__device__ __forceinline__ v4u bits4hi(const float (&x)[8])
{
    v4u r;
    r.x = __float_as_uint(x[4]); r.y = __float_as_uint(x[5]);
    r.z = __float_as_uint(x[6]); r.w = __float_as_uint(x[7]);
    return r;
}
__device__ __forceinline__ v4u words4(const uint32_t (&w)[4]) { v4u r; r.x = w[0]; r.y = w[1]; r.z = w[2]; r.w = w[3]; return r; }
__device__ __forceinline__ v2u words2(const uint32_t (&w)[2]) { v2u r; r.x = w[0]; r.y = w[1]; return r; }

// The random words of a lane's block for the three output streams (only those the mode uses).
template <uint32_t F>
__device__ __forceinline__ void block_draws(const TensorDesc& T, const StepScalars& S, uint64_t gblk,
                                            u32x4& rp, u32x4& rp2, u32x4& rm, u32x4& rv)
{
    using M = Mode<F>;
    rp = {}; rp2 = {}; rm = {}; rv = {};
    if (M::fp8p) {
        // a 32-bit word per element: the parameter stream counts blocks of four elements here
        rp = block_bits(2 * gblk, STREAM_P, T.tensor_id, S.step, S.seed_lo, S.seed_hi);
        rp2 = block_bits(2 * gblk + 1, STREAM_P, T.tensor_id, S.step, S.seed_lo, S.seed_hi);
    } else if (!M::rnep) rp = block_bits(gblk, STREAM_P, T.tensor_id, S.step, S.seed_lo, S.seed_hi);
    if (M::srm || M::fp8m) {
        rm = block_bits(gblk, STREAM_M, T.tensor_id, S.step, S.seed_lo, S.seed_hi);
        rv = block_bits(gblk, STREAM_V, T.tensor_id, S.step, S.seed_lo, S.seed_hi);
    }
}

// One whole block of a lane that lies inside its tensor, as straight-line code: the block's loads
// are issued first (buffer accesses through the descriptors of the workgroup's chunk: `span`
// blocks starting at element lc0 of the tensor, the lane's block is the lane-th), the Philox
// draws, which need no data, run while the loads are in flight, then the update and the stores.
template <uint32_t F, bool CLIP, bool NT, bool VAR>
__device__ __forceinline__ void inner_block(const TensorDesc& T, const StepScalars& S, float c,
                                            uint64_t gblk, int64_t lc0, uint32_t lane, uint32_t span)
{
    using M = Mode<F>;
    const uint32_t o16 = lane * 16u, o32 = lane * 32u;          // byte offsets in BF16 / binary32 arrays
    const rsrc_t rp = M::fp8p ? chunk_rsrc<uint8_t>(T.p, lc0, span * 8u) : chunk_rsrc<uint16_t>(T.p, lc0, span * 8u);
    const rsrc_t rg = chunk_rsrc<uint16_t>(T.g, lc0, span * 8u);
    const rsrc_t rm = M::fp32m ? chunk_rsrc<float>(T.m, lc0, span * 8u)
                    : M::fp8m  ? chunk_rsrc<uint8_t>(T.m, lc0, span * 8u) : chunk_rsrc<uint16_t>(T.m, lc0, span * 8u);
    const rsrc_t rv = M::fp32m ? chunk_rsrc<float>(T.v, lc0, span * 8u)
                    : M::fp8m  ? chunk_rsrc<uint8_t>(T.v, lc0, span * 8u) : chunk_rsrc<uint16_t>(T.v, lc0, span * 8u);
    const rsrc_t ra = M::master ? chunk_rsrc<float>(T.aux, lc0, span * 8u) : chunk_rsrc<uint16_t>(T.aux, lc0, span * 8u);
    v4u pq = {}, aq = {}, mq0 = {}, mq1 = {}, vq0 = {}, vq1 = {}, xq0 = {}, xq1 = {};
    v2u m8 = {}, v8 = {}, p8 = {};
    if (M::fp8p) p8 = buf_load8<NT>(rp, lane * 8u);
    else if (!M::master) pq = buf_load16<NT>(rp, o16);
    const v4u gq = buf_load16<NT>(rg, o16);
    if (M::fp32m) {
        mq0 = buf_load16<NT>(rm, o32); mq1 = buf_load16<NT>(rm, o32 + 16u);
        vq0 = buf_load16<NT>(rv, o32); vq1 = buf_load16<NT>(rv, o32 + 16u);
    } else if (M::fp8m) {
        m8 = buf_load8<NT>(rm, lane * 8u);
        v8 = buf_load8<NT>(rv, lane * 8u);
    } else {
        mq0 = buf_load16<NT>(rm, o16);
        vq0 = buf_load16<NT>(rv, o16);
    }
    if (M::master) { xq0 = buf_load16<NT>(ra, o32); xq1 = buf_load16<NT>(ra, o32 + 16u); }
    if (M::kahan) aq = buf_load16<NT>(ra, o16);

    u32x4 dp, dp2, dm, dv;
    block_draws<F>(T, S, gblk, dp, dp2, dm, dv);

    LaneRegs<8> L;
    const int m_exp = (int)(int8_t)(T.flags >> DESC_MEXP_SHIFT), v_exp = (int)(int8_t)(T.flags >> DESC_VEXP_SHIFT);
    const int p_exp = (int)(int8_t)(T.flags >> DESC_PEXP_SHIFT);
    if (M::fp8p) fp8_decode8<0>(p8, pow2f(-p_exp), L.p);
    else if (!M::master) unpack8(pq, L.p);
    unpack8(gq, L.g);
    if (M::fp32m)     { floats8(mq0, mq1, L.m); floats8(vq0, vq1, L.v); }
    else if (M::fp8m) { fp8_decode8<0>(m8, pow2f(-m_exp), L.m); fp8_decode8<1>(v8, pow2f(-v_exp), L.v); }
    else              { unpack8(mq0, L.m); unpack8(vq0, L.v); }
    if (M::master) floats8(xq0, xq1, L.aux);
    if (M::kahan) unpack8(aq, L.aux);
    const bool nan = update_lane<F, CLIP, VAR, 8>(L, S, c, dp.w, dm.w, dv.w);
    const bool integer_path = nan || (VAR && (S.variant & VARIANT_FP8_INTEGER));
    if (M::fp8p) buf_store8<NT>(rp, lane * 8u, fp8_param_out(L.aux, p_exp, dp.w, dp2.w, integer_path));
    else buf_store16<NT>(rp, o16, words4(L.po));
    if (M::fp32m) {
        buf_store16<NT>(rm, o32, bits4lo(L.m)); buf_store16<NT>(rm, o32 + 16u, bits4hi(L.m));
        buf_store16<NT>(rv, o32, bits4lo(L.v)); buf_store16<NT>(rv, o32 + 16u, bits4hi(L.v));
    } else if (M::fp8m) {
        v2u mo, vo;
        fp8_moments_out(L.m, L.v, m_exp, v_exp, dm.w, dv.w, integer_path, mo, vo);
        buf_store8<NT>(rm, lane * 8u, mo);
        buf_store8<NT>(rv, lane * 8u, vo);
    } else {
        buf_store16<NT>(rm, o16, words4(L.mo));
        buf_store16<NT>(rv, o16, words4(L.vo));
    }
    if (M::master) { buf_store16<NT>(ra, o32, bits4lo(L.aux)); buf_store16<NT>(ra, o32 + 16u, bits4hi(L.aux)); }
    if (M::kahan) buf_store16<NT>(ra, o16, words4(L.ao));
}

// A block that straddles the first or last element of its tensor (counter blocks that do not
// start at element 0, or a size that is not a multiple of 8): element-wise accesses with bounds,
// zeros outside [0, numel).
template <uint32_t F, bool CLIP, bool VAR>
__device__ __forceinline__ void edge_block(const TensorDesc& T, const StepScalars& S, float c,
                                           uint64_t gblk, int64_t l0)
{
    using M = Mode<F>;
    const uint64_t numel = T.numel;
    LaneRegs<8> L;
    const int m_exp = (int)(int8_t)(T.flags >> DESC_MEXP_SHIFT), v_exp = (int)(int8_t)(T.flags >> DESC_VEXP_SHIFT);
    const int p_exp = (int)(int8_t)(T.flags >> DESC_PEXP_SHIFT);
    if (M::fp8p) fp8_decode8<0>(load8_u8(reinterpret_cast<const uint8_t*>(T.p), l0, numel), pow2f(-p_exp), L.p);
    else if (!M::master) unpack8(load8_bf16<false>(T.p, l0, numel, false), L.p);
    unpack8(load8_bf16<false>(T.g, l0, numel, false), L.g);
    if (M::fp32m) {
        load8_f32<false>(static_cast<const float*>(T.m), l0, numel, false, L.m);
        load8_f32<false>(static_cast<const float*>(T.v), l0, numel, false, L.v);
    } else if (M::fp8m) {
        fp8_decode8<0>(load8_u8(static_cast<const uint8_t*>(T.m), l0, numel), pow2f(-m_exp), L.m);
        fp8_decode8<1>(load8_u8(static_cast<const uint8_t*>(T.v), l0, numel), pow2f(-v_exp), L.v);
    } else {
        unpack8(load8_bf16<false>(static_cast<const uint16_t*>(T.m), l0, numel, false), L.m);
        unpack8(load8_bf16<false>(static_cast<const uint16_t*>(T.v), l0, numel, false), L.v);
    }
    if (M::master) load8_f32<false>(static_cast<const float*>(T.aux), l0, numel, false, L.aux);
    if (M::kahan) unpack8(load8_bf16<false>(static_cast<const uint16_t*>(T.aux), l0, numel, false), L.aux);
    u32x4 dp, dp2, dm, dv;
    block_draws<F>(T, S, gblk, dp, dp2, dm, dv);
    const bool nan = update_lane<F, CLIP, VAR, 8>(L, S, c, dp.w, dm.w, dv.w);
    const bool integer_path = nan || (VAR && (S.variant & VARIANT_FP8_INTEGER));
    if (M::fp8p) store8_u8(reinterpret_cast<uint8_t*>(T.p), l0, numel, fp8_param_out(L.aux, p_exp, dp.w, dp2.w, integer_path));
    else store8_bf16<false>(T.p, l0, numel, false, words4(L.po));
    if (M::fp32m) {
        store8_f32<false>(static_cast<float*>(T.m), l0, numel, false, L.m);
        store8_f32<false>(static_cast<float*>(T.v), l0, numel, false, L.v);
    } else if (M::fp8m) {
        v2u mo, vo;
        fp8_moments_out(L.m, L.v, m_exp, v_exp, dm.w, dv.w, integer_path, mo, vo);
        store8_u8(static_cast<uint8_t*>(T.m), l0, numel, mo);
        store8_u8(static_cast<uint8_t*>(T.v), l0, numel, vo);
    } else {
        store8_bf16<false>(static_cast<uint16_t*>(T.m), l0, numel, false, words4(L.mo));
        store8_bf16<false>(static_cast<uint16_t*>(T.v), l0, numel, false, words4(L.vo));
    }
    if (M::master) store8_f32<false>(static_cast<float*>(T.aux), l0, numel, false, L.aux);
    if (M::kahan) store8_bf16<false>(static_cast<uint16_t*>(T.aux), l0, numel, false, words4(L.ao));
}

// One whole block of a lane, at any element offset (see inner_block and edge_block).
template <uint32_t F, bool CLIP, bool NT, bool VAR>
__device__ __forceinline__ void general_block(const TensorDesc& T, const StepScalars& S, float c,
                                              uint64_t gblk, int64_t lc0, uint32_t lane, uint32_t span)
{
    const int64_t l0 = lc0 + (int64_t)lane * 8;
    if (block_inside(l0, T.numel)) inner_block<F, CLIP, NT, VAR>(T, S, c, gblk, lc0, lane, span);
    else edge_block<F, CLIP, VAR>(T, S, c, gblk, l0);
}

// F: SR_FLAG_* bits of the step.  CLIP: scale gradients by min(1, max_norm/(norm + 1e-6)).
// NT: streaming cache policy.  VAR: the arithmetic variants of StepScalars::variant are honoured
// (false: default arithmetic only).  One wave per workgroup, one chunk per workgroup.
template <uint32_t F, bool CLIP, bool NT, bool VAR>
__global__ __launch_bounds__(kThreads) void adamw_kernel(const AdamwBatch B)
{
    using M = Mode<F>;
    const uint32_t chunk = blockIdx.x;
    const uint32_t ti = find_tensor(B.chunk_start, B.s.n_tensors, chunk);
    const TensorDesc& T = B.t[ti];
    const uint64_t numel = T.numel;
    const uint64_t G0 = T.elem_offset;
    const uint64_t gblk0 = G0 >> 3;
    const uint64_t nblk = ((G0 + numel - 1) >> 3) - gblk0 + 1;     // host guarantees numel > 0
    const bool vec = (T.flags & DESC_VEC) != 0;
    const uint32_t tensor_id = T.tensor_id;
    const StepScalars& S = B.s;
    const uint64_t cl = chunk - B.chunk_start[ti];                  // chunk index inside the tensor

    float c = 1.0f;
    if (CLIP) {
        const float norm = *S.d_norm;
        // NaN and infinities are the encodings whose exponent field is all ones (wave-uniform test)
        if (S.skip_nonfinite && (__float_as_uint(norm) & 0x7F800000u) == 0x7F800000u) return;
        c = S.max_norm / (norm + 1e-6f);
        if (c > 1.0f) c = 1.0f;
    }

    if constexpr (M::half) {
        // Binary32 moments (and master parameters): a lane owns HALF a block (4 elements), so that
        // every access of the wave is one contiguous run (BF16 arrays: 8 bytes per lane; binary32
        // arrays: 16 bytes per lane) and a wave issues few, short accesses -- measured 16% faster
        // than whole blocks per lane, whose binary32 accesses would be strided.  The two lanes of
        // a block draw the same Philox block and each uses its half.  A chunk is kThreads*4
        // elements = kThreads/2 blocks.  (For BF16 moments the same ownership, with the three
        // Philox blocks of a lane pair shared through DPP, was measured 5% slower than whole
        // blocks: BF16 moments keep whole blocks.)
        const uint64_t efirst = cl * (uint64_t)(kThreads * 4);
        if (vec && efirst + (uint64_t)(kThreads * 4) <= numel) {          // wave-uniform
            const uint64_t e = efirst + (uint64_t)threadIdx.x * 4;
            uint32_t pw[2] = {0, 0};
            LaneRegs<4> L;
            if constexpr (M::master) {
                // buffer accesses (measured 29.8 ms against 30.9 ms with global ones on 6.66e9 elements)
                const uint32_t o8 = threadIdx.x * 8u, o16 = threadIdx.x * 16u;
                const rsrc_t rp = chunk_rsrc<uint16_t>(T.p, (int64_t)efirst, kThreads * 4u);
                const rsrc_t rg = chunk_rsrc<uint16_t>(T.g, (int64_t)efirst, kThreads * 4u);
                const rsrc_t rm = chunk_rsrc<float>(T.m, (int64_t)efirst, kThreads * 4u);
                const rsrc_t rv = chunk_rsrc<float>(T.v, (int64_t)efirst, kThreads * 4u);
                const rsrc_t rx = chunk_rsrc<float>(T.aux, (int64_t)efirst, kThreads * 4u);   // master parameters
                floats4(buf_load16<NT>(rx, o16), L.aux);
                unpack4(buf_load8<NT>(rg, o8), L.g);
                floats4(buf_load16<NT>(rm, o16), L.m);
                floats4(buf_load16<NT>(rv, o16), L.v);
                update_lane<F, CLIP, VAR, 4>(L, S, c, pw, pw, pw);
                buf_store8<NT>(rp, o8, words2(L.po));
                buf_store16<NT>(rm, o16, bits4(L.m));
                buf_store16<NT>(rv, o16, bits4(L.v));
                buf_store16<NT>(rx, o16, bits4(L.aux));
            } else {
                // global accesses: with BF16 parameters read and written 8 bytes per lane this mix
                // is 3% faster than with buffer accesses (23.1 against 23.8 ms)
                float* mp = static_cast<float*>(T.m) + e;
                float* vp = static_cast<float*>(T.v) + e;
                unpack4(load_v2<NT>(T.p + e), L.p);
                unpack4(load_v2<NT>(T.g + e), L.g);
                floats4(load_v4<NT, 4>(mp), L.m);
                floats4(load_v4<NT, 4>(vp), L.v);
                if (!M::rnep) {
                    const u32x4 r = block_bits((G0 + e) >> 3, STREAM_P, tensor_id, S.step, S.seed_lo, S.seed_hi);
                    const bool upper = (threadIdx.x & 1u) != 0;            // elements 4..7 of the block
                    pw[0] = upper ? r.w[2] : r.w[0];
                    pw[1] = upper ? r.w[3] : r.w[1];
                }
                update_lane<F, CLIP, VAR, 4>(L, S, c, pw, pw, pw);
                store_v2<NT>(T.p + e, words2(L.po));
                store_v4<NT, 4>(mp, bits4(L.m));
                store_v4<NT, 4>(vp, bits4(L.v));
            }
            return;
        }
        // Tail chunk, or counter blocks that do not start at element 0: the chunk's kThreads/2
        // blocks, one whole block per lane.
        const uint64_t b0 = cl * (uint64_t)(kThreads / 2), b = b0 + threadIdx.x;
        if (threadIdx.x >= kThreads / 2 || b >= nblk) return;
        general_block<F, CLIP, NT, VAR>(T, S, c, gblk0 + b, (int64_t)((gblk0 + b0) << 3) - (int64_t)G0, threadIdx.x, kThreads / 2);
    } else {
        // BF16 moments: a lane owns one whole block; a chunk is kThreads blocks.
        const uint64_t b0 = cl * (uint64_t)kThreads, b = b0 + threadIdx.x;
        if (b >= nblk) return;
        general_block<F, CLIP, NT, VAR>(T, S, c, gblk0 + b, (int64_t)((gblk0 + b0) << 3) - (int64_t)G0, threadIdx.x, kThreads);
    }
}

// --------------------------------------------------------------------- stream probe

// The memory traffic of the BF16 update with no arithmetic: reads the blocks of p, g, m, v and
// writes p, m, v back.  `mask` is 0 at run time (the data are unchanged) but unknown to the
// compiler, so neither the loads nor the stores can be dropped.  Same geometry as the update:
// one wave per workgroup, one block per lane, streaming buffer accesses.
__global__ __launch_bounds__(kThreads) void stream_probe_kernel(uint16_t* __restrict__ p, const uint16_t* __restrict__ g,
                                                               uint16_t* __restrict__ m, uint16_t* __restrict__ v,
                                                               uint64_t nblk, uint64_t wg0, uint32_t mask)
{
    const uint64_t b0 = ((uint64_t)blockIdx.x + wg0) * kThreads, b = b0 + threadIdx.x;
    if (b >= nblk) return;
    const int64_t e0 = (int64_t)(b0 << 3);
    const rsrc_t rp = chunk_rsrc<uint16_t>(p, e0, kThreads * 8u), rg = chunk_rsrc<uint16_t>(g, e0, kThreads * 8u);
    const rsrc_t rm = chunk_rsrc<uint16_t>(m, e0, kThreads * 8u), rv = chunk_rsrc<uint16_t>(v, e0, kThreads * 8u);
    const uint32_t off = threadIdx.x * 16u;
    const v4u P = buf_load16<true>(rp, off), G = buf_load16<true>(rg, off);
    const v4u M = buf_load16<true>(rm, off), V = buf_load16<true>(rv, off);
    const v4u k = G & mask;
    buf_store16<true>(rp, off, P ^ k);
    buf_store16<true>(rm, off, M ^ k);
    buf_store16<true>(rv, off, V ^ k);
}

// The same for the step with 8-bit moments: 16 bytes of p and g and 8 bytes of the m and v codes
// read per lane, 16 bytes of p and 8 of each code array written back unchanged.
__global__ __launch_bounds__(kThreads) void stream_probe_fp8m_kernel(uint16_t* __restrict__ p, const uint16_t* __restrict__ g,
                                                                    uint8_t* __restrict__ m, uint8_t* __restrict__ v,
                                                                    uint64_t nblk, uint64_t wg0, uint32_t mask)
{
    const uint64_t b0 = ((uint64_t)blockIdx.x + wg0) * kThreads, b = b0 + threadIdx.x;
    if (b >= nblk) return;
    const int64_t e0 = (int64_t)(b0 << 3);
    const rsrc_t rp = chunk_rsrc<uint16_t>(p, e0, kThreads * 8u), rg = chunk_rsrc<uint16_t>(g, e0, kThreads * 8u);
    const rsrc_t rm = chunk_rsrc<uint8_t>(m, e0, kThreads * 8u), rv = chunk_rsrc<uint8_t>(v, e0, kThreads * 8u);
    const v4u P = buf_load16<true>(rp, threadIdx.x * 16u), G = buf_load16<true>(rg, threadIdx.x * 16u);
    const v2u M = buf_load8<true>(rm, threadIdx.x * 8u), V = buf_load8<true>(rv, threadIdx.x * 8u);
    const v4u k = G & mask;
    v2u k2; k2.x = k.x; k2.y = k.y;
    buf_store16<true>(rp, threadIdx.x * 16u, P ^ k);
    buf_store8<true>(rm, threadIdx.x * 8u, M ^ k2);
    buf_store8<true>(rv, threadIdx.x * 8u, V ^ k2);
}

// ----------------------------------------------------------------------- standalone SR cast

// A lane owns half a block (4 elements) at a time: one 16-byte load and one 8-byte store per lane,
// every access of the wave contiguous; the two lanes of a block draw the same Philox block.  A
// workgroup takes kCastIters such rows (all loads first).
constexpr int kCastIters = SR_TUNE_CAST_ITERS;
constexpr int kCastChunkElems = kThreads * 4 * kCastIters;

template <bool NT>
__global__ __launch_bounds__(kThreads) void cast_kernel(const float* __restrict__ src,
                                                        uint16_t* __restrict__ dst, uint64_t n,
                                                        uint64_t chunk0, uint32_t seed_lo, uint32_t seed_hi,
                                                        uint32_t step, uint32_t tensor_id)
{
    const uint64_t cfirst = ((uint64_t)blockIdx.x + chunk0) * (uint64_t)kCastChunkElems;
    if (cfirst + (uint64_t)kCastChunkElems <= n) {                 // wave-uniform
        const rsrc_t rs = chunk_rsrc<float>(src, (int64_t)cfirst, kCastChunkElems);
        const rsrc_t rd = chunk_rsrc<uint16_t>(dst, (int64_t)cfirst, kCastChunkElems);
        v4u xs[kCastIters];
#pragma unroll
        for (int it = 0; it < kCastIters; ++it) xs[it] = buf_load16<NT>(rs, (uint32_t)(it * kThreads + threadIdx.x) * 16u);
#pragma unroll
        for (int it = 0; it < kCastIters; ++it) {
            const uint32_t row = (uint32_t)(it * kThreads + threadIdx.x);
            const uint64_t e = cfirst + (uint64_t)row * 4;
            const v4u x = xs[it];
            const u32x4 r = block_bits(e >> 3, STREAM_CAST, tensor_id, step, seed_lo, seed_hi);
            const bool upper = ((e >> 2) & 1u) != 0;
            const uint32_t w0 = upper ? r.w[2] : r.w[0], w1 = upper ? r.w[3] : r.w[1];
            const float y0 = __uint_as_float(x.x), y1 = __uint_as_float(x.y);
            const float y2 = __uint_as_float(x.z), y3 = __uint_as_float(x.w);
            const bool nan = __builtin_amdgcn_ballot_w64((y0 != y0) | (y1 != y1) | (y2 != y2) | (y3 != y3)) != 0;
            v2u o;
            if (nan) { o.x = sr_pair_nan_safe(y0, y1, w0); o.y = sr_pair_nan_safe(y2, y3, w1); }
            else     { o.x = sr_pair(y0, y1, w0);          o.y = sr_pair(y2, y3, w1); }
            buf_store8<NT>(rd, row * 8u, o);
        }
        return;
    }
    // Tail chunk: its blocks, one per lane and pass, the last one element-wise.
    const uint64_t nblk = (n + 7) >> 3;
    const uint64_t bfirst = cfirst >> 3;
    for (uint64_t b = bfirst + threadIdx.x; b < nblk; b += kThreads) {
        const int64_t l0 = (int64_t)(b << 3);
        const bool full = block_inside(l0, n);
        float y[8];
        load8_f32<NT>(src, l0, n, full, y);
        const u32x4 r = block_bits(b, STREAM_CAST, tensor_id, step, seed_lo, seed_hi);
        const v4u o = any_nan8(y) ? sr8<true>(y, r) : sr8<false>(y, r);
        store8_bf16<NT>(dst, l0, n, full, o);
    }
}

// --------------------------------------------------- standalone SR cast to 8-bit formats

// A lane owns four elements: one 16-byte load, one Philox block (a 32-bit word per element), one
// 4-byte store; every access of the wave is contiguous.  FMT 0: E4M3, 1: E5M2.  The range and NaN
// rules only matter from the binade that holds the format's largest finite value upwards: they are
// applied in a branch taken when some lane of the wave holds such a value.
constexpr int kFp8Iters = SR_TUNE_FP8_ITERS;     // groups of 4 elements per lane
constexpr int kFp8ChunkElems = kThreads * 4 * kFp8Iters;

template <int FMT, bool NT>
__global__ __launch_bounds__(kThreads) void cast_fp8_kernel(const float* __restrict__ src,
                                                            uint8_t* __restrict__ dst, uint64_t n,
                                                            uint64_t chunk0, uint32_t seed_lo, uint32_t seed_hi,
                                                            uint32_t step, uint32_t tensor_id, uint32_t integer_path)
{
    using P = Fp8<FMT>;
    const uint64_t cfirst = ((uint64_t)blockIdx.x + chunk0) * (uint64_t)kFp8ChunkElems;
    if (cfirst + (uint64_t)kFp8ChunkElems <= n) {                     // wave-uniform: a whole chunk
        const rsrc_t rs = chunk_rsrc<float>(src, (int64_t)cfirst, kFp8ChunkElems);
        const rsrc_t rd = chunk_rsrc<uint8_t>(dst, (int64_t)cfirst, kFp8ChunkElems);
        v4u xs[kFp8Iters];
#pragma unroll
        for (int it = 0; it < kFp8Iters; ++it) xs[it] = buf_load16<NT>(rs, (uint32_t)(it * kThreads + threadIdx.x) * 16u);
#pragma unroll
        for (int it = 0; it < kFp8Iters; ++it) {
            const uint32_t row = (uint32_t)(it * kThreads) + threadIdx.x;
            const uint64_t e = cfirst + (uint64_t)row * 4;
            const u32x4 r = philox4x32_10((uint32_t)(e >> 2), (STREAM_FP8 << 29) | (uint32_t)(e >> 34), tensor_id, step,
                                          seed_lo, seed_hi);
            const v4u x = xs[it];
            const uint32_t b[4] = {x.x, x.y, x.z, x.w};
            // the range rules apply when some lane holds a value in the format's top binade or
            // above (or an infinity or a NaN): integer path for the whole wave
            // (integer_path: a test switch that sends every wave down the integer path)
            const bool ranged = integer_path != 0 ||
                                __builtin_amdgcn_ballot_w64(max_magnitude4(b) >= (P::efmax << 23)) != 0;
            const uint32_t o = fp8_encode4<FMT>(b, r.w, ranged);
            __builtin_amdgcn_raw_buffer_store_b32(o, rd, (int)(row * 4u), 0, NT ? 2 : 0);
        }
        return;
    }
    // tail chunk: element-wise with bounds
#pragma unroll
    for (int it = 0; it < kFp8Iters; ++it) {
        const uint64_t e = cfirst + (uint64_t)(it * kThreads + threadIdx.x) * 4;
        if (e >= n) return;
        const u32x4 r = philox4x32_10((uint32_t)(e >> 2), (STREAM_FP8 << 29) | (uint32_t)(e >> 34), tensor_id, step,
                                      seed_lo, seed_hi);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (e + j < n) dst[e + j] = (uint8_t)fp8_code<FMT>(__float_as_uint(src[e + j]), r.w[j]);
        }
    }
}

// ------------------------------------------------------------------------- gradient norm

// x of the lane that a DPP control selects (0.0 where the control selects none or the row is masked).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_read(double x)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(x), CTRL, ROW_MASK, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(x), CTRL, ROW_MASK, 0xF, true);
    return __hiloint2double(hi, lo);
}

// Sum of x over the 64 lanes in a fixed order, returned in every lane: running sums inside each row
// of 16 lanes (row_shr 1, 2, 4, 8), then row 0's total into row 1 and row 2's into row 3
// (row_bcast:15), then the lower half's total into the upper half (row_bcast:31); lane 63 holds the
// wave's sum.  Register-to-register moves: no trip through the LDS crossbar as with ds_bpermute.
__device__ __forceinline__ double wave_sum(double x)
{
    x += dpp_read<0x111, 0xF>(x);
    x += dpp_read<0x112, 0xF>(x);
    x += dpp_read<0x114, 0xF>(x);
    x += dpp_read<0x118, 0xF>(x);
    x += dpp_read<0x142, 0xA>(x);
    x += dpp_read<0x143, 0xC>(x);
    const int lo = __builtin_amdgcn_readlane(__double2loint(x), 63);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(x), 63);
    return __hiloint2double(hi, lo);
}

// ----------------------------------------------------------------- gradient accumulation

// acc <- Q(acc + scale g) over micro-batches, every tensor BF16: t = scale g; s = acc + t (one
// rounding each); Q = stochastic rounding with output stream 4 and the micro-step in the counter,
// or round-to-nearest.  With ACC_NORM each chunk also leaves the binary64 sum of squares of the
// values it wrote, so the global norm of the accumulated gradient costs no second pass over it.
__global__ __launch_bounds__(kAccThreads) void accumulate_kernel(const AccBatch B, double* __restrict__ partials)
{
    const uint32_t chunk = blockIdx.x;
    const uint32_t ti = find_tensor(B.chunk_start, B.n_tensors, chunk);
    const AccDesc& T = B.t[ti];
    const uint64_t numel = T.numel;
    const uint64_t G0 = T.elem_offset;
    const uint64_t gblk0 = G0 >> 3;
    const uint64_t nblk = ((G0 + numel - 1) >> 3) - gblk0 + 1;
    const bool rne = (B.mode & ACC_RNE) != 0, first = (B.mode & ACC_FIRST) != 0;
    const uint64_t bchunk = (uint64_t)(chunk - B.chunk_start[ti]) * (uint64_t)(kAccThreads * kAccIters);
    const uint64_t bfirst = bchunk + threadIdx.x;
    const int64_t lc0 = (int64_t)((gblk0 + bchunk) << 3) - (int64_t)G0;       // first element of the chunk
    const rsrc_t ra = chunk_rsrc<uint16_t>(T.acc, lc0, kAccChunkElems), rg = chunk_rsrc<uint16_t>(T.g, lc0, kAccChunkElems);

    double sq = 0.0;
#pragma unroll 2
    for (int it = 0; it < kAccIters; ++it) {
        const uint64_t b = bfirst + (uint64_t)it * kAccThreads;
        if (b >= nblk) break;
        const int64_t l0 = (int64_t)((gblk0 + b) << 3) - (int64_t)G0;
        const bool full = block_inside(l0, numel);
        const uint32_t off = (uint32_t)(it * kAccThreads + threadIdx.x) * 16u;
        // whole blocks: buffer loads first, the Philox draw (which needs no data) while they are
        // in flight; blocks at a tensor's ragged ends: element-wise with bounds
        v4u gq = {}, aq = {};
        if (full) {
            gq = buf_load16<true>(rg, off);
            if (!first) aq = buf_load16<true>(ra, off);
        }
        u32x4 r = {};
        if (!rne) r = block_bits(gblk0 + b, STREAM_ACC, T.tensor_id, B.micro_step, B.seed_lo, B.seed_hi);
        if (!full) {
            gq = load8_bf16<false>(T.g, l0, numel, false);
            if (!first) aq = load8_bf16<false>(T.acc, l0, numel, false);
        }
        float a[8], g[8], s[8];
        unpack8(gq, g);
        unpack8(aq, a);                                          // zeros for the first micro-batch
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float t = B.scale * g[j];
            s[j] = a[j] + t;
        }
        v4u o;
        if (rne) {
            o.x = rne_pair(s[0], s[1]); o.y = rne_pair(s[2], s[3]);
            o.z = rne_pair(s[4], s[5]); o.w = rne_pair(s[6], s[7]);
        } else {
            o = any_nan8(s) ? sr8<true>(s, r) : sr8<false>(s, r);
        }
        if (full) buf_store16<true>(ra, off, o);
        else store8_bf16<false>(T.acc, l0, numel, false, o);
        if (B.mode & ACC_NORM) {
            float w[8];
            unpack8(o, w);
            if (full) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const double wd = (double)w[j];
                    sq = __builtin_fma(wd, wd, sq);
                }
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    // lanes of a partial block wrote only elements inside the tensor
                    const int64_t l = l0 + j;
                    const double wd = (l >= 0 && (uint64_t)l < numel) ? (double)w[j] : 0.0;
                    sq = __builtin_fma(wd, wd, sq);
                }
            }
        }
    }
    if (B.mode & ACC_NORM) {
        sq = wave_sum(sq);
        if constexpr (kAccThreads == 64) {                     // one wave: its sum is the chunk's
            if (threadIdx.x == 0) partials[B.partial_base + chunk] = sq;
        } else {
            __shared__ double wsum[kAccThreads / 64];
            if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = sq;
            __syncthreads();
            if (threadIdx.x == 0) {
                double t = wsum[0];
#pragma unroll
                for (int w = 1; w < kAccThreads / 64; ++w) t += wsum[w];
                partials[B.partial_base + chunk] = t;
            }
        }
    }
}

// Pass 1: one binary64 partial sum of squares per chunk.  g is widened to binary64 before
// squaring, so tiny or huge gradients neither underflow nor overflow, and each square is exact.
__global__ __launch_bounds__(kNormThreads) void sumsq_partial_kernel(const NormBatch B, double* __restrict__ partials)
{
    __shared__ double wsum[kNormThreads / 64];
    const uint32_t chunk = blockIdx.x;
    const uint32_t ti = find_tensor(B.chunk_start, B.n_tensors, chunk);
    const uint16_t* g = B.t[ti].g;
    const uint64_t numel = B.t[ti].numel;
    const uint64_t nblk = (numel + 7) >> 3;
    const uint64_t bchunk = (uint64_t)(chunk - B.chunk_start[ti]) * (uint64_t)(kNormThreads * kNormIters);
    const uint64_t bfirst = bchunk + threadIdx.x;
    const rsrc_t rg = chunk_rsrc<uint16_t>(g, (int64_t)(bchunk << 3), kNormChunkElems);

    double acc = 0.0;
#pragma unroll 4
    for (int it = 0; it < kNormIters; ++it) {
        const uint64_t b = bfirst + (uint64_t)it * kNormThreads;
        if (b >= nblk) break;
        const int64_t l0 = (int64_t)(b << 3);
        const bool full = block_inside(l0, numel);
        float x[8];
        unpack8(full ? buf_load16<true>(rg, (uint32_t)(it * kNormThreads + threadIdx.x) * 16u)
                     : load8_bf16<false>(g, l0, numel, false), x);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const double xd = (double)x[j];
            acc = __builtin_fma(xd, xd, acc);   // product exact (8-bit significands): one rounding
        }
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = wsum[0];
#pragma unroll
        for (int w = 1; w < kNormThreads / 64; ++w) s += wsum[w];
        partials[B.partial_base + chunk] = s;
    }
}

// Intermediate pass for very many partial sums: workgroup w adds in[w*kReduceFan ...) in a fixed
// order and writes out[w].
__global__ __launch_bounds__(kReduceThreads) void sumsq_reduce_kernel(const double* __restrict__ in, uint32_t n_in,
                                                                     double* __restrict__ out)
{
    __shared__ double wsum[kReduceThreads / 64];
    const uint64_t base = (uint64_t)blockIdx.x * kReduceFan;
    double acc = 0.0;
#pragma unroll 4
    for (int k = 0; k < kReduceFan / kReduceThreads; ++k) {
        const uint64_t i = base + (uint64_t)k * kReduceThreads + threadIdx.x;
        if (i < n_in) acc += in[i];
    }
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = wsum[0];
#pragma unroll
        for (int w = 1; w < kReduceThreads / 64; ++w) t += wsum[w];
        out[blockIdx.x] = t;
    }
}

// Pass 2: one workgroup adds the partial sums in a fixed order and writes (float) sqrt(S) to `out`
// and/or S itself to `out_sumsq` (either may be null).
__global__ __launch_bounds__(kFinalThreads) void sumsq_final_kernel(const double* __restrict__ partials,
                                                                   uint32_t n_partials, float* __restrict__ out,
                                                                   double* __restrict__ out_sumsq)
{
    __shared__ double wsum[kFinalThreads / 64];
    double acc = 0.0;
#pragma unroll 8
    for (uint32_t i = threadIdx.x; i < n_partials; i += kFinalThreads) acc += partials[i];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kFinalThreads / 64; ++w) s += wsum[w];
        if (out) *out = (float)__builtin_sqrt(s);
        if (out_sumsq) *out_sumsq = s;
    }
}

}  // namespace sr
