// Host side of the C ABI declared in include/sradamw.h: argument validation, the scalars of one
// step (formed in binary64, rounded once), packing of the multi-tensor chunk tables into kernel
// argument batches, and the launches on the caller's stream.  No device memory is allocated and
// nothing synchronises with the host.
#include "../../include/sradamw.h"
#include "sr_kernels.h"
#include "sr_host.h"

#include <atomic>
#include <cmath>
#include <cstring>
#include <mutex>

namespace {

using namespace sr;
using sr_host::blocks_spanned;
using sr_host::chunks_of;
using sr_host::range_wraps;
using sr_host::split_tensor;

thread_local int g_last_hip_error = 0;

inline int hip_fail(hipError_t e)
{
    g_last_hip_error = (int)e;
    return SR_ERR_HIP;
}

// Launch with the launch's own status (a status left behind by an unrelated earlier call of the
// application on this thread is neither reported nor cleared).  Argument types are taken from the
// kernel's signature, so every argument is converted before its address is passed.
template <class T> struct same_type { using type = T; };
template <class... P>
inline hipError_t launch_lds(void (*kernel)(P...), uint32_t grid, uint32_t block, uint32_t lds_bytes,
                             hipStream_t stream, typename same_type<P>::type... args)
{
    void* ptrs[] = {const_cast<void*>(static_cast<const void*>(&args))...};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), dim3(grid), dim3(block), ptrs, lds_bytes, stream);
}
template <class... P>
inline hipError_t launch(void (*kernel)(P...), uint32_t grid, uint32_t block, hipStream_t stream,
                         typename same_type<P>::type... args)
{
    return launch_lds(kernel, grid, block, 0u, stream, args...);
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// beta^t by repeated squaring in binary64.
double pow_uint(double base, uint32_t e)
{
    double r = 1.0;
    for (; e; e >>= 1) {
        if (e & 1u) r *= base;
        base *= base;
    }
    return r;
}

// Nontemporal loads and stores in the streaming kernels (measured +12% on the update).
constexpr bool kNT = true;
// Blocks per chunk (= per workgroup): BF16 moments, a lane owns one block; binary32 moments, a lane
// owns half a block.
constexpr uint64_t kBlocksPerChunkBf16 = (uint64_t)kThreads;
constexpr uint64_t kBlocksPerChunkFp32 = (uint64_t)kThreads / 2;
// A dispatch packet counts its grid in work-items with 32 bits, so a launch of T-lane workgroups
// holds at most (2^32 - 1) / T of them.  Larger jobs are cut into several launches (tensors into
// pieces at counter-block boundaries: a piece is itself a slice with its own elem_offset, so the
// result does not depend on the cut).  Tests lower the limit to reach those paths with small inputs.
std::atomic<uint32_t> g_launch_limit{0};
inline uint32_t max_grid(uint32_t threads)
{
    const uint32_t hw = 0xFFFFFFFFu / threads;
    const uint32_t lim = g_launch_limit.load(std::memory_order_relaxed);
    return lim && lim < hw ? lim : hw;
}
// Test switch: every wave of the 8-bit conversions takes the integer path.
std::atomic<uint32_t> g_fp8_integer{0};

// Waves resident per CU.  A stream that mixes reads and writes runs FASTER on MI355X with fewer
// waves in flight than the 32 single-wave workgroups a CU can hold: each kernel class below states
// how many it lets reside, and the launch reserves that share of the CU's 160 KiB of LDS per
// workgroup (LDS that no kernel touches, granted in units of 1280 bytes: sr_host::occupancy_lds)
// so that the hardware admits no more.  0 = no cap.  The debug hook overrides the number for
// measurements.
std::atomic<uint32_t> g_resident_waves{0};
inline uint32_t occupancy_lds(uint32_t class_default)
{
    const uint32_t forced = g_resident_waves.load(std::memory_order_relaxed);
    return sr_host::occupancy_lds(forced ? forced : class_default);
}
constexpr uint32_t kWavesUpdateBf16 = SR_TUNE_WAVES_BF16;    // BF16 moments (14 bytes per element)
constexpr uint32_t kWavesUpdateKahan = SR_TUNE_WAVES_KAHAN;  // BF16 moments + BF16 compensation (18)
constexpr uint32_t kWavesUpdateFp32 = SR_TUNE_WAVES_FP32;    // binary32 moments / master parameters
constexpr uint32_t kWavesUpdateFp8 = SR_TUNE_WAVES_FP8M;     // 8-bit moments
constexpr uint32_t kWavesCast = SR_TUNE_WAVES_CAST;          // the standalone cast to BF16
constexpr uint32_t kWavesCast8 = SR_TUNE_WAVES_CAST8;        // the standalone cast to an 8-bit format
constexpr uint32_t kWavesAcc = SR_TUNE_WAVES_ACC;            // gradient accumulation

template <uint32_t F, bool VAR>
hipError_t launch_adamw_v(bool clip, const AdamwBatch& batch, uint32_t n_chunks, hipStream_t stream)
{
    const uint32_t lds = occupancy_lds(Mode<F>::fp32m ? kWavesUpdateFp32 : (Mode<F>::fp8m || Mode<F>::fp8p) ? kWavesUpdateFp8
                                       : Mode<F>::kahan ? kWavesUpdateKahan : kWavesUpdateBf16);
    return clip ? launch_lds(adamw_kernel<F, true, kNT, VAR>, n_chunks, kThreads, lds, stream, batch)
                : launch_lds(adamw_kernel<F, false, kNT, VAR>, n_chunks, kThreads, lds, stream, batch);
}

// The default arithmetic runs in kernels compiled without the variant branches.
template <uint32_t F>
hipError_t launch_adamw(bool clip, const AdamwBatch& batch, uint32_t n_chunks, hipStream_t stream)
{
    return batch.s.variant ? launch_adamw_v<F, true>(clip, batch, n_chunks, stream)
                           : launch_adamw_v<F, false>(clip, batch, n_chunks, stream);
}

// The flag combinations that exist as kernels (normalised: RNE_MOMENTS dropped with FP32 moments).
hipError_t launch_adamw_variant(uint32_t flags, bool clip, const AdamwBatch& b, uint32_t n, hipStream_t s)
{
    switch (flags) {
        case 0u:                                              return launch_adamw<0u>(clip, b, n, s);
        case SR_FLAG_RNE_MOMENTS:                             return launch_adamw<SR_FLAG_RNE_MOMENTS>(clip, b, n, s);
        case SR_FLAG_RNE_PARAMS:                              return launch_adamw<SR_FLAG_RNE_PARAMS>(clip, b, n, s);
        case SR_FLAG_RNE_PARAMS | SR_FLAG_RNE_MOMENTS:        return launch_adamw<SR_FLAG_RNE_PARAMS | SR_FLAG_RNE_MOMENTS>(clip, b, n, s);
        case SR_FLAG_FP32_MOMENTS:                            return launch_adamw<SR_FLAG_FP32_MOMENTS>(clip, b, n, s);
        case SR_FLAG_FP32_MOMENTS | SR_FLAG_RNE_PARAMS:       return launch_adamw<SR_FLAG_FP32_MOMENTS | SR_FLAG_RNE_PARAMS>(clip, b, n, s);
        case SR_FLAG_FP32_MOMENTS | SR_FLAG_MASTER_FP32:      return launch_adamw<SR_FLAG_FP32_MOMENTS | SR_FLAG_MASTER_FP32>(clip, b, n, s);
        case SR_FLAG_KAHAN:                                   return launch_adamw<SR_FLAG_KAHAN>(clip, b, n, s);
        case SR_FLAG_FP8_MOMENTS:                             return launch_adamw<SR_FLAG_FP8_MOMENTS>(clip, b, n, s);
        case SR_FLAG_FP8_MOMENTS | SR_FLAG_RNE_PARAMS:        return launch_adamw<SR_FLAG_FP8_MOMENTS | SR_FLAG_RNE_PARAMS>(clip, b, n, s);
        case SR_FLAG_FP8_PARAMS:                              return launch_adamw<SR_FLAG_FP8_PARAMS>(clip, b, n, s);
        case SR_FLAG_FP8_PARAMS | SR_FLAG_FP8_MOMENTS:        return launch_adamw<SR_FLAG_FP8_PARAMS | SR_FLAG_FP8_MOMENTS>(clip, b, n, s);
        default:                                              return hipErrorInvalidValue;   // unreachable after validation
    }
}

// Scratch of the entry point that allocates nothing (grad_global_norm_static): the partial sums
// of the norm's first pass.  One copy per device that loads this library, held until the process
// ends.  In host code the array's name is only a handle: its device address is looked up once per
// device (with that device current) and only that address is passed to kernels.
constexpr uint64_t kStaticPartials = SR_STATIC_SCRATCH_BYTES / sizeof(double);
static __device__ __align__(256) unsigned char scratch[SR_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double* g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of `scratch`.  The first call on a device asks the runtime for the
// symbol's address (no allocation; do it outside a stream capture); later calls read the table.
int static_scratch(double** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return SR_ERR_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!p) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = static_cast<double*>(p);
    }
    *out = g_scratch_ptr[dev];
    return SR_OK;
}

}  // namespace

extern "C" {

int sr_version(void) { return 100; }

int sr_last_hip_error(void) { return g_last_hip_error; }

void sr_debug_set(uint32_t key, uint32_t value)
{
    switch (key) {
        case SR_DEBUG_LAUNCH_LIMIT:   g_launch_limit.store(value, std::memory_order_relaxed); break;
        case SR_DEBUG_FP8_INTEGER:    g_fp8_integer.store(value, std::memory_order_relaxed); break;
        case SR_DEBUG_RESIDENT_WAVES: g_resident_waves.store(value, std::memory_order_relaxed); break;
        default: break;
    }
}

int sr_stream_probe(void* d_p, const void* d_g, void* d_m, void* d_v, uint64_t numel, void* stream)
{
    const uint64_t nblk = numel >> 3;                 // whole blocks only; a tail is left untouched
    if (nblk == 0) return SR_OK;
    if (!d_p || !d_g || !d_m || !d_v) return SR_ERR_NULL;
    if (!aligned(d_p, 2) || !aligned(d_g, 2) || !aligned(d_m, 2) || !aligned(d_v, 2)) return SR_ERR_ALIGN;
    const uint64_t wgs = (nblk + kThreads - 1) / kThreads;
    const uint32_t mg = max_grid(kThreads);
    for (uint64_t w0 = 0; w0 < wgs; w0 += mg) {
        const uint32_t grid = (uint32_t)(wgs - w0 < mg ? wgs - w0 : mg);
        const hipError_t e = launch_lds(stream_probe_kernel, grid, kThreads, occupancy_lds(kWavesUpdateBf16), static_cast<hipStream_t>(stream),
                                    static_cast<uint16_t*>(d_p), static_cast<const uint16_t*>(d_g),
                                    static_cast<uint16_t*>(d_m), static_cast<uint16_t*>(d_v), nblk, w0, 0u);
        if (e != hipSuccess) return hip_fail(e);
    }
    return SR_OK;
}

int sr_stream_probe_fp8m(void* d_p, const void* d_g, void* d_m8, void* d_v8, uint64_t numel, void* stream)
{
    const uint64_t nblk = numel >> 3;                 // whole blocks only; a tail is left untouched
    if (nblk == 0) return SR_OK;
    if (!d_p || !d_g || !d_m8 || !d_v8) return SR_ERR_NULL;
    if (!aligned(d_p, 2) || !aligned(d_g, 2)) return SR_ERR_ALIGN;
    const uint64_t wgs = (nblk + kThreads - 1) / kThreads;
    const uint32_t mg = max_grid(kThreads);
    for (uint64_t w0 = 0; w0 < wgs; w0 += mg) {
        const uint32_t grid = (uint32_t)(wgs - w0 < mg ? wgs - w0 : mg);
        const hipError_t e = launch_lds(stream_probe_fp8m_kernel, grid, kThreads, occupancy_lds(kWavesUpdateFp8), static_cast<hipStream_t>(stream),
                                    static_cast<uint16_t*>(d_p), static_cast<const uint16_t*>(d_g),
                                    static_cast<uint8_t*>(d_m8), static_cast<uint8_t*>(d_v8), nblk, w0, 0u);
        if (e != hipSuccess) return hip_fail(e);
    }
    return SR_OK;
}

const char* sr_strerror(int code)
{
    switch (code) {
        case SR_OK:            return "ok";
        case SR_ERR_NULL:      return "a required pointer is NULL";
        case SR_ERR_ARG:       return "invalid argument (step, hyper-parameter, flag, scale exponent, reserved field or index range)";
        case SR_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SR_ERR_ALIGN:     return "tensor pointer not aligned to its element size";
        case SR_ERR_HIP:       return "HIP launch failed (see sr_last_hip_error)";
        case SR_ERR_SIZE:      return "the list needs more partial sums than the library's static scratch holds";
        default:               return "unknown error code";
    }
}

uint64_t sr_workspace_bytes(uint32_t n_tensors, uint64_t total_numel)
{
    const uint64_t chunks = total_numel / (uint64_t)kNormChunkElems + (uint64_t)n_tensors + 1;
    return (chunks * sizeof(double) + 255u) & ~(uint64_t)255u;
}

int sr_cast_f32_bf16(const float* d_src, void* d_dst, uint64_t n, uint64_t seed, uint32_t step,
                     uint32_t tensor_id, void* stream)
{
    if (n == 0) return SR_OK;
    if (!d_src || !d_dst) return SR_ERR_NULL;
    if (!aligned(d_src, 4) || !aligned(d_dst, 2)) return SR_ERR_ALIGN;
    const uint64_t chunks = (n + (uint64_t)kCastChunkElems - 1) / (uint64_t)kCastChunkElems;
    const uint32_t mg = max_grid(kThreads);
    for (uint64_t c0 = 0; c0 < chunks; c0 += mg) {
        const uint32_t grid = (uint32_t)(chunks - c0 < mg ? chunks - c0 : mg);
        const hipError_t e = launch_lds(cast_kernel<kNT>, grid, kThreads, occupancy_lds(kWavesCast), static_cast<hipStream_t>(stream), d_src,
                                    static_cast<uint16_t*>(d_dst), n, c0, (uint32_t)(seed & 0xFFFFFFFFu),
                                    (uint32_t)(seed >> 32), step, tensor_id);
        if (e != hipSuccess) return hip_fail(e);
    }
    return SR_OK;
}

int sr_cast_f32_fp8(const float* d_src, void* d_dst, uint64_t n, uint32_t format, uint64_t seed,
                    uint32_t step, uint32_t tensor_id, void* stream)
{
    if (format != SR_FP8_E4M3 && format != SR_FP8_E5M2) return SR_ERR_ARG;
    if (n == 0) return SR_OK;
    if (!d_src || !d_dst) return SR_ERR_NULL;
    if (!aligned(d_src, 4)) return SR_ERR_ALIGN;
    if (n > (1ull << 61)) return SR_ERR_ARG;                        // block index must fit 29 + 32 bits
    const uint64_t chunks = (n + (uint64_t)kFp8ChunkElems - 1) / (uint64_t)kFp8ChunkElems;
    const uint32_t mg = max_grid(kThreads);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t lo = (uint32_t)(seed & 0xFFFFFFFFu), hi = (uint32_t)(seed >> 32);
    for (uint64_t c0 = 0; c0 < chunks; c0 += mg) {
        const uint32_t grid = (uint32_t)(chunks - c0 < mg ? chunks - c0 : mg);
        const uint32_t lds = occupancy_lds(kWavesCast8);
        const uint32_t integer_path = g_fp8_integer.load(std::memory_order_relaxed) ? 1u : 0u;
        const hipError_t e = format == SR_FP8_E4M3
            ? launch_lds(cast_fp8_kernel<0, kNT>, grid, kThreads, lds, s, d_src, static_cast<uint8_t*>(d_dst), n, c0, lo, hi, step, tensor_id, integer_path)
            : launch_lds(cast_fp8_kernel<1, kNT>, grid, kThreads, lds, s, d_src, static_cast<uint8_t*>(d_dst), n, c0, lo, hi, step, tensor_id, integer_path);
        if (e != hipSuccess) return hip_fail(e);
    }
    return SR_OK;
}

// Both norm entry points and the variant that brings its own scratch: `partials` is device memory
// for `capacity` binary64 partial sums (the caller's workspace, or the library's static array).
static int sum_of_squares(const sr_tensor_t* tensors, uint32_t n_tensors, float* d_norm_out, double* d_sumsq_out,
                          double* partials, uint64_t capacity, void* stream)
{
    if (!d_norm_out && !d_sumsq_out) return SR_ERR_NULL;
    if (n_tensors && !tensors) return SR_ERR_NULL;
    if (!aligned(d_norm_out, 4) || !aligned(d_sumsq_out, 8)) return SR_ERR_ALIGN;
    uint64_t total_chunks = 0;
    for (uint32_t i = 0; i < n_tensors; ++i) {
        if (tensors[i].numel == 0) continue;
        if (!tensors[i].g) return SR_ERR_NULL;
        if (!aligned(tensors[i].g, 2)) return SR_ERR_ALIGN;
        uint64_t nch = 0;
        if (!chunks_of(tensors[i].numel, kNormChunkElems, &nch)) return SR_ERR_ARG;
        total_chunks += nch;
        if (total_chunks > 0xFFFFFFFFull) return SR_ERR_ARG;      // partial sums are indexed with 32 bits
    }
    if (total_chunks) {
        if (!partials || !aligned(partials, 8)) return SR_ERR_WORKSPACE;
        if (capacity < total_chunks) return SR_ERR_WORKSPACE;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);

    NormBatch batch;
    std::memset(&batch, 0, sizeof(batch));
    uint32_t nb = 0, chunks_in_batch = 0, base = 0;
    auto flush = [&]() -> hipError_t {
        if (nb == 0) return hipSuccess;
        batch.n_tensors = nb;
        batch.partial_base = base;
        batch.chunk_start[nb] = chunks_in_batch;
        const hipError_t e = launch(sumsq_partial_kernel, chunks_in_batch, kNormThreads, s, batch, partials);
        base += chunks_in_batch;
        nb = 0; chunks_in_batch = 0;
        return e;
    };
    const uint32_t mg = max_grid(kNormThreads);
    const uint64_t piece_elems = (uint64_t)mg * kNormChunkElems;      // whole chunks: same partial sums however cut
    for (uint32_t i = 0; i < n_tensors; ++i) {
        for (uint64_t off = 0; off < tensors[i].numel; off += piece_elems) {
            const uint64_t numel = tensors[i].numel - off < piece_elems ? tensors[i].numel - off : piece_elems;
            const uint32_t nch = (uint32_t)((numel + kNormChunkElems - 1) / kNormChunkElems);
            if (nb == kNormMaxBatch || (uint64_t)chunks_in_batch + nch > mg) {
                const hipError_t e = flush();
                if (e != hipSuccess) return hip_fail(e);
            }
            batch.t[nb].g = static_cast<const uint16_t*>(tensors[i].g) + off;
            batch.t[nb].numel = numel;
            batch.chunk_start[nb] = chunks_in_batch;
            chunks_in_batch += nch;
            ++nb;
        }
    }
    hipError_t e = flush();
    if (e != hipSuccess) return hip_fail(e);
    e = launch(sumsq_final_kernel, 1, kFinalThreads, s, partials, (uint32_t)total_chunks, d_norm_out, d_sumsq_out);
    return e == hipSuccess ? SR_OK : hip_fail(e);
}

int grad_global_norm(const sr_tensor_t* tensors, uint32_t n_tensors, float* d_norm_out,
                     void* d_workspace, uint64_t workspace_bytes, void* stream)
{
    return sum_of_squares(tensors, n_tensors, d_norm_out, nullptr, static_cast<double*>(d_workspace),
                          workspace_bytes / sizeof(double), stream);
}

int grad_sum_of_squares(const sr_tensor_t* tensors, uint32_t n_tensors, double* d_sumsq_out,
                        void* d_workspace, uint64_t workspace_bytes, void* stream)
{
    return sum_of_squares(tensors, n_tensors, nullptr, d_sumsq_out, static_cast<double*>(d_workspace),
                          workspace_bytes / sizeof(double), stream);
}

int grad_global_norm_static(const sr_tensor_t* tensors, uint32_t n_tensors, float* d_norm_out, void* stream)
{
    uint64_t total_chunks = 0;
    for (uint32_t i = 0; tensors && i < n_tensors; ++i) {
        uint64_t nch = 0;
        if (!chunks_of(tensors[i].numel, kNormChunkElems, &nch)) return SR_ERR_ARG;
        total_chunks += nch;
        if (total_chunks > kStaticPartials) return SR_ERR_SIZE;
    }
    double* partials = nullptr;
    const int rc = static_scratch(&partials);
    if (rc != SR_OK) return rc;
    return sum_of_squares(tensors, n_tensors, d_norm_out, nullptr, partials, kStaticPartials, stream);
}

uint64_t sr_accumulate_workspace_bytes(uint32_t n_tensors, uint64_t total_numel)
{
    // first-level partials plus the folded levels (each kReduceFan times smaller)
    // a tensor of numel elements whose counter blocks start mid-block spans up to numel/512 + 2 chunks
    uint64_t chunks = total_numel / (uint64_t)kAccChunkElems + 2 * (uint64_t)n_tensors + 1;
    uint64_t total = chunks;
    while (chunks > kReduceAbove) { chunks = (chunks + kReduceFan - 1) / kReduceFan; total += chunks; }
    return (total * sizeof(double) + 255u) & ~(uint64_t)255u;
}

int sr_grad_accumulate(const sr_accum_t* tensors, uint32_t n_tensors, float scale, uint32_t micro_step,
                       uint64_t seed, uint32_t flags, float* d_norm_out, void* d_workspace,
                       uint64_t workspace_bytes, void* stream)
{
    if (n_tensors && !tensors) return SR_ERR_NULL;
    if (flags & ~(SR_ACC_RNE | SR_ACC_FIRST)) return SR_ERR_ARG;
    if (!std::isfinite(scale)) return SR_ERR_ARG;
    if (d_norm_out && !aligned(d_norm_out, 4)) return SR_ERR_ALIGN;
    const uint64_t blocks_per_chunk = (uint64_t)kAccThreads * kAccIters;
    uint64_t total_chunks = 0;
    for (uint32_t i = 0; i < n_tensors; ++i) {
        const sr_accum_t& t = tensors[i];
        if (t.reserved != 0) return SR_ERR_ARG;
        if (t.numel == 0) continue;
        if (!t.acc || !t.grad) return SR_ERR_NULL;
        if (!aligned(t.acc, 2) || !aligned(t.grad, 2)) return SR_ERR_ALIGN;
        if (range_wraps(t.elem_offset, t.numel)) return SR_ERR_ARG;
        const uint64_t nblk = blocks_spanned(t.numel, t.elem_offset);
        total_chunks += (nblk + blocks_per_chunk - 1) / blocks_per_chunk;
        if (total_chunks > 0xFFFFFFFFull) return SR_ERR_ARG;      // partial sums are indexed with 32 bits
    }
    if (d_norm_out && total_chunks) {
        uint64_t need = total_chunks, level = total_chunks;
        while (level > kReduceAbove) { level = (level + kReduceFan - 1) / kReduceFan; need += level; }
        if (!d_workspace || !aligned(d_workspace, 8)) return SR_ERR_WORKSPACE;
        if (workspace_bytes < need * sizeof(double)) return SR_ERR_WORKSPACE;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    double* partials = static_cast<double*>(d_workspace);

    AccBatch batch;
    std::memset(&batch, 0, sizeof(batch));
    batch.scale = scale;
    batch.seed_lo = (uint32_t)(seed & 0xFFFFFFFFu);
    batch.seed_hi = (uint32_t)(seed >> 32);
    batch.micro_step = micro_step;
    batch.mode = (flags & SR_ACC_RNE ? ACC_RNE : 0u) | (flags & SR_ACC_FIRST ? ACC_FIRST : 0u) |
                 (d_norm_out ? ACC_NORM : 0u);
    uint32_t nb = 0, chunks_in_batch = 0, base = 0;
    auto flush = [&]() -> hipError_t {
        if (nb == 0) return hipSuccess;
        batch.n_tensors = nb;
        batch.partial_base = base;
        batch.chunk_start[nb] = chunks_in_batch;
        const hipError_t e = launch_lds(accumulate_kernel, chunks_in_batch, kAccThreads, occupancy_lds(kWavesAcc), s, batch, partials);
        base += chunks_in_batch;
        nb = 0; chunks_in_batch = 0;
        return e;
    };
    const uint32_t mg = max_grid(kAccThreads);
    for (uint32_t i = 0; i < n_tensors; ++i) {
        const sr_accum_t& t = tensors[i];
        if (t.numel == 0) continue;
        const hipError_t pe = split_tensor(t.numel, t.elem_offset, (uint64_t)mg * blocks_per_chunk,
                                           [&](uint64_t local, uint64_t numel, uint64_t goff) -> hipError_t {
            const uint64_t nblk = blocks_spanned(numel, goff);
            const uint32_t nch = (uint32_t)((nblk + blocks_per_chunk - 1) / blocks_per_chunk);
            if (nb == kAccMaxBatch || (uint64_t)chunks_in_batch + nch > mg) {
                const hipError_t e = flush();
                if (e != hipSuccess) return e;
            }
            AccDesc& d = batch.t[nb];
            d.acc = static_cast<uint16_t*>(t.acc) + local;
            d.g = static_cast<const uint16_t*>(t.grad) + local;
            d.numel = numel;
            d.elem_offset = goff;
            d.tensor_id = t.tensor_id;
            d.pad_ = 0;
            batch.chunk_start[nb] = chunks_in_batch;
            chunks_in_batch += nch;
            ++nb;
            return hipSuccess;
        });
        if (pe != hipSuccess) return hip_fail(pe);
    }
    hipError_t e = flush();
    if (e != hipSuccess) return hip_fail(e);
    if (d_norm_out) {
        // fold the partial sums level by level (each level behind the previous one in the
        // workspace), then one workgroup finishes
        uint32_t n_level = (uint32_t)total_chunks;
        double* level = partials;
        while (n_level > kReduceAbove) {
            const uint32_t n_next = (n_level + kReduceFan - 1) / kReduceFan;
            e = launch(sumsq_reduce_kernel, n_next, kReduceThreads, s, level, n_level, level + n_level);
            if (e != hipSuccess) return hip_fail(e);
            level += n_level;
            n_level = n_next;
        }
        e = launch(sumsq_final_kernel, 1, kFinalThreads, s, level, n_level, d_norm_out, nullptr);
        if (e != hipSuccess) return hip_fail(e);
    }
    return SR_OK;
}

int sr_adamw_step(const sr_tensor_t* tensors, uint32_t n_tensors, const sr_hyper_t* hyper,
                  uint32_t step, uint64_t seed, uint32_t flags, const float* d_grad_norm,
                  float max_norm, void* stream)
{
    if (!hyper) return SR_ERR_NULL;
    if (n_tensors && !tensors) return SR_ERR_NULL;
    if (step == 0) return SR_ERR_ARG;
    if (flags & ~(SR_FLAG_FP32_MOMENTS | SR_FLAG_RNE_MOMENTS | SR_FLAG_RNE_PARAMS | SR_FLAG_MASTER_FP32 |
                  SR_FLAG_KAHAN | SR_FLAG_EPS_IN_ROOT | SR_FLAG_DIV_BIAS | SR_FLAG_FP8_MOMENTS |
                  SR_FLAG_SKIP_NONFINITE_NORM | SR_FLAG_FP8_PARAMS))
        return SR_ERR_ARG;
    // a guard of the clipped step, not a strategy: it selects no kernel
    const bool skip_nonfinite = (flags & SR_FLAG_SKIP_NONFINITE_NORM) != 0;
    flags &= ~SR_FLAG_SKIP_NONFINITE_NORM;
    // variants of the arithmetic combine with any strategy and do not select a kernel
    uint32_t variant = 0;
    if (flags & SR_FLAG_EPS_IN_ROOT) variant |= VARIANT_EPS_IN_ROOT;
    if (flags & SR_FLAG_DIV_BIAS) variant |= VARIANT_DIV_BIAS;
    flags &= ~(SR_FLAG_EPS_IN_ROOT | SR_FLAG_DIV_BIAS);
    if ((flags & SR_FLAG_MASTER_FP32) && flags != (SR_FLAG_MASTER_FP32 | SR_FLAG_FP32_MOMENTS)) return SR_ERR_ARG;
    if ((flags & SR_FLAG_KAHAN) && flags != SR_FLAG_KAHAN) return SR_ERR_ARG;
    if ((flags & SR_FLAG_FP8_PARAMS) && (flags & ~(SR_FLAG_FP8_PARAMS | SR_FLAG_FP8_MOMENTS))) return SR_ERR_ARG;
    if ((flags & SR_FLAG_FP8_MOMENTS) && (flags & ~(SR_FLAG_FP8_MOMENTS | SR_FLAG_RNE_PARAMS | SR_FLAG_FP8_PARAMS))) return SR_ERR_ARG;
    const sr_hyper_t h = *hyper;
    if (!std::isfinite(h.lr) || !std::isfinite(h.eps) || !std::isfinite(h.weight_decay) ||
        !std::isfinite(h.beta1) || !std::isfinite(h.beta2)) return SR_ERR_ARG;
    if (!(h.beta1 >= 0.0f && h.beta1 < 1.0f) || !(h.beta2 >= 0.0f && h.beta2 < 1.0f)) return SR_ERR_ARG;
    if (h.eps < 0.0f) return SR_ERR_ARG;
    const bool clip = d_grad_norm != nullptr;
    if (clip) {
        if (!std::isfinite(max_norm) || !(max_norm > 0.0f)) return SR_ERR_ARG;
        if (!aligned(d_grad_norm, 4)) return SR_ERR_ALIGN;
    }
    const bool fp32m = (flags & SR_FLAG_FP32_MOMENTS) != 0;
    if (fp32m) flags &= ~SR_FLAG_RNE_MOMENTS;                      // no BF16 moment write-back to round
    const bool master = (flags & SR_FLAG_MASTER_FP32) != 0;
    const bool kahan = (flags & SR_FLAG_KAHAN) != 0;
    const bool fp8m = (flags & SR_FLAG_FP8_MOMENTS) != 0;
    const bool fp8p = (flags & SR_FLAG_FP8_PARAMS) != 0;
    const uintptr_t moment_align = fp32m ? 4 : fp8m ? 1 : 2, param_align = fp8p ? 1 : 2;

    // Validate the whole list before anything is enqueued.
    for (uint32_t i = 0; i < n_tensors; ++i) {
        const sr_tensor_t& t = tensors[i];
        if (t.reserved != 0) return SR_ERR_ARG;
        if (fp8m) {
            if (t.m_exp < -100 || t.m_exp > 100 || t.v_exp < -100 || t.v_exp > 100) return SR_ERR_ARG;
        } else if (t.m_exp != 0 || t.v_exp != 0) {
            return SR_ERR_ARG;
        }
        if (fp8p ? (t.p_exp < -100 || t.p_exp > 100) : t.p_exp != 0) return SR_ERR_ARG;
        if (t.numel == 0) continue;
        if (!t.p || !t.g || !t.m || !t.v) return SR_ERR_NULL;
        if ((master || kahan) && !t.aux) return SR_ERR_NULL;
        if (!aligned(t.p, param_align) || !aligned(t.g, 2) || !aligned(t.m, moment_align) || !aligned(t.v, moment_align))
            return SR_ERR_ALIGN;
        if ((master && !aligned(t.aux, 4)) || (kahan && !aligned(t.aux, 2))) return SR_ERR_ALIGN;
        if (range_wraps(t.elem_offset, t.numel)) return SR_ERR_ARG;
        // an 8-bit parameter draws a 32-bit word per element: its stream counts blocks of four
        // elements, whose index must leave the counter's three stream bits free
        if (fp8p && t.elem_offset + t.numel > (1ull << 63)) return SR_ERR_ARG;
    }

    AdamwBatch batch;
    std::memset(&batch, 0, sizeof(batch));
    StepScalars& S = batch.s;
    S.beta1 = h.beta1;
    S.beta2 = h.beta2;
    S.omb1 = (float)(1.0 - (double)h.beta1);
    S.omb2 = (float)(1.0 - (double)h.beta2);
    S.rbc1 = (float)(1.0 / (1.0 - pow_uint((double)h.beta1, step)));
    S.rbc2 = (float)(1.0 / (1.0 - pow_uint((double)h.beta2, step)));
    S.bc1 = (float)(1.0 - pow_uint((double)h.beta1, step));
    S.bc2 = (float)(1.0 - pow_uint((double)h.beta2, step));
    S.variant = variant | (fp8m && g_fp8_integer.load(std::memory_order_relaxed) ? VARIANT_FP8_INTEGER : 0u);
    S.lr = h.lr;
    S.eps = h.eps;
    S.lw = (float)((double)h.lr * (double)h.weight_decay);
    S.max_norm = max_norm;
    S.d_norm = d_grad_norm;
    S.skip_nonfinite = (skip_nonfinite && clip) ? 1u : 0u;
    S.seed_lo = (uint32_t)(seed & 0xFFFFFFFFu);
    S.seed_hi = (uint32_t)(seed >> 32);
    S.step = step;

    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t nb = 0, chunks_in_batch = 0;
    auto flush = [&]() -> hipError_t {
        if (nb == 0) return hipSuccess;
        S.n_tensors = nb;
        batch.chunk_start[nb] = chunks_in_batch;
        const hipError_t e = launch_adamw_variant(flags, clip, batch, chunks_in_batch, s);
        nb = 0; chunks_in_batch = 0;
        return e;
    };
    const uint32_t mg = max_grid(kThreads);
    const uint64_t per_chunk = fp32m ? kBlocksPerChunkFp32 : kBlocksPerChunkBf16;
    const uint64_t moment_size = fp32m ? 4 : fp8m ? 1 : 2, aux_size = master ? 4 : 2, param_size = fp8p ? 1 : 2;
    for (uint32_t i = 0; i < n_tensors; ++i) {
        const sr_tensor_t& t = tensors[i];
        if (t.numel == 0) continue;
        const hipError_t pe = split_tensor(t.numel, t.elem_offset, (uint64_t)mg * per_chunk,
                                           [&](uint64_t local, uint64_t numel, uint64_t goff) -> hipError_t {
            const uint64_t nblk = blocks_spanned(numel, goff);
            const uint32_t nch = (uint32_t)((nblk + per_chunk - 1) / per_chunk);
            if (nb == kMaxBatch || (uint64_t)chunks_in_batch + nch > mg) {
                const hipError_t e = flush();
                if (e != hipSuccess) return e;
            }
            TensorDesc& d = batch.t[nb];
            d.p = reinterpret_cast<uint16_t*>(static_cast<char*>(t.p) + local * param_size);
            d.g = static_cast<const uint16_t*>(t.g) + local;
            d.m = static_cast<char*>(t.m) + local * moment_size;
            d.v = static_cast<char*>(t.v) + local * moment_size;
            d.aux = (master || kahan) ? static_cast<char*>(t.aux) + local * aux_size : nullptr;
            d.numel = numel;
            d.elem_offset = goff;
            d.tensor_id = t.tensor_id;
            d.flags = ((goff & 7u) == 0 ? DESC_VEC : 0u) |
                      (fp8m ? ((uint32_t)(uint8_t)t.m_exp << DESC_MEXP_SHIFT) | ((uint32_t)(uint8_t)t.v_exp << DESC_VEXP_SHIFT) : 0u) |
                      (fp8p ? (uint32_t)(uint8_t)t.p_exp << DESC_PEXP_SHIFT : 0u);
            batch.chunk_start[nb] = chunks_in_batch;
            chunks_in_batch += nch;
            ++nb;
            return hipSuccess;
        });
        if (pe != hipSuccess) return hip_fail(pe);
    }
    const hipError_t e = flush();
    return e == hipSuccess ? SR_OK : hip_fail(e);
}

}  // extern "C"
