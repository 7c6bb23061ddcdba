/*
 * sradamw.h -- C ABI of the MI355X (gfx950) SR-AdamW update library.
 *
 * The library implements the optimizer step of BF16+SR training
 * (arXiv 2502.20566, Algorithm 1, Section 3): an AdamW update computed in
 * binary32 over BF16 parameters, gradients and moments whose write-backs to
 * BF16 are stochastically rounded (Eq.(2), Section 2.1), with the random bits
 * taken from a stateless counter generator so that every data-parallel
 * replica rounds identically (Algorithm 1, lines 9 and 11).
 *
 * Conventions for every entry point
 *   - Pointers named d_* and every pointer inside sr_tensor_t are DEVICE
 *     pointers owned by the caller; all other pointers are HOST pointers that
 *     are read before the call returns and may be freed right after it.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work on it: no host synchronisation, no device
 *     allocation, no hidden state.  Results are ordered by the stream.  The
 *     calling thread's current device must be the device of the stream and
 *     of the tensors.
 *   - Return value: SR_OK (0) or a negative SR_ERR_* code.  Arguments are
 *     validated on the host first; on an argument error (every code but
 *     SR_ERR_HIP) nothing is enqueued.  SR_ERR_HIP means the runtime refused
 *     a launch.  A call that needs several launches (a list of more tensors
 *     than one launch takes, a job beyond one dispatch's size, the passes of
 *     a norm) enqueues them in list order and stops at the first refusal: the
 *     launches before it stay enqueued and will run, so a tensor list may then
 *     be updated in part (whole tensors from the front of the list, possibly a
 *     leading piece of one very large tensor), and a norm or sum output is not
 *     written.  The library cannot take enqueued work back; a caller that
 *     must recover keeps a copy of the state or treats the error as fatal for
 *     the step (a refused launch means the stream or device is unusable).
 *   - Sizes: any tensor that fits in device memory is accepted.  A launch
 *     holds at most 2^32 - 1 work-items; larger jobs (more than about 3.4e10
 *     elements of a BF16-moment list, 1.7e10 of an FP32-moment list or of a
 *     cast) are enqueued as several launches, with identical results.
 *   - Outputs depend only on the input bits, the hyper-parameters, `step`,
 *     `seed`, `tensor_id` and the element's index elem_offset + i -- never on
 *     launch geometry, list order, how a list is split over calls, pointer
 *     alignment or the rank that runs it.
 */
#ifndef SRADAMW_H
#define SRADAMW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SR_OK              0
#define SR_ERR_NULL      (-1)  /* a required pointer is NULL                              */
#define SR_ERR_ARG       (-2)  /* step == 0, beta outside [0,1), eps < 0, non-finite
                                  hyper-parameter, max_norm <= 0 with clipping, unknown
                                  or incompatible flags, non-zero reserved field, index
                                  range overflow                                          */
#define SR_ERR_WORKSPACE (-3)  /* workspace NULL, misaligned (8 bytes) or too small       */
#define SR_ERR_ALIGN     (-4)  /* a BF16 pointer not 2-byte / an FP32 pointer not 4-byte
                                  aligned (arrays of 8-bit codes may start at any byte).
                                  Nothing more is required: tensors may be views
                                  starting at any element of a larger buffer and keep the
                                  vector path                                             */
#define SR_ERR_HIP       (-5)  /* a launch failed; see sr_last_hip_error()                */
#define SR_ERR_SIZE      (-6)  /* the input needs more scratch than the static array of
                                  grad_global_norm_static holds                           */

/* bytes of the static device array behind grad_global_norm_static */
#define SR_STATIC_SCRATCH_BYTES 1048576u

/* flags of sr_adamw_step */
#define SR_FLAG_FP32_MOMENTS 1u /* m, v are binary32 and stored unrounded; SR on p only
                                   (the full-precision optimizer states of Section 3, last
                                   paragraph, and of the ablation in Appendix C)           */
#define SR_FLAG_RNE_MOMENTS  2u /* BF16 m, v written back with round-to-nearest-even,
                                   Eq.(1): the paper's own setting, SR on line 10 only.
                                   Ignored together with SR_FLAG_FP32_MOMENTS.             */
#define SR_FLAG_RNE_PARAMS   4u /* the parameter write-back is round-to-nearest-even too;
                                   with SR_FLAG_RNE_MOMENTS this is the "BF16" strategy of
                                   Section 5.1 (every tensor BF16, default rounding): no
                                   random bits are drawn                                   */
/* Comparison strategies that carry an auxiliary tensor in sr_tensor_t.aux (Section 5.1
   "Baselines" and the related work of Section 1).  Each must be the only flag set, except
   that SR_FLAG_MASTER_FP32 requires SR_FLAG_FP32_MOMENTS.                                 */
#define SR_FLAG_MASTER_FP32  8u /* O2-style mixed precision: aux = binary32 master
                                   parameters [numel], updated in binary32 and stored
                                   unrounded; m, v binary32; p (BF16, write-only) receives
                                   RNE(master), the model copy                             */
#define SR_FLAG_KAHAN       16u /* BF16 + Kahan summation on the parameter: aux = BF16
                                   compensation c [numel] (in/out, start it at zero).  With
                                   s the step's total update (plain result p - s):
                                   yk = (-s) - c; t = p + yk; p <- RNE(t);
                                   c <- RNE((p_new - p) - yk); m, v written with RNE       */

/* Variants of the arithmetic; combine with any of the above. */
#define SR_FLAG_EPS_IN_ROOT 32u /* denominator sqrt(v' rbc2 + eps) instead of
                                   sqrt(v' rbc2) + eps: eps inside the root, the form of the
                                   update in Appendix B                                    */
#define SR_FLAG_DIV_BIAS    64u /* bias corrections as the divisions of Algorithm 1 lines
                                   7-8 as printed, m'/(1-beta1^t) and v'/(1-beta2^t) with
                                   1-beta^t formed in binary64 and rounded once, instead of
                                   multiplications by the rounded reciprocals              */
/* Guard for clipped steps (clipping itself is not in the paper). */
#define SR_FLAG_SKIP_NONFINITE_NORM 256u /* with d_grad_norm: when the norm it holds is NaN
                                   or infinite (an overflowed or poisoned gradient) the
                                   step changes nothing -- p, m, v and aux keep their
                                   bits.  Without this flag the clip formula is applied
                                   as it stands: a NaN norm makes every p, m, v NaN, an
                                   infinite norm scales the gradient to zero while decay
                                   and moment decay still apply.  The caller still
                                   advances or repeats `step` as it sees fit.            */
/* A storage format of the moments (not one of the paper's strategies). */
#define SR_FLAG_FP8_MOMENTS 128u /* extension (the paper's conclusion names FP8 as the next
                                   target of SR and gives no design): m and v are 8-bit
                                   codes, one byte per element, m in E4M3 and v in E5M2
                                   (see sr_cast_f32_fp8 for the formats), each with a
                                   power-of-two scale per tensor given in the tensor's
                                   m_exp and v_exp fields: m = decode(m8) 2^-m_exp,
                                   v = decode(v8) 2^-v_exp, the update as for every other
                                   strategy, m8 <- Q_SR(m' 2^m_exp), v8 <- Q_SR(v' 2^v_exp)
                                   with the element's 16-bit draws of streams 1 and 2 in
                                   the top half of the 32-bit random word of
                                   sr_cast_f32_fp8's rule (the fraction is cut to 16
                                   bits).  10 bytes moved per element instead of 14.
                                   Combines with SR_FLAG_RNE_PARAMS, SR_FLAG_FP8_PARAMS,
                                   SR_FLAG_EPS_IN_ROOT, SR_FLAG_DIV_BIAS and
                                   SR_FLAG_SKIP_NONFINITE_NORM only.  Both write-backs
                                   saturate: a scaled m' beyond 448 is stored as 448, a scaled v'
                                   beyond 57344 (or one that Q_SR would round to E5M2's
                                   infinity) as 57344, so the state never holds an
                                   infinity.  NaN codes stay NaN codes; NaN signs and
                                   payloads are not specified.                          */

#define SR_FLAG_FP8_PARAMS 512u /* extension, the 8-bit write-back of the parameter that the
                                   paper's conclusion points to (no design is given there):
                                   p is held as E4M3 codes, one byte per element, with a
                                   power-of-two scale per tensor, p = decode(p8) 2^-p_exp;
                                   the update as for every other strategy;
                                   p8 <- Q_SR(y 2^p_exp) by the rule of sr_cast_f32_fp8
                                   (Eq.(2) on the E4M3 grid, the 20-bit draw from the top of
                                   the element's own 32-bit word: word i&3 of Philox block
                                   i>>2 of stream 0, i = elem_offset + index).  Scaled
                                   magnitudes from 448 upwards are stored as 448; NaN becomes
                                   the NaN code.  m, v: BF16 with SR (12 bytes moved per
                                   element), or with SR_FLAG_FP8_MOMENTS 8-bit codes (8
                                   bytes).  Combines with SR_FLAG_FP8_MOMENTS,
                                   SR_FLAG_EPS_IN_ROOT, SR_FLAG_DIV_BIAS and
                                   SR_FLAG_SKIP_NONFINITE_NORM only; elem_offset + numel
                                   must not exceed 2^63.                                  */

/* One tensor of the multi-tensor list. */
typedef struct sr_tensor {
    void*       p;           /* BF16 [numel], in/out: parameters x_t (E4M3 codes, one byte
                                each, with SR_FLAG_FP8_PARAMS)                            */
    const void* g;           /* BF16 [numel], in    : reduced gradient (Alg.1 line 4)     */
    void*       m;           /* BF16 or binary32 [numel], in/out: first moment (E4M3 codes,
                                one byte each, with SR_FLAG_FP8_MOMENTS)                  */
    void*       v;           /* same type as m, in/out: second moment (E5M2 codes with
                                SR_FLAG_FP8_MOMENTS)                                      */
    void*       aux;         /* NULL unless a flag names it: binary32 master parameters
                                (SR_FLAG_MASTER_FP32) or BF16 Kahan compensation
                                (SR_FLAG_KAHAN), in/out                                   */
    uint64_t    numel;       /* may be 0 (tensor skipped); may exceed 2^32                */
    uint64_t    elem_offset; /* index of element 0 in the RNG counter; 0 for a whole
                                tensor, the shard's start for a slice of a larger one     */
    uint32_t    tensor_id;   /* RNG counter word; keep it stable across steps and ranks   */
    int8_t      m_exp;       /* SR_FLAG_FP8_MOMENTS: m = decode(m8) 2^-m_exp, in
                                [-100, 100]; must be 0 without that flag                  */
    int8_t      v_exp;       /* SR_FLAG_FP8_MOMENTS: v = decode(v8) 2^-v_exp, in
                                [-100, 100]; must be 0 without that flag                  */
    int8_t      p_exp;       /* SR_FLAG_FP8_PARAMS: p = decode(p8) 2^-p_exp, in
                                [-100, 100]; must be 0 without that flag                  */
    uint8_t     reserved;    /* must be 0                                                 */
} sr_tensor_t;

/* Hyper-parameters of Algorithm 1: alpha_t, beta_1, beta_2, epsilon, lambda. */
typedef struct sr_hyper {
    float lr, beta1, beta2, eps, weight_decay;
} sr_hyper_t;

/*
 * Stochastic rounding of binary32 to BF16, Eq.(2) of Section 2.1, in the
 * add-uniform-noise-then-truncate form of Section 3:
 *   d_dst[i] = Q_SR(d_src[i]) with the 16 random bits of element i taken from
 *   Philox4x32-10(counter = (i>>3 low word, 3<<29 | i>>3 high bits, tensor_id,
 *   step), key = seed) -- slice i&7 of the 128 output bits.
 * A value v between adjacent BF16 values lo < hi becomes hi with probability
 * (v-lo)/(hi-lo); BF16 values are unchanged; a magnitude above the largest
 * BF16 may round to infinity; infinities pass; NaN becomes a quiet NaN with
 * the same sign.  d_src: binary32 [n] (4-byte aligned), d_dst: BF16 [n]
 * (2-byte aligned), both device, must not overlap.  n == 0 is a no-op.
 */
int sr_cast_f32_bf16(const float* d_src, void* d_dst, uint64_t n,
                     uint64_t seed, uint32_t step, uint32_t tensor_id, void* stream);

/*
 * Extension: stochastic rounding of binary32 to an 8-bit floating-point format
 * (the paper's conclusion names FP8 as the next target of SR and specifies
 * nothing; Eq.(2) of Section 2.1 is applied to the grid of the chosen OCP 8-bit
 * format).  format = SR_FP8_E4M3: 4 exponent bits (bias 7), 3 mantissa bits, no
 * infinities, largest finite value 448; magnitudes >= 448 and infinities
 * saturate to 448.  format = SR_FP8_E5M2: 5 exponent bits (bias 15), 2 mantissa
 * bits, binary16-like: a magnitude above 57344 rounds to infinity with the
 * probability Eq.(2) gives for an upper neighbour 65536, infinities pass.
 * Subnormals of both formats are produced; NaN becomes S.1111111.  Element i
 * owns word i&3 of Philox4x32-10(counter = (i>>2 low word, 5<<29 | i>>2 high
 * bits, tensor_id, step), key = seed) and draws r = its top D bits, D = 20 for
 * E4M3 and 21 for E5M2 (the bits binary32 has below the format's mantissa).
 * With lo <= |v| < hi adjacent grid magnitudes and
 * k = floor(2^D (|v|-lo)/(hi-lo)) the result is hi exactly when r + k >= 2^D:
 * the probability of Eq.(2) exactly for |v| at or above the format's smallest
 * normal, and short of it by less than 2^-D below (the fraction is truncated).
 * This is the function the chip's own conversion instruction computes.
 * d_src: binary32 [n] (4-byte aligned),
 * d_dst: one byte per element [n], both device, must not overlap; n <= 2^61;
 * n == 0 is a no-op.  SR_ERR_ARG for an unknown format.
 */
#define SR_FP8_E4M3 0u
#define SR_FP8_E5M2 1u
int sr_cast_f32_fp8(const float* d_src, void* d_dst, uint64_t n, uint32_t format, uint64_t seed,
                    uint32_t step, uint32_t tensor_id, void* stream);

/*
 * Global L2 norm of the gradients of a tensor list (the quantity a gradient
 * clip needs; the paper's training frameworks clip, Algorithm 1 does not
 * mention it): *d_norm_out = (float) sqrt( sum over all tensors and elements
 * of g^2 ), squares and sum in binary64, two passes (per-workgroup partial
 * sums into the workspace, then one workgroup), fixed summation tree, no
 * atomics.  Uses only .g and .numel of each entry (host array of n_tensors
 * entries).  d_norm_out: device scalar, 4-byte aligned.  d_workspace: device
 * scratch of at least sr_workspace_bytes(n_tensors, total numel) bytes,
 * 8-byte aligned; its contents after the call are unspecified.  An empty
 * list writes 0.
 */
int grad_global_norm(const sr_tensor_t* tensors, uint32_t n_tensors, float* d_norm_out,
                     void* d_workspace, uint64_t workspace_bytes, void* stream);

/*
 * grad_global_norm for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same kernels, same result bits; the partial sums go to a
 * static device array inside the library (SR_STATIC_SCRATCH_BYTES per device
 * that uses the library, held until the process ends) instead of a caller
 * workspace, and the call allocates nothing.  The array holds one partial sum
 * per 65536 gradient elements of each tensor (rounded up per tensor): lists
 * that need more than SR_STATIC_SCRATCH_BYTES / 8 of them -- about 8.5e9
 * elements -- are rejected with SR_ERR_SIZE and nothing is enqueued.  Nothing in
 * the array has to start at zero (every partial sum that is read has been
 * written by the same call).  All calls on one device share the array: calls
 * that may run concurrently on one device (different streams) race; order
 * them.  The first call on a device looks the array's address up in the
 * runtime (no allocation): make that call outside a stream capture.
 */
int grad_global_norm_static(const sr_tensor_t* tensors, uint32_t n_tensors, float* d_norm_out,
                            void* stream);

/*
 * The same two passes, leaving the binary64 sum of squares S itself in
 * *d_sumsq_out (device, 8-byte aligned) instead of (float) sqrt(S): what a
 * job whose gradients are sharded over ranks adds up (one all-reduce of a
 * double) before it takes the root and hands the norm to sr_adamw_step
 * (Algorithm 1 runs data-parallel; the clip needs the norm of the whole
 * gradient).  Arguments and workspace as for grad_global_norm.
 */
int grad_sum_of_squares(const sr_tensor_t* tensors, uint32_t n_tensors, double* d_sumsq_out,
                        void* d_workspace, uint64_t workspace_bytes, void* stream);

/*
 * One AdamW step with stochastically rounded write-backs over a tensor list
 * (Algorithm 1, lines 5-10; eps outside the root).  Per element, in binary32
 * with one rounding per operation and no fused multiply-add:
 *   g' = g c                       c = 1, or min(1, max_norm/(norm + 1e-6)) when clipping
 *   m' = beta1 m + (1-beta1) g'    v' = beta2 v + (1-beta2) g'^2
 *   u  = (m' rbc1) / (sqrt(v' rbc2) + eps)          rbc_i = 1/(1 - beta_i^step)
 *   y  = p - (lr u + (lr weight_decay) p)
 *   p <- Q_SR(y), m <- Q_SR(m'), v <- Q_SR(v')      (RNG streams 0, 1, 2 of element i:
 *        counter word 1 = stream<<29 | high bits of (elem_offset+i)>>3)
 * 1-beta, rbc and lr*weight_decay are formed in binary64 on the host and
 * rounded once.  The update uses the unrounded m', v'.  p, m, v are updated
 * in place; distinct tensors must not overlap.
 *   tensors      host array of n_tensors entries (n_tensors == 0: no-op)
 *   step         t >= 1
 *   flags        SR_FLAG_* bits
 *   d_grad_norm  NULL = no clipping; else device scalar holding the global
 *                gradient norm (as written by grad_global_norm on the same
 *                stream); gradients are scaled in registers, d g is not
 *                rewritten.  The scale is c = max_norm / (norm + 1e-6) in
 *                binary32, replaced by 1 when c > 1: a NaN norm gives c = NaN
 *                (every output NaN), an infinite norm c = 0 -- see
 *                SR_FLAG_SKIP_NONFINITE_NORM for a step that skips itself instead
 *   max_norm     > 0, used only with d_grad_norm
 */
int sr_adamw_step(const sr_tensor_t* tensors, uint32_t n_tensors, const sr_hyper_t* hyper,
                  uint32_t step, uint64_t seed, uint32_t flags,
                  const float* d_grad_norm, float max_norm, void* stream);

/* One accumulator/gradient pair of a multi-tensor gradient accumulation. */
typedef struct sr_accum {
    void*       acc;         /* BF16 [numel], in/out: accumulated gradient                 */
    const void* grad;        /* BF16 [numel], in    : this micro-batch's gradient          */
    uint64_t    numel;       /* may be 0                                                   */
    uint64_t    elem_offset; /* index of element 0 in the RNG counter (as in sr_tensor_t)  */
    uint32_t    tensor_id;   /* RNG counter word                                           */
    uint32_t    reserved;    /* must be 0                                                  */
} sr_accum_t;

#define SR_ACC_RNE   1u      /* round the accumulator to nearest-even instead of SR        */
#define SR_ACC_FIRST 2u      /* first micro-batch: acc is not read (taken as zero)         */

/*
 * BF16 gradient accumulation over micro-batches with a stochastically rounded
 * write-back, and (optionally) the global norm of the result in the same pass.
 * Section 3 keeps all training tensors in BF16; that includes the gradient
 * buffer that micro-batches accumulate into (accumulation steps: Section 5.2);
 * nearest rounding would stop accumulating once acc dwarfs the micro-gradient
 * (the x + u example of Section 2.1), SR does not in expectation.
 * Per element, binary32, one rounding per operation:
 *     t = scale * grad;  s = acc + t;  acc <- Q_SR(s)
 * with the 16 random bits of element i from Philox4x32-10(counter = (i>>3 low
 * word, 4<<29 | i>>3 high bits, tensor_id, micro_step), key = seed), i =
 * elem_offset + index.  Give every accumulation call of a training run its
 * own micro_step.
 *   d_norm_out  NULL, or a device scalar that receives (float) sqrt(sum of
 *               squares of the accumulator values written by this call), in
 *               binary64, fixed summation tree -- the norm a following
 *               sr_adamw_step clips with, at no extra pass over the gradients
 *   d_workspace only used with d_norm_out: at least
 *               sr_accumulate_workspace_bytes(n_tensors, total numel) bytes,
 *               8-byte aligned
 */
int sr_grad_accumulate(const sr_accum_t* tensors, uint32_t n_tensors, float scale,
                       uint32_t micro_step, uint64_t seed, uint32_t flags, float* d_norm_out,
                       void* d_workspace, uint64_t workspace_bytes, void* stream);

/* Workspace bound for sr_grad_accumulate with a norm (multiple of 256). */
uint64_t sr_accumulate_workspace_bytes(uint32_t n_tensors, uint64_t total_numel);

/* Bytes of device workspace grad_global_norm needs for a list of n_tensors
 * tensors with total_numel elements in all (an upper bound, multiple of 256). */
uint64_t sr_workspace_bytes(uint32_t n_tensors, uint64_t total_numel);

/* Static description of an SR_ERR_* code. */
const char* sr_strerror(int code);

/* hipError_t value of the most recent SR_ERR_HIP on the calling thread (0 if none). */
int sr_last_hip_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int sr_version(void);

/* ======================================================================
 * NOT PART OF THE METHOD.  What follows serves measurement and tests: two
 * traffic probes -- bench.py times them beside the update, and a caller can
 * time them on candidate buffers to choose where its arrays lie (on MI355X
 * the placement of p, g, m, v in physical memory moves the step by several
 * percent) -- and one hook through which the tests reach code paths that
 * otherwise need huge inputs or rare values.  Nothing in the update path
 * depends on them.
 * ====================================================================== */

/*
 * Measurement aid, not part of the method: the memory traffic of the BF16 step
 * (8 bytes read, 6 written per element: the 14 bytes per element of an
 * all-BF16 state, Section 3) with no arithmetic -- reads p, g, m, v and writes
 * p, m, v back UNCHANGED, in the launch geometry of sr_adamw_step.  Its time on
 * the caller's own buffers is the rate this access pattern can reach on them,
 * the ceiling the step is compared with.  BF16 arrays [numel], 2-byte aligned;
 * only whole 8-element blocks are touched.
 */
int sr_stream_probe(void* d_p, const void* d_g, void* d_m, void* d_v, uint64_t numel, void* stream);

/*
 * The same measurement aid for the step with 8-bit moments (SR_FLAG_FP8_MOMENTS:
 * 6 bytes read, 4 written per element): reads BF16 p, g and the one-byte code
 * arrays d_m8, d_v8 and writes p, m8, v8 back UNCHANGED.  p, g 2-byte aligned;
 * only whole 8-element blocks are touched.
 */
int sr_stream_probe_fp8m(void* d_p, const void* d_g, void* d_m8, void* d_v8, uint64_t numel, void* stream);

/*
 * Process-wide switches for tests and measurements (not synchronised with
 * calls running on other threads; set them while no call is in flight).
 * Results of every entry point must not depend on them.
 *   SR_DEBUG_LAUNCH_LIMIT    value = most workgroups one launch may hold
 *                            (0 = the hardware limit): small inputs are cut
 *                            into several launches, as huge ones are
 *   SR_DEBUG_FP8_INTEGER     value != 0: every wave of sr_cast_f32_fp8 and of
 *                            the 8-bit-moment write-back takes the integer
 *                            path instead of the chip's conversion instruction
 *                            (both compute the same function; this lets a
 *                            test prove it on the same inputs)
 *   SR_DEBUG_RESIDENT_WAVES  value = waves the streaming kernels allow to
 *                            reside per compute unit (0 = the library's own
 *                            setting per kernel, 32 = no cap; the hardware
 *                            grants LDS in units of 1280 bytes, so only 24,
 *                            20, 18, 16, 14, 12, 11, 10, 9, 8, ... differ)
 * Unknown keys are ignored.
 */
#define SR_DEBUG_LAUNCH_LIMIT   0u
#define SR_DEBUG_FP8_INTEGER    1u
#define SR_DEBUG_RESIDENT_WAVES 2u
void sr_debug_set(uint32_t key, uint32_t value);

#ifdef __cplusplus
}
#endif
#endif /* SRADAMW_H */
