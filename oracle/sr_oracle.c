/*
 * CPU oracle for the SR-AdamW update path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition that the GPU library is checked
 * against.  Nothing in the product path may call it, link it or fall back
 * to it; it shares no source, header, table or constant with the HIP code.
 *
 * What it follows (arXiv 2502.20566, "Stochastic Rounding for LLM Training:
 * Theory and Practice"):
 *   - stochastic rounding Q_SR: Eq.(2), Section 2.1 -- written out as the
 *     interval definition on VALUES (frexp/ldexp/floor in double), not as
 *     the add-noise-and-truncate trick the GPU uses (Section 3, "dithering");
 *   - the coupling of the random draw to the outcome: proof of the Lemma on
 *     the SR perturbation, Appendix B (round up when the draw falls below the
 *     fractional position q), in the equivalent integer form
 *     "away from zero iff r16 + k >= 65536";
 *   - AdamW with SR on the write-back: Algorithm 1, lines 5-10, Section 3,
 *     with eps outside the root (the standard AdamW denominator; line 10 as
 *     printed takes a second root of an already rooted quantity);
 *   - shared randomness across replicas: Algorithm 1 lines 9/11, realised as
 *     a stateless counter RNG (Philox4x32-10, Salmon et al., SC'11) keyed on
 *     (seed, step, tensor id, element index, output stream): no rank and no
 *     launch geometry enters the key.
 *
 * Arithmetic contract of the update: IEEE binary32, round to nearest even,
 * one rounding per listed operation, no fused multiply-add, correctly
 * rounded sqrt and divide, no flushing of subnormals.  Build with
 *   gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp
 * (x86-64 scalar SSE arithmetic: float expressions are evaluated in float).
 *
 * Pins (tests/test_oracle_*.py): exhaustive SR counts over all 2^16 draws,
 * exact unbiasedness and second moment, Philox known-answer vectors of the
 * Random123 distribution, 10^4-seed mean test, the random-walk example of
 * Section 2.2, Adam step-1 closed form, exact-rational evaluation of
 * Algorithm 1 on tiny inputs, torch.optim.AdamW on FP32 state, exact norms;
 * for the 8-bit extension (the conclusion's FP8 remark; the formats are the
 * OCP ones, not the paper's): torch's float8 decoders for the grids, exact
 * rational thresholds on brute-force neighbours, torch's nearest conversion;
 * for the update with 8-bit moments: bit equality with the BF16-moment path on
 * states both can hold (values from torch's decoders), exact-rational write-back
 * thresholds with draws read from the Philox streams, means over 4000 seeds.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REF_FLAG_FP32_MOMENTS 1u
#define REF_FLAG_RNE_MOMENTS  2u
#define REF_FLAG_RNE_PARAMS   4u
#define REF_FLAG_MASTER_FP32  8u
#define REF_FLAG_KAHAN       16u
#define REF_FLAG_EPS_IN_ROOT 32u
#define REF_FLAG_DIV_BIAS    64u
#define REF_FLAG_FP8_MOMENTS 128u

/* ---------------------------------------------------------------- RNG --- */

/* Philox4x32 with 10 rounds.  One round maps (c0,c1,c2,c3) under key (k0,k1)
 * to (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)); the key is
 * advanced by the two Weyl constants between rounds. */
void ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += W0; k1 += W1; }
        uint64_t prod0 = M0 * (uint64_t)c0;
        uint64_t prod1 = M1 * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prod1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod1;
        uint32_t n2 = (uint32_t)(prod0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 16 random bits of element `i` (index within its tensor, 64-bit) of
 * output stream `stream` (0 = parameter, 1 = first moment, 2 = second moment,
 * 3 = standalone cast).  Eight consecutive elements share one Philox block:
 * counter = (block low word, stream<<29 | block high bits, tensor id, step),
 * key = the two halves of the seed; element j = i mod 8 takes the low (j even)
 * or high (j odd) half of output word j/2. */
uint32_t ref_r16(uint64_t seed, uint32_t step, uint32_t tensor_id, uint64_t i, uint32_t stream)
{
    uint64_t blk = i >> 3;
    uint32_t ctr[4], key[2], w[4];
    ctr[0] = (uint32_t)(blk & 0xFFFFFFFFu);
    ctr[1] = (stream << 29) | (uint32_t)(blk >> 32);
    ctr[2] = tensor_id;
    ctr[3] = step;
    key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    key[1] = (uint32_t)(seed >> 32);
    ref_philox4x32_10(ctr, key, w);
    unsigned j = (unsigned)(i & 7u);
    return (w[j >> 1] >> (16u * (j & 1u))) & 0xFFFFu;
}

/* out[n] = r16 of elements i0 .. i0+n-1 (for distribution tests). */
void ref_r16_many(uint64_t seed, uint32_t step, uint32_t tensor_id, uint64_t i0, uint64_t n,
                  uint32_t stream, uint16_t* out)
{
    for (uint64_t i = 0; i < n; ++i)
        out[i] = (uint16_t)ref_r16(seed, step, tensor_id, i0 + i, stream);
}

/* ------------------------------------------------------ BF16 encoding --- */

static float bf16_bits_to_float(uint16_t h)
{
    /* BF16 is the upper half of the binary32 encoding: decoding is exact. */
    uint32_t b = (uint32_t)h << 16;
    float f; memcpy(&f, &b, 4); return f;
}

static uint16_t float_on_bf16_grid_to_bits(float f)
{
    /* Only ever called with a value that IS a BF16 value (or +-inf): the low
     * half of the encoding is zero, nothing is rounded here. */
    uint32_t b; memcpy(&b, &f, 4);
    if (b & 0xFFFFu) abort();
    return (uint16_t)(b >> 16);
}

/* ------------------------------------------------ stochastic rounding --- */

/* Q_SR of Eq.(2) for binary32 -> BF16 with the draw r16 in [0, 65535].
 *   a  = |y|;  lo = largest BF16 magnitude <= a;  hi = next BF16 magnitude;
 *   k  = 65536 (a - lo)/(hi - lo)   (an integer: exactly 2^16 binary32
 *        values lie in [lo, hi) at uniform spacing, subnormal range included);
 *   magnitude = hi  iff  r16 + k >= 65536,  else lo;  sign of y is kept.
 * So P(away from zero) = k/65536 = (a - lo)/(hi - lo), which is Eq.(2) for
 * either sign, and a value already on the BF16 grid (k = 0) never moves.
 * Above the largest finite BF16, hi = 2^128 is emitted as infinity.
 * Infinities pass through; a NaN becomes the quiet NaN with the same sign
 * and the same upper payload bits. */
uint16_t ref_sr_round(float y, uint32_t r16)
{
    uint32_t ybits; memcpy(&ybits, &y, 4);
    if (isnan(y)) return (uint16_t)((ybits >> 16) | 0x0040u);
    if (isinf(y)) return (uint16_t)(ybits >> 16);

    double a = fabs((double)y);
    double lo, hi;
    if (a == 0.0) {
        lo = 0.0; hi = ldexp(1.0, -133);
    } else {
        int e;
        (void)frexp(a, &e);              /* a = f * 2^e with f in [0.5, 1) */
        int q = e - 8;                   /* BF16 keeps 8 significant bits  */
        if (q < -133) q = -133;          /* fixed spacing below 2^-126      */
        double spacing = ldexp(1.0, q);
        lo = floor(a / spacing) * spacing;
        hi = lo + spacing;
    }
    double k = 65536.0 * (a - lo) / (hi - lo);
    if (k != floor(k) || k < 0.0 || k > 65535.0) abort();   /* exact by construction */
    double mag = ((double)r16 + k >= 65536.0) ? hi : lo;
    float out = (mag >= ldexp(1.0, 128)) ? INFINITY : (float)mag;   /* (float)mag is exact */
    out = copysignf(out, y);
    return float_on_bf16_grid_to_bits(out);
}

/* Round-to-nearest-even to BF16 by value (Eq.(1), ties to the even
 * significand): the deterministic comparison rounding. */
uint16_t ref_rne_round(float y)
{
    uint32_t ybits; memcpy(&ybits, &y, 4);
    if (isnan(y)) return (uint16_t)((ybits >> 16) | 0x0040u);
    if (isinf(y)) return (uint16_t)(ybits >> 16);
    double a = fabs((double)y);
    double mag = 0.0;
    if (a != 0.0) {
        int e; (void)frexp(a, &e);
        int q = e - 8; if (q < -133) q = -133;
        double spacing = ldexp(1.0, q);
        double n = floor(a / spacing);
        double rem = a / spacing - n;            /* exact: a/spacing has <= 24 bits */
        if (rem > 0.5 || (rem == 0.5 && fmod(n, 2.0) == 1.0)) n += 1.0;
        mag = n * spacing;
    }
    float out = (mag >= ldexp(1.0, 128)) ? INFINITY : (float)mag;
    out = copysignf(out, y);
    return float_on_bf16_grid_to_bits(out);
}

void ref_sr_round_many(const float* y, const uint32_t* r16, uint64_t n, uint16_t* out)
{
    for (uint64_t i = 0; i < n; ++i) out[i] = ref_sr_round(y[i], r16[i]);
}

/* All 65536 draws for one input, out[r] = Q_SR(*y; r).  The input is passed
 * by address so that a signalling-NaN encoding reaches the function intact. */
void ref_sr_round_all_draws(const float* y, uint16_t* out)
{
    for (uint32_t r = 0; r < 65536u; ++r) out[r] = ref_sr_round(*y, r);
}

/* Standalone cast: dst[i] = Q_SR(src[i]; r16(seed, step, tensor_id, elem_offset + i, stream 3)). */
void ref_sr_cast_f32_bf16(const float* src, uint16_t* dst, uint64_t n,
                          uint64_t seed, uint32_t step, uint32_t tensor_id,
                          uint64_t elem_offset, int nthreads)
{
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        uint32_t r = ref_r16(seed, step, tensor_id, elem_offset + (uint64_t)i, 3u);
        dst[i] = ref_sr_round(src[i], r);
    }
}

/* ------------------------------------------ 8-bit formats (extension) --- */

/* The paper's conclusion names 8-bit floating point as the next target of
 * stochastic rounding and specifies nothing; Eq.(2) applies to any grid.  The
 * two grids here are the OCP 8-bit floating-point formats (OFP8):
 *   format 0, E4M3: 1 sign, 4 exponent bits (bias 7), 3 mantissa bits; no
 *     infinities; S.1111.111 is the only NaN; largest finite value 448.
 *   format 1, E5M2: 1 sign, 5 exponent bits (bias 15), 2 mantissa bits;
 *     S.11111.00 is infinity, S.11111.{01,10,11} are NaNs; largest finite 57344.
 * Exponent field 0 holds zero and the subnormals (no implicit leading one). */

/* Value of code `code` (0..255): NaN for a NaN code, +-inf for an infinity. */
double ref_fp8_decode(uint32_t code, int format)
{
    int mb = format == 0 ? 3 : 2, bias = format == 0 ? 7 : 15;
    int sign = (code >> 7) & 1;
    int e = (int)((code & 0x7Fu) >> mb);
    int m = (int)(code & ((1u << mb) - 1u));
    double v;
    if (format == 0 && (code & 0x7Fu) == 0x7Fu) return NAN;
    if (format == 1 && e == 31) v = (m == 0) ? INFINITY : NAN;
    else if (e == 0) v = ldexp((double)m, 1 - bias - mb);
    else v = ldexp((double)((1 << mb) + m), e - bias - mb);
    return sign ? -v : v;
}

/* The 32 random bits of element i: word i mod 4 of the Philox block i div 4. */
uint32_t ref_r32(uint64_t seed, uint32_t step, uint32_t tensor_id, uint64_t i, uint32_t stream)
{
    uint64_t blk = i >> 2;
    uint32_t ctr[4], key[2], w[4];
    ctr[0] = (uint32_t)(blk & 0xFFFFFFFFu);
    ctr[1] = (stream << 29) | (uint32_t)(blk >> 32);
    ctr[2] = tensor_id;
    ctr[3] = step;
    key[0] = (uint32_t)(seed & 0xFFFFFFFFu);
    key[1] = (uint32_t)(seed >> 32);
    ref_philox4x32_10(ctr, key, w);
    return w[i & 3u];
}

/* Eq.(2) on an 8-bit grid, by the interval definition on VALUES: lo = largest
 * grid magnitude <= |y|, hi = next one.  The draw has D = 23 - mb bits, as many
 * as binary32 has below the format's mantissa (20 for E4M3, 21 for E5M2): the
 * top D bits of the element's 32-bit random word.  k = floor(2^D (|y|-lo)/(hi-lo))
 * and the magnitude becomes hi exactly when r_D + k >= 2^D (probability k/2^D).
 * For every |y| at or above the format's smallest normal, (|y|-lo)/(hi-lo) has
 * at most D fractional bits, so the probability is Eq.(2)'s exactly; below it
 * (the fixed spacing of the subnormal range) the fraction is truncated to D
 * bits, a bias of less than 2^-D of one spacing.  Sign kept.  Out of range:
 * E5M2 follows the binary16-like rule (a magnitude above 57344 has hi = 65536,
 * emitted as infinity; infinities pass); E4M3 has no infinity and saturates
 * (magnitudes >= 448, infinities included, become 448).  NaN becomes S.1111111
 * in either format. */
uint8_t ref_sr_round_fp8(float y, uint32_t r32, int format)
{
    const int mb = format == 0 ? 3 : 2, emin = format == 0 ? -6 : -14;
    const double maxfin = format == 0 ? 448.0 : 57344.0;
    uint32_t bits; memcpy(&bits, &y, 4);
    const uint8_t sign = (uint8_t)((bits >> 31) << 7);
    if (y != y) return (uint8_t)(sign | 0x7Fu);
    double a = fabs((double)y);
    double mag;
    if (format == 0 && a >= maxfin) mag = maxfin;
    else if (isinf(a)) mag = INFINITY;
    else if (a == 0.0) mag = 0.0;
    else {
        int e2; (void)frexp(a, &e2);                 /* a = f 2^e2, f in [0.5, 1)  */
        int E = e2 - 1; if (E < emin) E = emin;      /* exponent of the grid cell  */
        double spacing = ldexp(1.0, E - mb);
        double t = a / spacing;                      /* exact: power-of-two scale  */
        double n = floor(t);
        const int D = 23 - mb;
        double scale = ldexp(1.0, D);
        double k = floor((t - n) * scale);           /* t - n exact; scaled exactly */
        double rD = (double)(r32 >> (32 - D));       /* the draw: top D bits of the word */
        if (rD + k >= scale) n += 1.0;
        mag = n * spacing;
        if (mag > maxfin) mag = INFINITY;            /* E5M2 only: hi = 65536      */
    }
    /* encode: the code whose decoded magnitude is mag (it exists by construction) */
    for (uint32_t c = 0; c < 128u; ++c) {
        double v = ref_fp8_decode(c, format);
        if (v == mag) return (uint8_t)(sign | c);
    }
    abort();
}

/* dst[i] = Q_SR(src[i]; r32(seed, step, tensor_id, elem_offset + i, stream 5)). */
void ref_sr_cast_f32_fp8(const float* src, uint8_t* dst, uint64_t n, int format,
                         uint64_t seed, uint32_t step, uint32_t tensor_id,
                         uint64_t elem_offset, int nthreads)
{
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)n; ++i) {
        uint32_t r = ref_r32(seed, step, tensor_id, elem_offset + (uint64_t)i, 5u);
        dst[i] = ref_sr_round_fp8(src[i], r, format);
    }
}

/* ------------------------------------------------------------- AdamW --- */

typedef struct {
    float beta1, beta2;   /* as given                                            */
    float omb1, omb2;     /* 1 - beta, formed in double, rounded once            */
    float rbc1, rbc2;     /* 1/(1 - beta^t), formed in double, rounded once      */
    float lr, eps;        /* as given                                            */
    float lw;             /* lr * weight_decay, formed in double, rounded once   */
    float clip;           /* gradient scale c (1 when clipping is off)           */
    float bc1, bc2;       /* 1 - beta^t, formed in double, rounded once          */
} ref_scalars_t;

static double pow_uint(double base, uint32_t e)
{
    /* beta^t by binary exponentiation in double */
    double result = 1.0;
    while (e) {
        if (e & 1u) result *= base;
        base *= base;
        e >>= 1;
    }
    return result;
}

/* Scalars of one step (Algorithm 1, lines 5-8 and 10).  `norm` is the global
 * gradient norm or NULL for no clipping; with clipping the gradient is scaled
 * by c = min(1, max_norm/(norm + 1e-6)) in binary32 arithmetic. */
void ref_adamw_scalars(float lr, float beta1, float beta2, float eps, float weight_decay,
                       uint32_t step, const float* norm, float max_norm, ref_scalars_t* s)
{
    s->beta1 = beta1; s->beta2 = beta2;
    s->omb1 = (float)(1.0 - (double)beta1);
    s->omb2 = (float)(1.0 - (double)beta2);
    s->rbc1 = (float)(1.0 / (1.0 - pow_uint((double)beta1, step)));
    s->rbc2 = (float)(1.0 / (1.0 - pow_uint((double)beta2, step)));
    s->bc1 = (float)(1.0 - pow_uint((double)beta1, step));
    s->bc2 = (float)(1.0 - pow_uint((double)beta2, step));
    s->lr = lr; s->eps = eps;
    s->lw = (float)((double)lr * (double)weight_decay);
    s->clip = 1.0f;
    if (norm) {
        float denom = *norm + 1e-6f;
        float c = max_norm / denom;
        if (c > 1.0f) c = 1.0f;
        s->clip = c;
    }
}

/* One element of Algorithm 1 lines 5-10 before the write-back rounding:
 * returns the unrounded new parameter y and the unrounded moments m1, v1. */
static void adamw_element(const ref_scalars_t* s, uint32_t flags, float p, float g, float m, float v,
                          float* y_out, float* m1_out, float* v1_out, float* sum_out)
{
    float g1 = g * s->clip;
    /* line 5: m <- beta1 m + (1 - beta1) g */
    float t1 = s->beta1 * m;
    float t2 = s->omb1 * g1;
    float m1 = t1 + t2;
    /* line 6: v <- beta2 v + (1 - beta2) g^2 */
    float gg = g1 * g1;
    float t3 = s->beta2 * v;
    float t4 = s->omb2 * gg;
    float v1 = t3 + t4;
    /* lines 7-8: bias corrections: multiplications by host reciprocals, or, with
     * REF_FLAG_DIV_BIAS, the divisions by 1 - beta^t as the lines are printed */
    float mh, vh;
    if (flags & REF_FLAG_DIV_BIAS) { mh = m1 / s->bc1; vh = v1 / s->bc2; }
    else                           { mh = m1 * s->rbc1; vh = v1 * s->rbc2; }
    /* line 10: x - (alpha mhat/(sqrt(vhat) + eps) + alpha lambda x); with
     * REF_FLAG_EPS_IN_ROOT the denominator is sqrt(vhat + eps), the form of Appendix B */
    float d;
    if (flags & REF_FLAG_EPS_IN_ROOT) { float ve = vh + s->eps; d = sqrtf(ve); }
    else                              { d = sqrtf(vh) + s->eps; }
    float u = mh / d;
    float a = s->lr * u;
    float b = s->lw * p;
    float sum = a + b;
    float y = p - sum;
    *y_out = y; *m1_out = m1; *v1_out = v1;
    if (sum_out) *sum_out = sum;
}

/* Unrounded results (for the FP32-intermediate checks). m, v are BF16 bit
 * patterns unless REF_FLAG_FP32_MOMENTS. */
void ref_adamw_unrounded(const uint16_t* p, const uint16_t* g, const void* m, const void* v,
                         uint64_t numel, const ref_scalars_t* s, uint32_t flags,
                         float* y, float* m1, float* v1)
{
    const int fp32m = (flags & REF_FLAG_FP32_MOMENTS) != 0;
    for (uint64_t i = 0; i < numel; ++i) {
        float mi = fp32m ? ((const float*)m)[i] : bf16_bits_to_float(((const uint16_t*)m)[i]);
        float vi = fp32m ? ((const float*)v)[i] : bf16_bits_to_float(((const uint16_t*)v)[i]);
        adamw_element(s, flags, bf16_bits_to_float(p[i]), bf16_bits_to_float(g[i]), mi, vi,
                      &y[i], &m1[i], &v1[i], NULL);
    }
}

/* One tensor of one step, in place over p, m, v (and aux).
 *   BF16 moments (default): p, m, v all written back with SR, streams 0, 1, 2;
 *   REF_FLAG_FP32_MOMENTS : m, v are binary32 and stored unrounded, SR on p only;
 *   REF_FLAG_RNE_MOMENTS  : BF16 moments written back with round-to-nearest-even
 *                           (the paper's own setting: SR on line 10 only);
 *   REF_FLAG_RNE_PARAMS   : the parameter write-back is round-to-nearest-even too
 *                           (with RNE_MOMENTS: the "BF16" nearest-rounding strategy of
 *                           Section 5.1, no random bits at all);
 * Comparison strategies of Section 5.1 / Section 1 that carry an auxiliary tensor `aux`:
 *   REF_FLAG_MASTER_FP32  : O2-style mixed precision: aux = binary32 master parameters,
 *                           updated in binary32 and stored unrounded; m, v binary32
 *                           (FP32_MOMENTS must be set); p = RNE(master) is the BF16 model copy;
 *   REF_FLAG_KAHAN        : BF16 + Kahan summation on the parameter (Zamirai et al., cited in
 *                           Section 1): aux = BF16 compensation c.  With the step's total
 *                           update s (so that the plain result would be p - s):
 *                             yk = (-s) - c;  t = p + yk;  p' = RNE(t);
 *                             c' = RNE((p' - p) - yk);   m, v written back with RNE.
 * Variants of the arithmetic (any strategy): REF_FLAG_EPS_IN_ROOT, REF_FLAG_DIV_BIAS, see
 * adamw_element.
 * Element i of the tensor uses RNG index elem_offset + i. */
void ref_sr_adamw_tensor(uint16_t* p, const uint16_t* g, void* m, void* v, void* aux,
                         uint64_t numel, uint32_t tensor_id, uint64_t elem_offset,
                         const ref_scalars_t* s, uint32_t step, uint64_t seed,
                         uint32_t flags, int nthreads)
{
    const int fp32m  = (flags & REF_FLAG_FP32_MOMENTS) != 0;
    const int master = (flags & REF_FLAG_MASTER_FP32) != 0;
    const int kahan  = (flags & REF_FLAG_KAHAN) != 0;
    const int rnem   = kahan || (flags & REF_FLAG_RNE_MOMENTS) != 0;
    const int rnep   = (flags & REF_FLAG_RNE_PARAMS) != 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)numel; ++ii) {
        uint64_t i = (uint64_t)ii;
        uint64_t gi = elem_offset + i;
        float pi = master ? ((float*)aux)[i] : bf16_bits_to_float(p[i]);
        float gr = bf16_bits_to_float(g[i]);
        float mi = fp32m ? ((float*)m)[i] : bf16_bits_to_float(((uint16_t*)m)[i]);
        float vi = fp32m ? ((float*)v)[i] : bf16_bits_to_float(((uint16_t*)v)[i]);
        float y, m1, v1, sum;
        adamw_element(s, flags, pi, gr, mi, vi, &y, &m1, &v1, &sum);
        if (master) {
            ((float*)aux)[i] = y;
            p[i] = ref_rne_round(y);
        } else if (kahan) {
            float c  = bf16_bits_to_float(((uint16_t*)aux)[i]);
            float ns = -sum;
            float yk = ns - c;
            float t  = pi + yk;
            uint16_t pn = ref_rne_round(t);
            float d1 = bf16_bits_to_float(pn) - pi;
            float cn = d1 - yk;
            p[i] = pn;
            ((uint16_t*)aux)[i] = ref_rne_round(cn);
        } else if (rnep) {
            p[i] = ref_rne_round(y);
        } else {
            p[i] = ref_sr_round(y, ref_r16(seed, step, tensor_id, gi, 0u));
        }
        if (fp32m) {
            ((float*)m)[i] = m1;
            ((float*)v)[i] = v1;
        } else if (rnem) {
            ((uint16_t*)m)[i] = ref_rne_round(m1);
            ((uint16_t*)v)[i] = ref_rne_round(v1);
        } else {
            ((uint16_t*)m)[i] = ref_sr_round(m1, ref_r16(seed, step, tensor_id, gi, 1u));
            ((uint16_t*)v)[i] = ref_sr_round(v1, ref_r16(seed, step, tensor_id, gi, 2u));
        }
    }
}

/* Extension (the conclusion names FP8 as the next target of SR and says no more):
 * one tensor of one step with the moments held in 8 bits, m as E4M3 and v as E5M2
 * codes, one byte per element, each with a power-of-two scale per tensor:
 *     m = decode(m8) * 2^-m_exp,      v = decode(v8) * 2^-v_exp           (exact)
 *     y, m1, v1 by adamw_element as for every other strategy
 *     m8 <- Q_SR,E4M3(m1 * 2^m_exp),  v8 <- Q_SR,E5M2(v1 * 2^v_exp)
 * The two products are binary32 multiplications (exact unless the product leaves
 * binary32's normal range).  Q_SR is ref_sr_round_fp8 with the element's 16-bit
 * draws of output streams 1 and 2 -- the same draws the BF16 moments use -- placed
 * in the top half of the 32-bit word: the rounding sees k = floor(2^16 frac) of the
 * dropped fraction (bias below 2^-16 of one grid spacing).  The parameter is
 * written back as in the BF16 strategies: SR with stream 0, or nearest with
 * REF_FLAG_RNE_PARAMS.  |m_exp|, |v_exp| <= 100 keeps the decode exact.
 * The write-back of v saturates like that of m: where Q_SR gives E5M2's infinity
 * (a scaled value above 57344 that rounds up, or an infinite one) the largest
 * finite code S.11110.11 is stored instead, because an infinite second moment
 * would stay infinite (beta2 * inf) and stop its parameter for good.  NaN stays NaN. */
void ref_sr_adamw_tensor_fp8m(uint16_t* p, const uint16_t* g, uint8_t* m8, uint8_t* v8,
                              uint64_t numel, uint32_t tensor_id, uint64_t elem_offset,
                              const ref_scalars_t* s, uint32_t step, uint64_t seed,
                              uint32_t flags, int m_exp, int v_exp, int nthreads)
{
    const int rnep = (flags & REF_FLAG_RNE_PARAMS) != 0;
    const float m_scale = (float)ldexp(1.0, m_exp), v_scale = (float)ldexp(1.0, v_exp);
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)numel; ++ii) {
        uint64_t i = (uint64_t)ii;
        uint64_t gi = elem_offset + i;
        float pi = bf16_bits_to_float(p[i]);
        float gr = bf16_bits_to_float(g[i]);
        float mi = (float)ldexp(ref_fp8_decode(m8[i], 0), -m_exp);
        float vi = (float)ldexp(ref_fp8_decode(v8[i], 1), -v_exp);
        float y, m1, v1;
        adamw_element(s, flags, pi, gr, mi, vi, &y, &m1, &v1, NULL);
        p[i] = rnep ? ref_rne_round(y) : ref_sr_round(y, ref_r16(seed, step, tensor_id, gi, 0u));
        float ms = m1 * m_scale;
        float vs = v1 * v_scale;
        m8[i] = ref_sr_round_fp8(ms, ref_r16(seed, step, tensor_id, gi, 1u) << 16, 0);
        uint8_t vc = ref_sr_round_fp8(vs, ref_r16(seed, step, tensor_id, gi, 2u) << 16, 1);
        if ((vc & 0x7Fu) == 0x7Cu) vc = (uint8_t)((vc & 0x80u) | 0x7Bu);      /* infinity -> largest finite */
        v8[i] = vc;
    }
}

/* Extension, one step further: the PARAMETER held in 8 bits too (the write-back the paper's
 * conclusion points to; the paper gives no design).  p8 holds E4M3 codes, one byte per
 * element, with a power-of-two scale per tensor:
 *     p = decode(p8) * 2^-p_exp                                              (exact)
 *     y, m1, v1 by adamw_element as for every other strategy
 *     p8 <- Q_SR,E4M3(y * 2^p_exp)        (a binary32 multiplication, then Eq.(2) on the grid)
 * Q_SR is ref_sr_round_fp8 with the element's full 32-bit word of output stream 0 (word
 * i mod 4 of Philox block i div 4, the layout of the standalone 8-bit cast): the draw has the
 * 20 bits binary32 keeps below E4M3's mantissa, so the probability is Eq.(2)'s exactly for every
 * scaled value at or above 2^-6.  E4M3 has no infinity: scaled magnitudes from 448 upwards
 * are stored as 448; NaN becomes the NaN code.  The moments are BF16 with SR (streams 1, 2,
 * 16-bit draws, as in ref_sr_adamw_tensor) when m8 is NULL -- then m16, v16 are used -- or
 * 8-bit codes exactly as in ref_sr_adamw_tensor_fp8m when m8, v8 are given. */
void ref_sr_adamw_tensor_fp8p(uint8_t* p8, const uint16_t* g, uint16_t* m16, uint16_t* v16,
                              uint8_t* m8, uint8_t* v8,
                              uint64_t numel, uint32_t tensor_id, uint64_t elem_offset,
                              const ref_scalars_t* s, uint32_t step, uint64_t seed,
                              uint32_t flags, int p_exp, int m_exp, int v_exp, int nthreads)
{
    const int fp8m = m8 != NULL;
    const float p_scale = (float)ldexp(1.0, p_exp);
    const float m_scale = (float)ldexp(1.0, m_exp), v_scale = (float)ldexp(1.0, v_exp);
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)numel; ++ii) {
        uint64_t i = (uint64_t)ii;
        uint64_t gi = elem_offset + i;
        float pi = (float)ldexp(ref_fp8_decode(p8[i], 0), -p_exp);
        float gr = bf16_bits_to_float(g[i]);
        float mi = fp8m ? (float)ldexp(ref_fp8_decode(m8[i], 0), -m_exp) : bf16_bits_to_float(m16[i]);
        float vi = fp8m ? (float)ldexp(ref_fp8_decode(v8[i], 1), -v_exp) : bf16_bits_to_float(v16[i]);
        float y, m1, v1;
        adamw_element(s, flags, pi, gr, mi, vi, &y, &m1, &v1, NULL);
        float ys = y * p_scale;
        p8[i] = ref_sr_round_fp8(ys, ref_r32(seed, step, tensor_id, gi, 0u), 0);
        if (fp8m) {
            float ms = m1 * m_scale;
            float vs = v1 * v_scale;
            m8[i] = ref_sr_round_fp8(ms, ref_r16(seed, step, tensor_id, gi, 1u) << 16, 0);
            uint8_t vc = ref_sr_round_fp8(vs, ref_r16(seed, step, tensor_id, gi, 2u) << 16, 1);
            if ((vc & 0x7Fu) == 0x7Cu) vc = (uint8_t)((vc & 0x80u) | 0x7Bu);
            v8[i] = vc;
        } else {
            m16[i] = ref_sr_round(m1, ref_r16(seed, step, tensor_id, gi, 1u));
            v16[i] = ref_sr_round(v1, ref_r16(seed, step, tensor_id, gi, 2u));
        }
    }
}

/* The unrounded results of the same step (for the checks of its arithmetic). */
void ref_adamw_unrounded_fp8m(const uint16_t* p, const uint16_t* g, const uint8_t* m8, const uint8_t* v8,
                              uint64_t numel, const ref_scalars_t* s, uint32_t flags, int m_exp, int v_exp,
                              float* y, float* m1, float* v1)
{
    for (uint64_t i = 0; i < numel; ++i) {
        float mi = (float)ldexp(ref_fp8_decode(m8[i], 0), -m_exp);
        float vi = (float)ldexp(ref_fp8_decode(v8[i], 1), -v_exp);
        adamw_element(s, flags, bf16_bits_to_float(p[i]), bf16_bits_to_float(g[i]), mi, vi,
                      &y[i], &m1[i], &v1[i], NULL);
    }
}

/* ------------------------------------------------ gradient accumulation --- */

#define REF_ACC_RNE   1u   /* round the accumulator to nearest-even instead of stochastically */
#define REF_ACC_FIRST 2u   /* first micro-batch: the old accumulator is not read (taken as 0)  */

/* BF16 gradient accumulation over micro-batches with a stochastically rounded write-back
 * (every tensor stays BF16, Section 3; fewer or more accumulation steps are the knob Section 5.2
 * "Memory" mentions).  Per element, binary32, one rounding per operation:
 *     t = scale * g;   s = acc + t;   acc <- Q_SR(s)
 * with the random bits of output stream 4 and `micro_step` in the counter's step word.
 * Element i uses RNG index elem_offset + i. */
void ref_grad_accumulate(uint16_t* acc, const uint16_t* g, uint64_t numel, float scale,
                         uint32_t micro_step, uint64_t seed, uint32_t tensor_id,
                         uint64_t elem_offset, uint32_t flags, int nthreads)
{
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(static)
    for (int64_t ii = 0; ii < (int64_t)numel; ++ii) {
        uint64_t i = (uint64_t)ii;
        float a = (flags & REF_ACC_FIRST) ? 0.0f : bf16_bits_to_float(acc[i]);
        float t = scale * bf16_bits_to_float(g[i]);
        float s = a + t;
        acc[i] = (flags & REF_ACC_RNE) ? ref_rne_round(s)
                                       : ref_sr_round(s, ref_r16(seed, micro_step, tensor_id, elem_offset + i, 4u));
    }
}

/* ------------------------------------------------------ gradient norm --- */

/* Global L2 norm over a list of BF16 gradient tensors: sum of squares in
 * long double with Neumaier compensation, tensors in list order, elements in
 * index order; norm = (float)sqrt((double)S). */
float ref_grad_global_norm(const uint16_t* const* g, const uint64_t* numel, uint32_t n_tensors)
{
    long double sum = 0.0L, comp = 0.0L;
    for (uint32_t t = 0; t < n_tensors; ++t) {
        const uint16_t* gt = g[t];
        for (uint64_t i = 0; i < numel[t]; ++i) {
            long double x = (long double)bf16_bits_to_float(gt[i]);
            long double term = x * x;                 /* exact: 16-bit product */
            long double s2 = sum + term;
            if (fabsl(sum) >= fabsl(term)) comp += (sum - s2) + term;
            else                           comp += (term - s2) + sum;
            sum = s2;
        }
    }
    double S = (double)(sum + comp);
    return (float)sqrt(S);
}

int ref_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
