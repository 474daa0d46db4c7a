/*
 * CPU oracle for the NVFP4 double-block quantizer and the quantized GEMM.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference the GPU
 * library is checked against.  It shares no code, table or header with the HIP
 * path, and nothing in the product path may call it: only tests/, the smoke
 * check and the bench's cpu_baseline leg load it.
 *
 * What it follows (TetraJet-v2, arXiv 2510.27527):
 *   - E2M1 value set {0, +-0.5, 1, 1.5, 2, 3, 4, 6}          Sec. 2.1 "NVFP4 Format"
 *   - group quantization P_i = round_FP4(X_i / S)             Sec. 2.1 "Quantization"
 *   - deterministic rounding = nearest FP4 value              Sec. 2.1, round_{FP4,D}
 *   - stochastic rounding between neighbours q1 <= x < q2     Sec. 2.1, round_{FP4,S}
 *   - double-block scaling S_global, S_block                  Sec. 2.2 (display eq.)
 *   - the six quantizers / three matrix products              Sec. 2.3 (display eq.)
 *
 * Where the paper leaves the arithmetic open, this file takes the readings
 * listed here (the same list is in the design document):
 *   R1  All quantizer arithmetic that decides a code is IEEE binary32,
 *       round-to-nearest-even, one rounding per written operation, no fused
 *       multiply-add, subnormals kept.  Order:  S_g = amax_g / 2688 ;
 *       i_g = 1 / S_g ; s = amax_b * (i_g * (1/6)) ; S_b = e4m3(s) ;
 *       r = i_g * (1 / S_b) ; y = x * r ; a = min(|y|, 6), with 1/6 the binary32
 *       constant.  (Divisions are per outer group or per scale value, never
 *       per element.)
 *   R2  S_g is floored at 2^-100 (keeps 1/d finite); an all-zero outer group
 *       gets S_g = 1 and all-zero scales and codes.
 *   R3  The block scale is rounded to E4M3 (bias 7, no infinity, max 448,
 *       subnormals k * 2^-9) either to nearest-even (SCALE_NE) or upward
 *       (SCALE_UP); both saturate at 448.  Default: NE for deterministic
 *       rounding, UP for stochastic rounding (a scale rounded down would clip
 *       the block maximum and bias the estimate).
 *   R4  Deterministic rounding breaks ties toward the even code.
 *   R5  Stochastic rounding: the paper's rule is "x + xi <= midpoint -> q1" with
 *       xi ~ U(-D/2, D/2), D = q2 - q1.  With f = (a - q1)/D and v = xi/D + 1/2
 *       (uniform on the unit interval) that is "q2 iff f + v > 1".  The one change
 *       made here is the random variate: v is drawn from the 22-bit grid
 *       {0, 1, .., 2^22-1} / 2^22, and a goes to q2 iff f + u/2^22 >= 1, i.e. iff
 *       u + floor(f * 2^22) >= 2^22.  So P(q2) = floor(f * 2^22) / 2^22.  From 1 to
 *       6 a binary32 value has at most 22 bits below the E2M1 mantissa bit, f * 2^22
 *       is an integer and the rounding is exactly unbiased; below 1 (the E2M1
 *       subnormal range) the bits of a below 2^-23 cannot reach the decision, and
 *       the mean falls short of a by less than 2^-23 (toward zero).
 *   R6  The 22 random bits of output element e (index in the quantized
 *       operand's own [rows x K] view) come from a counter-based 32-bit hash h of
 *       the quad index e>>2, keyed by (seed, tensor id): element i = e&3 of the
 *       quad takes the top 22 bits of h rotated right by 8*i bits, so each
 *       element's leading byte is a byte of h of its own; see rand22() below.
 *   R7  A code is sign<<3 | index into the ascending value set, the sign bit
 *       being the input's sign bit (so -0 codes occur and decode to -0).
 *       Element k of a row sits in byte k/2, even k in the low nibble.
 *   R8  Re-quantizing an NVFP4 tensor (Q4, Q6 of Sec. 2.3) starts from its
 *       binary32 dequantized value  x = RN( (P * S_b) * S_g ).
 *   R12 Random Hadamard transform (Sec. 4.1, block size 16): x <- x S H along the
 *       grouped axis, before any scale is taken.  S: the sign of position k (the
 *       same for every row, and for both operands of a product) is one bit of
 *       the counter-based generator of R6 under a key of its own: bit
 *       (15 + ((k mod 32) div 2) + 16 (k mod 2)) mod 32 of the 32-bit word of
 *       counter k div 32 (every bit of a word serves exactly one position).
 *       H = H_16 (Sylvester order, entries +-1/4), evaluated in binary32 as the
 *       four butterfly stages with strides 1, 2, 4, 8 in that order, one
 *       rounding per addition, then one multiplication by 1/4 (exact).
 *
 *   R13 OsciReset (Sec. 3.2-3.3, Alg. 1; Appendix Alg. 2): the master weights are
 *       binary32; Q(W) is the forward weight quantizer Q2 applied to them - groups
 *       along the input dimension, round-to-nearest, nearest-even scales, 1 x 128
 *       outer blocks - followed by the binary32 dequantization of R8.  Distances
 *       accumulate in binary32, one rounding per operation; the risk is the
 *       binary32 quotient dist_Q / dist_M (0 / 0 compares false: an element that
 *       never moved is not reset).
 *   R14 Memory-efficient OsciReset statistics (Appendix Alg. 3): the sensitivity
 *       score of a weight is s = |w - Q(w)| / binwidth(Q(w)) in binary32, one
 *       rounding per operation, with binwidth = b(code) * RN(S_b * S_g) and b the
 *       length of the interval of scaled values that round to the code's
 *       magnitude: 0.5 for 0, 0.5, 1 and 1.5; 0.75 for 2 (1.75 .. 2.5); 1 for 3;
 *       1.5 for 4 (3.5 .. 5); 1 for 6 (5 .. 6, nothing lies beyond the block
 *       maximum).  A block with scale 0 scores 0.  "Top p %" is the k elements
 *       with the largest scores, k given by the caller; equal scores are taken in
 *       ascending index order; the index list is kept in ascending order.
 *
 * Parity status: R1, R6, R7, R12 (which bits, which summation order) are not fixed by the paper ("parity unpinned" by
 * the paper itself); they are pinned by the property tests in tests/ (grid
 * membership, exact round trips, scale/absmax invariants, closed-form SR
 * probabilities, unbiasedness, brute-force GEMMs).
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#if defined(__FAST_MATH__)
#error "the oracle must be built without -ffast-math"
#endif

enum { ROUND_RTN = 0, ROUND_SR = 1 };
enum { SCALE_DEFAULT = 0, SCALE_NE = 1, SCALE_UP = 2 };
enum { OUTER_TENSOR = 0, OUTER_BLOCK128 = 1 };

/* Sec. 2.1: FP4Values, non-negative half in ascending order. */
static const float FP4_VALUES[8] = {0.0f, 0.5f, 1.0f, 1.5f, 2.0f, 3.0f, 4.0f, 6.0f};

/* ------------------------------------------------------------------ E4M3 -- */

/* value of a non-negative E4M3 code (0x00..0x7E); R3 */
float oracle_e4m3_value(uint8_t code)
{
    int e = (code >> 3) & 0xF, m = code & 7;
    if (e == 0) return ldexpf((float)m, -9);
    return ldexpf(1.0f + (float)m / 8.0f, e - 7);
}

/* round a non-negative binary32 to an E4M3 code; R3 */
uint8_t oracle_e4m3_round(float s, int mode)
{
    if (!(s > 0.0f)) return 0;
    if (s >= 448.0f) return 0x7E;
    /* lo = largest code whose value is <= s */
    int lo = 0;
    for (int c = 1; c <= 0x7E; ++c)
        if (oracle_e4m3_value((uint8_t)c) <= s) lo = c;
    if (oracle_e4m3_value((uint8_t)lo) == s) return (uint8_t)lo;
    int hi = lo + 1;
    if (mode == SCALE_UP) return (uint8_t)hi;
    double dl = (double)s - (double)oracle_e4m3_value((uint8_t)lo);
    double dh = (double)oracle_e4m3_value((uint8_t)hi) - (double)s;
    if (dl < dh) return (uint8_t)lo;
    if (dh < dl) return (uint8_t)hi;
    return (uint8_t)((lo & 1) ? hi : lo);
}

/* ------------------------------------------------------------------- RNG -- */

static uint64_t mix64(uint64_t z)
{
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

/* R6: the 64-bit stream key of (seed, tensor id) */
uint64_t oracle_stream_key(uint64_t seed, uint32_t tensor_id)
{
    uint64_t a = mix64(seed + 0x9E3779B97F4A7C15ull);
    uint64_t b = ((uint64_t)tensor_id + 1ull) * 0xD1B54A32D192ED03ull;
    return mix64(a ^ b);
}

/* R6: 32 random bits of quad p under key (k0 = low word, k1 = high word) */
uint32_t oracle_quad_bits(uint32_t p, uint64_t key)
{
    uint32_t k0 = (uint32_t)key, k1 = (uint32_t)(key >> 32);
    uint32_t h = p + k0;
    h ^= h >> 16; h *= 0x7FEB352Du;
    h ^= h >> 15; h ^= k1; h *= 0x846CA68Bu;
    h ^= h >> 16;
    return h;
}

/* R6: 22 random bits of element e */
uint32_t oracle_rand22(uint64_t e, uint64_t key)
{
    uint32_t h = oracle_quad_bits((uint32_t)(e >> 2), key);
    unsigned i = (unsigned)(e & 3);
    uint32_t w = i ? (h >> (8 * i)) | (h << (32 - 8 * i)) : h;   /* rotate right by 8 i */
    return w >> 10;                                              /* its top 22 bits */
}

/* -------------------------------------------------------------- rounding -- */

/* Sec. 2.1 round_{FP4,D}: index of the nearest FP4 value to a in [0,6]; ties to even index (R4) */
int oracle_round_rtn(float a)
{
    int best = 0;
    double bd = fabs((double)a - (double)FP4_VALUES[0]);
    for (int i = 1; i < 8; ++i) {
        double d = fabs((double)a - (double)FP4_VALUES[i]);
        if (d < bd || (d == bd && (i % 2 == 0))) { best = i; bd = d; }
    }
    return best;
}

/* Sec. 2.1 round_{FP4,S} with the discrete uniform of R5; u22 in [0, 2^22) */
int oracle_round_sr(float a, uint32_t u22)
{
    if (a >= 6.0f) return 7;
    int i1 = 0;
    for (int i = 0; i < 7; ++i)
        if (FP4_VALUES[i] <= a) i1 = i;                               /* q1 <= a < q2 */
    float q1 = FP4_VALUES[i1], q2 = FP4_VALUES[i1 + 1];
    double f = ((double)a - (double)q1) / ((double)q2 - (double)q1);
    uint32_t L = (uint32_t)floor(f * 4194304.0);                      /* R5: q2 iff f + u / 2^22 >= 1 */
    return (u22 + L >= 4194304u) ? i1 + 1 : i1;
}

/* test helper: over all 2^22 values of u, how often a is rounded up (returns -1 if the rounded-up set is not
 * the upper interval of u, or a result other than the two neighbours appears) */
int64_t oracle_round_sr_count_up(float a, int *lower_index)
{
    int base = oracle_round_sr(a, 0);
    int64_t ups = 0;
    int seen_up = 0;
    for (uint32_t u = 0; u < 4194304u; ++u) {
        int m = oracle_round_sr(a, u);
        if (m == base + 1) { seen_up = 1; ++ups; }
        else if (m != base || seen_up) return -1;
    }
    *lower_index = base;
    return ups;
}

/* ------------------------------------------------------------------- RHT -- */

/* R12: sign of position k along the grouped axis (1 = flipped) */
int oracle_rht_sign(uint64_t k, uint64_t key)
{
    uint32_t w = oracle_quad_bits((uint32_t)(k >> 5), key);
    unsigned bit = (unsigned)((15 + ((k & 31) >> 1) + 16 * (k & 1)) & 31);
    return (int)((w >> bit) & 1u);
}

/* Sec. 4.1: x <- x S H_16 on every aligned run of 16 along K, in place; x is [rows][K] (R12) */
int oracle_rht16_rows(float *x, int64_t rows, int64_t K, uint64_t key)
{
    if (rows < 0 || K < 0 || K % 16) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t b = 0; b < K / 16; ++b) {
            volatile float v[16];
            for (int i = 0; i < 16; ++i) {
                float xi = x[r * K + b * 16 + i];
                v[i] = oracle_rht_sign((uint64_t)(b * 16 + i), key) ? -xi : xi;
            }
            for (int h = 1; h < 16; h <<= 1)                     /* H_2d = [H_d H_d; H_d -H_d] / sqrt 2, unnormalised */
                for (int i = 0; i < 16; ++i)
                    if (!(i & h)) {
                        float a = v[i], c = v[i + h];
                        v[i] = a + c;
                        v[i + h] = a - c;
                    }
            for (int i = 0; i < 16; ++i) x[r * K + b * 16 + i] = v[i] * 0.25f;   /* (1 / sqrt 2)^4 */
        }
    return 0;
}

/* ------------------------------------------------------------- quantizer -- */

static float abs_max(const float *x, int64_t n)
{
    float m = 0.0f;
    for (int64_t i = 0; i < n; ++i) { float v = fabsf(x[i]); if (v > m) m = v; }
    return m;
}

/* Sec. 2.2: S_global of an outer group with absolute maximum amax (R1, R2) */
float oracle_global_scale(float amax)
{
    if (amax == 0.0f) return 1.0f;
    volatile float q = amax / 2688.0f;                 /* 448 * 6 */
    float floor_ = ldexpf(1.0f, -100);
    return q > floor_ ? q : floor_;
}

/*
 * Quantize x, viewed as [rows x K] with K the grouped (contiguous) axis.
 *   codes  [rows][K/2], scales [rows][K/16],
 *   gscale [1] (TENSOR) or [rows][K/128] (BLOCK128),
 *   amax_deq (optional, [1]): max |binary32 dequantized value| of the result.
 * Returns 0, or -1 on a bad shape / enum.
 */
static int quantize_rows_impl(const float *x, int64_t rows, int64_t K,
                              int rounding, int scale_round, int outer_mode,
                              uint64_t seed, uint32_t tensor_id,
                              uint8_t *codes, uint8_t *scales, float *gscale, float *amax_deq, float *y_out,
                              int64_t row0, const float *tensor_amax)
{
    /* x holds rows row0 .. row0 + rows - 1 of the tensor (row0 = 0: all of it); tensor_amax, when given, is the
     * whole tensor's max |x| (needed when x is only a slice) */
    if (rows < 0 || K < 0 || K % 16 || row0 < 0) return -1;
    if (outer_mode == OUTER_BLOCK128 && K % 128) return -1;
    if (outer_mode != OUTER_TENSOR && outer_mode != OUTER_BLOCK128) return -1;
    if (rounding != ROUND_RTN && rounding != ROUND_SR) return -1;
    if (scale_round == SCALE_DEFAULT) scale_round = rounding == ROUND_RTN ? SCALE_NE : SCALE_UP;
    if (scale_round != SCALE_NE && scale_round != SCALE_UP) return -1;
    if ((double)(row0 + rows) * (double)K > 17179869184.0) return -1;       /* quad index must fit 32 bits */

    const uint64_t key = oracle_stream_key(seed, tensor_id);
    const int64_t outer_len = outer_mode == OUTER_TENSOR ? K : 128;
    const int64_t outer_per_row = outer_mode == OUTER_TENSOR ? 1 : K / 128;

    float tensor_sg = 1.0f;
    if (outer_mode == OUTER_TENSOR) {
        float amax = 0.0f;
        for (int64_t r = 0; r < rows; ++r) { float m = abs_max(x + r * K, K); if (m > amax) amax = m; }
        if (tensor_amax) amax = *tensor_amax;
        tensor_sg = oracle_global_scale(amax);
        gscale[0] = tensor_sg;
    }

    float deq_max = 0.0f;
#pragma omp parallel for schedule(static) reduction(max : deq_max)
    for (int64_t r = 0; r < rows; ++r) {
        const float *xr = x + r * K;
        for (int64_t g = 0; g < outer_per_row; ++g) {
            float S_g = tensor_sg;
            if (outer_mode == OUTER_BLOCK128) {
                S_g = oracle_global_scale(abs_max(xr + g * 128, 128));
                gscale[r * outer_per_row + g] = S_g;
            }
            volatile float inv_sg = 1.0f / S_g;
            volatile float sixth = 1.0f / 6.0f;
            volatile float inv_cg = inv_sg * sixth;                     /* 1 / (6 S_global) */
            for (int64_t b = g * outer_len / 16; b < (g + 1) * outer_len / 16; ++b) {
                const float *xb = xr + b * 16;
                float amax_b = abs_max(xb, 16);
                volatile float s = amax_b * inv_cg;                    /* Sec. 2.2, S_block */
                uint8_t sc = oracle_e4m3_round(s, scale_round);
                scales[r * (K / 16) + b] = sc;
                float S_b = oracle_e4m3_value(sc);
                volatile float inv_sb = sc == 0 ? 0.0f : 1.0f / S_b;
                volatile float rcp = inv_sg * inv_sb;                   /* 1 / (S_global * S_block) */
                for (int i = 0; i < 16; ++i) {
                    int64_t k = b * 16 + i;
                    volatile float y = xb[i] * rcp;                    /* Sec. 2.2, argument of round_FP4 */
                    if (y_out) y_out[r * K + k] = y;
                    float a = fabsf(y); if (a > 6.0f) a = 6.0f;
                    int m;
                    if (rounding == ROUND_RTN) m = oracle_round_rtn(a);
                    else m = oracle_round_sr(a, oracle_rand22((uint64_t)((row0 + r) * K + k), key));
                    int neg = signbit(xb[i]) != 0;
                    uint8_t nib = (uint8_t)((neg << 3) | m);
                    uint8_t *byte = codes + r * (K / 2) + k / 2;
                    if (k & 1) *byte = (uint8_t)((*byte & 0x0F) | (nib << 4));
                    else       *byte = (uint8_t)((*byte & 0xF0) | nib);
                    volatile float pv = FP4_VALUES[m] * S_b;           /* exact */
                    volatile float dq = pv * S_g;
                    if (dq > deq_max) deq_max = dq;
                }
            }
        }
    }
    if (amax_deq) *amax_deq = deq_max;
    return 0;
}

int oracle_quantize_rows(const float *x, int64_t rows, int64_t K,
                         int rounding, int scale_round, int outer_mode,
                         uint64_t seed, uint32_t tensor_id,
                         uint8_t *codes, uint8_t *scales, float *gscale, float *amax_deq)
{
    return quantize_rows_impl(x, rows, K, rounding, scale_round, outer_mode, seed, tensor_id, codes, scales, gscale,
                              amax_deq, NULL, 0, NULL);
}

/* test helper: the same, and also the argument y of round_FP4 for every element ([rows][K]) */
int oracle_quantize_rows_y(const float *x, int64_t rows, int64_t K,
                           int rounding, int scale_round, int outer_mode,
                           uint64_t seed, uint32_t tensor_id,
                           uint8_t *codes, uint8_t *scales, float *gscale, float *amax_deq, float *y_out)
{
    return quantize_rows_impl(x, rows, K, rounding, scale_round, outer_mode, seed, tensor_id, codes, scales, gscale,
                              amax_deq, y_out, 0, NULL);
}

/* test helper: rows row0 .. row0 + rows - 1 of a larger tensor whose max |x| is tensor_amax (per-tensor outer scale);
 * the outputs cover the slice only.  The bytes equal those rows of the whole tensor's quantization. */
int oracle_quantize_rows_slice(const float *x, int64_t rows, int64_t K,
                               int rounding, int scale_round, int outer_mode,
                               uint64_t seed, uint32_t tensor_id, int64_t row0, float tensor_amax,
                               uint8_t *codes, uint8_t *scales, float *gscale)
{
    return quantize_rows_impl(x, rows, K, rounding, scale_round, outer_mode, seed, tensor_id, codes, scales, gscale,
                              NULL, NULL, row0, &tensor_amax);
}

/* test helper: the 22 random bits of elements 0 .. n-1 of a stream */
void oracle_rand22_fill(uint64_t key, int64_t n, uint32_t *out)
{
    for (int64_t e = 0; e < n; ++e) out[e] = oracle_rand22((uint64_t)e, key);
}

/* ----------------------------------------------------------- dequantizers -- */

static float code_value(uint8_t nib)
{
    float v = FP4_VALUES[nib & 7];
    return (nib & 8) ? -v : v;
}

/* R8: binary32 dequantized value RN((P*S_b)*S_g), layout [rows][K] */
int oracle_dequant_f32(const uint8_t *codes, const uint8_t *scales, const float *gscale,
                       int64_t rows, int64_t K, int outer_mode, float *out)
{
    if (K % 16 || (outer_mode == OUTER_BLOCK128 && K % 128)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            uint8_t byte = codes[r * (K / 2) + k / 2];
            uint8_t nib = (k & 1) ? (byte >> 4) : (byte & 0xF);
            float S_b = oracle_e4m3_value(scales[r * (K / 16) + k / 16]);
            float S_g = outer_mode == OUTER_TENSOR ? gscale[0] : gscale[r * (K / 128) + k / 128];
            volatile float pv = code_value(nib) * S_b;
            volatile float dq = pv * S_g;
            out[r * K + k] = dq;
        }
    return 0;
}

/* exact dequantized value P*S_b*S_g in binary64 (at most 30 significant bits), layout [rows][K] */
int oracle_dequant_f64(const uint8_t *codes, const uint8_t *scales, const float *gscale,
                       int64_t rows, int64_t K, int outer_mode, double *out)
{
    if (K % 16 || (outer_mode == OUTER_BLOCK128 && K % 128)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < K; ++k) {
            uint8_t byte = codes[r * (K / 2) + k / 2];
            uint8_t nib = (k & 1) ? (byte >> 4) : (byte & 0xF);
            double S_b = (double)oracle_e4m3_value(scales[r * (K / 16) + k / 16]);
            double S_g = (double)(outer_mode == OUTER_TENSOR ? gscale[0] : gscale[r * (K / 128) + k / 128]);
            out[r * K + k] = (double)code_value(nib) * S_b * S_g;
        }
    return 0;
}

/* -------------------------------------------------------------- OsciReset -- */

/* Q(W) of R13: quantize-dequantize a binary32 [rows][K] matrix the way the forward pass quantizes a weight */
int oracle_quant_dequant_weight(const float *W, int64_t rows, int64_t K, float *out)
{
    if (rows < 0 || K < 0 || K % 128) return -1;
    uint8_t *codes = (uint8_t *)calloc((size_t)(rows * K / 2) + 1, 1);
    uint8_t *scales = (uint8_t *)calloc((size_t)(rows * K / 16) + 1, 1);
    float *gs = (float *)calloc((size_t)(rows * (K / 128)) + 1, sizeof(float));
    int rc = quantize_rows_impl(W, rows, K, ROUND_RTN, SCALE_NE, OUTER_BLOCK128, 0, 0, codes, scales, gs, NULL, NULL, 0, NULL);
    if (rc == 0) rc = oracle_dequant_f32(codes, scales, gs, rows, K, OUTER_BLOCK128, out);
    free(codes); free(scales); free(gs);
    return rc;
}

/* Appendix Alg. 2 (UpdateOscillationStats) for one weight matrix.  t0 = 0 opens a period: the distances are cleared
 * and the snapshot W' is taken.  Otherwise dist_M += |W - W'|, dist_Q += |Q(W) - Q(W')|, then W' <- W. */
int oracle_osci_update(const float *W, float *W_prev, float *dist_m, float *dist_q, int64_t rows, int64_t K, int t0)
{
    if (rows < 0 || K < 0 || K % 128 || t0 < 0) return -1;
    const int64_t n = rows * K;
    if (t0 == 0) {
        for (int64_t i = 0; i < n; ++i) { dist_m[i] = 0.0f; dist_q[i] = 0.0f; W_prev[i] = W[i]; }
        return 0;
    }
    float *q = (float *)malloc(sizeof(float) * (size_t)(n + 1)), *qp = (float *)malloc(sizeof(float) * (size_t)(n + 1));
    int rc = oracle_quant_dequant_weight(W, rows, K, q);
    if (rc == 0) rc = oracle_quant_dequant_weight(W_prev, rows, K, qp);
    if (rc == 0)
        for (int64_t i = 0; i < n; ++i) {
            volatile float dm = fabsf(W[i] - W_prev[i]);
            volatile float dq = fabsf(q[i] - qp[i]);
            volatile float am = dist_m[i] + dm, aq = dist_q[i] + dq;
            dist_m[i] = am;
            dist_q[i] = aq;
            W_prev[i] = W[i];
        }
    free(q); free(qp);
    return rc;
}

/* Alg. 1 (OscillationSuppress) for one weight matrix: every element whose risk dist_Q / dist_M reaches tau is reset to
 * the centre of its quantization bin, w <- w_FP4 * scale = Q(W) at that element.  Returns the number of resets (< 0: error). */
int64_t oracle_osci_suppress(float *W, const float *dist_m, const float *dist_q, float tau, int64_t rows, int64_t K)
{
    if (rows < 0 || K < 0 || K % 128) return -1;
    const int64_t n = rows * K;
    float *q = (float *)malloc(sizeof(float) * (size_t)(n + 1));
    int64_t count = 0;
    if (oracle_quant_dequant_weight(W, rows, K, q) != 0) { free(q); return -1; }
    for (int64_t i = 0; i < n; ++i) {
        volatile float risk = dist_q[i] / dist_m[i];
        if (risk >= tau) { W[i] = q[i]; ++count; }
    }
    free(q);
    return count;
}

/* Appendix Alg. 3, first step of a period: Q(W) and the sensitivity score of every element (R14).  Either output may
 * be NULL.  Selection of the top k scores and the gathers are left to the caller (plain array operations). */
int oracle_osci_scores(const float *W, int64_t rows, int64_t K, float *q_out, float *score)
{
    static const float bin[8] = {0.5f, 0.5f, 0.5f, 0.5f, 0.75f, 1.0f, 1.5f, 1.0f};
    if (rows < 0 || K < 0 || K % 128) return -1;
    uint8_t *codes = (uint8_t *)calloc((size_t)(rows * K / 2) + 1, 1);
    uint8_t *scales = (uint8_t *)calloc((size_t)(rows * K / 16) + 1, 1);
    float *gs = (float *)calloc((size_t)(rows * (K / 128)) + 1, sizeof(float));
    float *q = (float *)malloc(sizeof(float) * (size_t)(rows * K + 1));
    int rc = quantize_rows_impl(W, rows, K, ROUND_RTN, SCALE_NE, OUTER_BLOCK128, 0, 0, codes, scales, gs, NULL, NULL, 0, NULL);
    if (rc == 0) rc = oracle_dequant_f32(codes, scales, gs, rows, K, OUTER_BLOCK128, q);
    if (rc == 0)
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t k = 0; k < K; ++k) {
                const int64_t i = r * K + k;
                uint8_t byte = codes[r * (K / 2) + k / 2];
                uint8_t nib = (k & 1) ? (byte >> 4) : (byte & 0xF);
                float S_b = oracle_e4m3_value(scales[r * (K / 16) + k / 16]);
                float S_g = gs[r * (K / 128) + k / 128];
                volatile float unit = S_b * S_g;
                volatile float width = bin[nib & 7] * unit;
                volatile float num = fabsf(W[i] - q[i]);
                volatile float sc = width == 0.0f ? 0.0f : num / width;
                if (score) score[i] = sc;
                if (q_out) q_out[i] = q[i];
            }
    free(codes); free(scales); free(gs); free(q);
    return rc;
}

/* ------------------------------------------------------------------ GEMM -- */

/* Sec. 2.3: C[m][n] = sum_k A[m][k] * B[n][k], binary64, k in ascending order.
 * abs_sum (optional) receives sum_k |A[m][k]| |B[n][k]| for tolerance scaling. */
int oracle_gemm_nt_f64(const double *A, const double *B, int64_t M, int64_t N, int64_t K,
                       double *C, double *abs_sum)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0, aacc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = A[m * K + k] * B[n * K + k];
                acc += p;
                aacc += fabs(p);
            }
            C[m * N + n] = acc;
            if (abs_sum) abs_sum[m * N + n] = aacc;
        }
    return 0;
}

/* ---------------------------------------------------------------- helpers -- */

void oracle_bf16_to_f32(const uint16_t *src, int64_t n, float *dst)
{
    for (int64_t i = 0; i < n; ++i) {
        uint32_t b = (uint32_t)src[i] << 16;
        memcpy(dst + i, &b, 4);
    }
}

/* dst[c][r] = src[r][c] */
void oracle_transpose_f32(const float *src, int64_t R, int64_t C, float *dst)
{
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < C; ++c)
        for (int64_t r = 0; r < R; ++r) dst[c * R + r] = src[r * C + c];
}

float oracle_abs_max_f32(const float *x, int64_t n) { return abs_max(x, n); }
