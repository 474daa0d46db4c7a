// Device-side number-format helpers for the NVFP4 kernels (gfx950).
//
// E2M1 / E4M3 / double-block arithmetic of TetraJet-v2 Sec. 2.1-2.2, written as
// bit manipulation on binary32.  Everything that decides a code is plain IEEE
// binary32 with one rounding per operation (the translation unit is compiled with
// -ffp-contract=off and subnormals enabled).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tj {

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }

// ---- lane exchange inside a row of 16 lanes (DPP) -------------------------------------------
template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
constexpr int DPP_QUAD_XOR1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_XOR2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int DPP_ROW_HALF_MIRROR = 0x141; // lane i <-> 7-i inside 8
constexpr int DPP_ROW_MIRROR = 0x140;      // lane i <-> 15-i inside 16
constexpr int DPP_ROW_SHL2 = 0x102;        // lane i reads lane i+2
constexpr int DPP_ROW_SHL4 = 0x104;        // lane i reads lane i+4

__device__ __forceinline__ float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- E4M3 (bias 7, no infinity, max 448 = 0x7E, subnormals k * 2^-9) ------------------------

// value of a code: the 7 payload bits sit where binary32 keeps exponent and top mantissa
// bits once shifted by 20; the 2^120 factor re-biases (127 - 7) and normalises subnormals.
__device__ __forceinline__ float e4m3_value(uint32_t code) { return u2f(code << 20) * 0x1p120f; }

// round a non-negative binary32 to the nearest code, ties to the even code, saturating
__device__ __forceinline__ uint32_t e4m3_round_ne(float s)
{
    uint32_t b = f2u(s);
    uint32_t rn = (b + 0x7FFFFu + ((b >> 20) & 1u)) >> 20;     // round mantissa to 3 bits
    int cn = (int)rn - (120 << 3);
    cn = cn > 0x7E ? 0x7E : cn;
    uint32_t cs = f2u(s + 16384.0f) & 0xFFu;                   // below 2^-6: multiples of 2^-9
    return s < 0x1p-6f ? cs : (uint32_t)cn;
}

// smallest code whose value is >= s, saturating
__device__ __forceinline__ uint32_t e4m3_round_up(float s)
{
    uint32_t b = f2u(s);
    int cn = (int)((b + 0xFFFFFu) >> 20) - (120 << 3);
    cn = cn > 0x7E ? 0x7E : cn;
    uint32_t cs = (uint32_t)ceilf(s * 512.0f);
    return s < 0x1p-6f ? cs : (uint32_t)cn;
}

// reciprocals of all E4M3 values into a 128-entry table (entry 0 = 0, so a zero scale gives all-zero codes); the first
// 128 threads of the workgroup write it, a barrier must follow
__device__ __forceinline__ void fill_inv_table(float *tab)
{
    if (threadIdx.x < 128) {
        float v = e4m3_value(threadIdx.x);
        tab[threadIdx.x] = (threadIdx.x == 0 || threadIdx.x == 127) ? 0.0f : 1.0f / v;
    }
}

template <bool UP>
__device__ __forceinline__ uint32_t e4m3_round(float s) { return UP ? e4m3_round_up(s) : e4m3_round_ne(s); }

// ---- E2M1 -----------------------------------------------------------------------------------

// value of a 3-bit magnitude code: E2M1 is a tiny IEEE format (bias 1, subnormal 0.5)
__device__ __forceinline__ float e2m1_value(uint32_t m) { return u2f(m << 22) * 0x1p126f; }

// Sec. 2.1 deterministic rounding of y: nearest value, ties to the even code, |y| clamped to 6;
// returns sign<<3 | magnitude code, the sign being y's sign bit
__device__ __forceinline__ uint32_t e2m1_rtn(float y)
{
    float a = fminf(fabsf(y), 6.0f);
    uint32_t b = f2u(fmaxf(a, 1.0f));
    uint32_t hi = (b + 0x1FFFFFu + ((b >> 22) & 1u)) >> 22;    // 254 (a <= 1) .. 259 (a = 6)
    uint32_t lo = (a > 0.25f ? 1u : 0u) + (a >= 0.75f ? 1u : 0u);
    return (hi + lo - 254u) | ((f2u(y) >> 28) & 8u);
}

// The same rounding for two values at once by the hardware's FP32 -> FP4 conversion, which lands in byte
// SEL of `old`: first value in the low nibble.  (It agrees with e2m1_rtn on every binary32 pattern below
// 16 in magnitude, both signs, -0 and subnormals included.)
template <int SEL>
__device__ __forceinline__ uint32_t e2m1_rtn_pair(uint32_t old, float y0, float y1)
{
    return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(old, y0, y1, 1.0f, SEL);
}

// Sec. 2.1 stochastic rounding of two values by the hardware's FP32 -> FP4 conversion with a random word.  Scaled
// by 2^-126 a magnitude's binary32 pattern is its E2M1 pattern extended by 22 fraction bits (fixed point below 1,
// where bits of the value below 2^-23 are dropped); the conversion adds 22 random bits to that fraction, truncates
// and saturates at 6, so a value moves to its upper neighbour with probability frac exactly.
// The first value takes bits 31..10 of the random word, the second bits 30..9: the two draws of one conversion
// share all but one bit, so a caller that wants independent draws converts twice and keeps one nibble of each.
//
// e2m1_sr8 rounds eight values: the even ones with the words h[j], the odd ones with the words g[j]; element 0 lands
// in the low nibble.  Written as one block of instructions because the conversion keeps the other three bytes of its
// destination, which the compiler's builtin for it does not model (it lets later conversions land in other
// registers); the two destination chains alternate so that no conversion follows the one it depends on directly,
// and the closing idle cycle covers the partial-register write before the first reader.
__device__ __forceinline__ uint32_t e2m1_sr8(float y0, float y1, float y2, float y3, float y4, float y5, float y6,
                                             float y7, const uint32_t (&h)[4], const uint32_t (&g)[4])
{
    const float2_t p0 = {y0, y1}, p1 = {y2, y3}, p2 = {y4, y5}, p3 = {y6, y7};
    uint32_t lo, hi;
    asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %2, %6, 1.0\n\t"
        "v_cvt_scalef32_sr_pk_fp4_f32 %1, %2, %10, 1.0\n\t"
        "v_cvt_scalef32_sr_pk_fp4_f32 %0, %3, %7, 1.0 op_sel:[0,0,1,0]\n\t"
        "v_cvt_scalef32_sr_pk_fp4_f32 %1, %3, %11, 1.0 op_sel:[0,0,1,0]\n\t"
        "v_cvt_scalef32_sr_pk_fp4_f32 %0, %4, %8, 1.0 op_sel:[0,0,0,1]\n\t"
        "v_cvt_scalef32_sr_pk_fp4_f32 %1, %4, %12, 1.0 op_sel:[0,0,0,1]\n\t"
        "v_cvt_scalef32_sr_pk_fp4_f32 %0, %5, %9, 1.0 op_sel:[0,0,1,1]\n\t"
        "v_cvt_scalef32_sr_pk_fp4_f32 %1, %5, %13, 1.0 op_sel:[0,0,1,1]\n\t"
        "s_nop 0"
        : "=&v"(lo), "=&v"(hi)
        : "v"(p0), "v"(p1), "v"(p2), "v"(p3), "v"(h[0]), "v"(h[1]), "v"(h[2]), "v"(h[3]), "v"(g[0]), "v"(g[1]),
          "v"(g[2]), "v"(g[3]));
    return (lo & 0x0F0F0F0Fu) | (hi & 0xF0F0F0F0u);
}

// ---- stochastic-rounding bit generator --------------------------------------------------------

// 32 bits for the element quad p (four consecutive elements of the quantized operand) of a stream
// keyed by (k0, k1): two rounds of xorshift-multiply with the second key word folded in between
__device__ __forceinline__ uint32_t quad_bits(uint32_t p, uint32_t k0, uint32_t k1)
{
    uint32_t h = p + k0;
    h ^= h >> 16;
    h *= 0x7FEB352Du;
    h = h ^ (h >> 15) ^ k1;
    h *= 0x846CA68Bu;
    h ^= h >> 16;
    return h;
}

// ---- random Hadamard transform (Sec. 4.1, block 16) ------------------------------------------

// x <- x H_16 (Sylvester order, entries +-1/4) on 16 values held by one lane: the four butterfly stages with strides
// 1, 2, 4, 8 in that order, one rounding per addition, then the (exact) factor 1/4
__device__ __forceinline__ void fwht16(float (&v)[16])
{
#pragma unroll
    for (int h = 1; h < 16; h <<= 1)
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (!(i & h)) {
                const float a = v[i], c = v[i + h];
                v[i] = a + c;
                v[i + h] = a - c;
            }
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = v[i] * 0.25f;
}

// Bit of a sign word that decides position k (k mod 32 = e) along the grouped axis: every bit serves one position.
// With this numbering the two bf16 of dword j of an aligned 8-run starting at e0 flip under
// rotate_right(word, e0 / 2 + j) & 0x80008000.
__device__ __forceinline__ constexpr int rht_sign_bit(int e) { return (15 + (e >> 1) + 16 * (e & 1)) & 31; }

// ---- outer scale (Sec. 2.2, S_global) ---------------------------------------------------------

struct OuterScale {
    float S_g;     // amax / (448*6), floored at 2^-100; 1 for an all-zero group
    float inv_sg;  // 1 / S_g
    float inv_cg;  // (1 / S_g) * (1/6)
};

__device__ __forceinline__ OuterScale outer_scale(float amax)
{
    OuterScale o;
    float q = amax / 2688.0f;
    q = fmaxf(q, 0x1p-100f);
    o.S_g = amax == 0.0f ? 1.0f : q;
    o.inv_sg = 1.0f / o.S_g;
    o.inv_cg = o.inv_sg * (1.0f / 6.0f);
    return o;
}

// bf16 pair -> two binary32
__device__ __forceinline__ float bf16_lo(uint32_t w) { return u2f(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return u2f(w & 0xFFFF0000u); }

__device__ __forceinline__ ushort2_t as_us2(uint32_t w) { return __builtin_bit_cast(ushort2_t, w); }
__device__ __forceinline__ uint32_t as_u32(ushort2_t v) { return __builtin_bit_cast(uint32_t, v); }

// max |.| of the 8 bf16 in v, as the bf16 bit pattern (finite inputs order like integers)
__device__ __forceinline__ uint32_t absmax8_bits(uint4 v)
{
    ushort2_t a = as_us2(v.x & 0x7FFF7FFFu), b = as_us2(v.y & 0x7FFF7FFFu);
    ushort2_t c = as_us2(v.z & 0x7FFF7FFFu), d = as_us2(v.w & 0x7FFF7FFFu);
    ushort2_t m = __builtin_elementwise_max(__builtin_elementwise_max(a, b), __builtin_elementwise_max(c, d));
    return m.x > m.y ? m.x : m.y;
}

}  // namespace tj
