// NVFP4 double-block quantizer kernels for gfx950 (TetraJet-v2 Sec. 2.1-2.2, the six
// quantizers of Sec. 2.3).  All of them are bandwidth-bound streaming kernels:
//   amax_partials   per-tensor max|x| of a bf16 array (TENSOR outer mode only)
//   quant_row       groups of 16 along the contiguous axis; 8 elements (one 128-bit load) per
//                   lane, two lanes per group, group maximum exchanged by DPP
//   quant_colw      groups of 16 down the columns, bf16 or packed NVFP4 source (Q5; Q4 / Q6): a wave owns a
//                   128 x 128 strip, a lane two columns; the output is the transposed operand
//   quant_dual      row-wise and column-wise operand of one bf16 tensor from one read (Q3 + Q5)
#include <type_traits>

#include "device_fmt.h"
#include "internal.h"

namespace tj {

namespace {

constexpr int kThreads = 256;
constexpr int kRowIter = 4;    // 128-bit chunks per thread in the row kernel

// 128-bit load of source data that this kernel reads exactly once (streaming hint: the line need not stay cached)
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_stream(const uint4 *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

struct KArgs {
    uint32_t *codes;
    uint8_t *scales;
    float *gscale;
    float *amax_deq;
    const float *amax_scalar;
    const float *amax_partials;
    int npart;
    uint32_t k0, k1;
    uint32_t r0, r1;      // random Hadamard transform: key words of the sign stream
};

// tensor maximum for this workgroup: a scalar, or the maximum of the partials
__device__ __forceinline__ float block_tensor_amax(const KArgs &a, float *red)
{
    if (a.amax_scalar) return a.amax_scalar[0];
    float m = 0.0f;
    for (int i = threadIdx.x; i < a.npart; i += kThreads) m = fmaxf(m, a.amax_partials[i]);
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// eight consecutive elements of one group -> eight codes in one dword (element 0 in the low nibble)
template <int ROUND, bool SUP>
__device__ __forceinline__ uint32_t quant8(const float (&x)[8], float r, uint32_t quad0, uint32_t k0, uint32_t k1)
{
    uint32_t out = 0;
    if (ROUND == 0) {
        out = e2m1_rtn_pair<0>(out, x[0] * r, x[1] * r);
        out = e2m1_rtn_pair<1>(out, x[2] * r, x[3] * r);
        out = e2m1_rtn_pair<2>(out, x[4] * r, x[5] * r);
        out = e2m1_rtn_pair<3>(out, x[6] * r, x[7] * r);
        return out;
    }
    // One 32-bit hash per four elements; element i of the quad is rounded with the top 22 bits of the hash rotated
    // right by 8 i, so its leading byte is a byte of its own.  The conversion looks at bits 31..10 of the word for
    // its first value and at bits 30..9 for its second, hence the rotation by one more bit for odd elements; two
    // conversions per pair, the first supplying the low nibbles, the second the high nibbles.  The conversion
    // saturates at 6 by itself.
    const uint32_t ha = quad_bits(quad0, k0, k1), hb = quad_bits(quad0 + 1, k0, k1);
    const uint32_t h[4] = {ha, __builtin_amdgcn_alignbit(ha, ha, 16), hb, __builtin_amdgcn_alignbit(hb, hb, 16)};
    const uint32_t g[4] = {__builtin_amdgcn_alignbit(ha, ha, 9), __builtin_amdgcn_alignbit(ha, ha, 25),
                           __builtin_amdgcn_alignbit(hb, hb, 9), __builtin_amdgcn_alignbit(hb, hb, 25)};
    return e2m1_sr8(x[0] * r, x[1] * r, x[2] * r, x[3] * r, x[4] * r, x[5] * r, x[6] * r, x[7] * r, h, g);
}

// workgroup maximum -> one atomic, and only if it can still raise the published value (the
// published value only grows, so a stale read costs an extra atomic, never a wrong result)
__device__ __forceinline__ void publish_deq_max(float v, float *dst, float *red)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        v = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        if (v > __builtin_nontemporal_load(dst)) atomicMax(reinterpret_cast<unsigned int *>(dst), f2u(v));
    }
}

// ------------------------------------------------------------------------------- amax ----

// One launch can serve two tensors (the two operands of a forward call): workgroups [0, j0.nblocks) take the first
// job, the rest the second.
struct AmaxJob {
    const uint4 *src;
    int64_t nchunks;
    float *partials;
    float *zero_me;       // optional: a float this launch also clears
    unsigned nblocks;
};

__global__ __launch_bounds__(kThreads) void amax_partials_kernel(AmaxJob j0, AmaxJob j1)
{
    __shared__ float red[4];
    const bool second = blockIdx.x >= j0.nblocks;
    const uint4 *__restrict__ src = second ? j1.src : j0.src;
    const int64_t nchunks = second ? j1.nchunks : j0.nchunks;
    float *partials = second ? j1.partials : j0.partials;
    float *zero_me = second ? j1.zero_me : j0.zero_me;
    const unsigned bid = second ? blockIdx.x - j0.nblocks : blockIdx.x, nb = second ? j1.nblocks : j0.nblocks;
    if (zero_me && bid == 0 && threadIdx.x == 0) zero_me[0] = 0.0f;
    uint32_t m = 0;
    const int64_t stride = (int64_t)nb * kThreads;
    int64_t c = (int64_t)bid * kThreads + threadIdx.x;
    for (; c + 3 * stride < nchunks; c += 4 * stride) {
        // streaming loads: measured 2 % on a whole layer step against ordinary loads
        uint4 v0 = ld_stream(src + c), v1 = ld_stream(src + c + stride), v2 = ld_stream(src + c + 2 * stride),
              v3 = ld_stream(src + c + 3 * stride);
        uint32_t a = absmax8_bits(v0), b = absmax8_bits(v1), d = absmax8_bits(v2), e = absmax8_bits(v3);
        uint32_t ab = a > b ? a : b, de = d > e ? d : e;
        uint32_t q = ab > de ? ab : de;
        m = m > q ? m : q;
    }
    for (; c < nchunks; c += stride) {
        uint32_t q = absmax8_bits(src[c]);
        m = m > q ? m : q;
    }
    float f = wave_max(u2f(m << 16));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = f;
    __syncthreads();
    if (threadIdx.x == 0) partials[bid] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// out may alias partials: it is written after every partial has been read
__global__ __launch_bounds__(kThreads) void amax_final_kernel(const float *partials, int npart, float *out)
{
    __shared__ float red[4];
    float m = 0.0f;
    for (int i = threadIdx.x; i < npart; i += kThreads) m = fmaxf(m, partials[i]);
    m = wave_max(m);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

__global__ void zero_scalar_kernel(float *p) { p[0] = 0.0f; }

// ---------------------------------------------------------------------------- row-wise ----

struct RowJob {
    const uint4 *src;
    int64_t nchunks;
    KArgs a;
    uint32_t nblk;       // RHT: 128-element blocks per row (K / 128)
};

// first_second: first workgroup of the second job (0xFFFFFFFF when the launch has one job)
// RHT (1 x 128 outer blocks only): every group of 16 is first multiplied by S H_16 (Sec. 4.1).  The two lanes of a
// group do the strides 1, 2, 4 on their own eight values and the stride 8 across the pair; the signs come from a
// table of the 256 sign words (32 positions each) that the workgroup's 64 outer blocks can touch.
template <int ROUND, bool SUP, int OUTER, bool DEQ, bool RHT = false>
__global__ __launch_bounds__(kThreads) void quant_row_kernel(RowJob j0, RowJob j1, unsigned first_second)
{
    static_assert(!RHT || (OUTER == 1 && !DEQ), "the transform is provided with 1 x 128 outer blocks");
    __shared__ float inv_tab[128];
    __shared__ float red[4];
    __shared__ uint32_t sign_tab[RHT ? kThreads : 1];
    const int tid = threadIdx.x;
    const bool second = blockIdx.x >= first_second;
    const uint4 *__restrict__ src = second ? j1.src : j0.src;
    const int64_t nchunks = second ? j1.nchunks : j0.nchunks;
    const KArgs a = second ? j1.a : j0.a;
    const unsigned bid = second ? blockIdx.x - first_second : blockIdx.x;
    // the workgroup's data first: these loads do not depend on the scale set-up below and overlap with it
    const int64_t c0 = (int64_t)bid * kRowIter * kThreads + tid;
    const bool full = ((int64_t)bid + 1) * kRowIter * kThreads <= nchunks;
    uint4 vs[kRowIter];
#pragma unroll
    for (int it = 0; it < kRowIter; ++it) {
        vs[it] = make_uint4(0, 0, 0, 0);
        if (full || c0 + it * kThreads < nchunks) vs[it] = ld_stream(src + c0 + it * kThreads);
    }
    fill_inv_table(inv_tab);
    if (RHT) {
        // entry t: sign word (t & 3) of the (t >> 2)-th outer block this workgroup covers; blocks wrap at the end of a row
        const uint32_t nblk = second ? j1.nblk : j0.nblk;
        const uint32_t kb = (uint32_t)(((uint64_t)bid * (kRowIter * kThreads / 16) + (uint32_t)(tid >> 2)) % nblk);
        sign_tab[tid] = quad_bits(kb * 4u + (uint32_t)(tid & 3), a.r0, a.r1);
    }
    OuterScale os;
    // Largest dequantized magnitude.  In tensor mode the group holding the tensor maximum always gets
    // the scale 448 and its largest element the code 6, so the maximum is 6 * 448 * S_g in closed form;
    // only a floored S_g (maximum below 2688 * 2^-100) needs the reduction over all groups.
    bool reduce_deq = DEQ && OUTER == 1 && a.amax_deq != nullptr;
    if (OUTER == 0) {
        const float amax = block_tensor_amax(a, red);
        os = outer_scale(amax);
        if (bid == 0 && tid == 0) a.gscale[0] = os.S_g;
        if (DEQ) {
            reduce_deq = a.amax_deq != nullptr && os.S_g == 0x1p-100f;
            if (!reduce_deq && a.amax_deq && bid == 0 && tid == 0) a.amax_deq[0] = amax == 0.0f ? 0.0f : 2688.0f * os.S_g;
        }
    }
    __syncthreads();
    float deq = 0.0f;
    // CHECK = false: every chunk of this workgroup exists (all but the last workgroup), no predication
    auto run = [&](auto chk) {
        constexpr bool CHECK = decltype(chk)::value;
#pragma unroll
        for (int it = 0; it < kRowIter; ++it) {
            const int64_t c = c0 + it * kThreads;
            const bool valid = !CHECK || c < nchunks;
            uint4 v = vs[it];
            float x[8];
            uint32_t bm;                                       // group maximum: bf16 pattern, or binary32 pattern with RHT
            if constexpr (!RHT) {
                const uint32_t hm = absmax8_bits(v);
                const uint32_t o1 = dpp<DPP_QUAD_XOR1>(hm);
                bm = hm > o1 ? hm : o1;
                x[0] = bf16_lo(v.x); x[1] = bf16_hi(v.x); x[2] = bf16_lo(v.y); x[3] = bf16_hi(v.y);
                x[4] = bf16_lo(v.z); x[5] = bf16_hi(v.z); x[6] = bf16_lo(v.w); x[7] = bf16_hi(v.w);
            } else {
                // signs: this chunk is run (tid & 3) of eight positions of its sign word
                const uint32_t w = sign_tab[it * (kThreads / 4) + (tid >> 2)];
                const int rot = 4 * (tid & 3);
                v.x ^= __builtin_amdgcn_alignbit(w, w, rot) & 0x80008000u;
                v.y ^= __builtin_amdgcn_alignbit(w, w, rot + 1) & 0x80008000u;
                v.z ^= __builtin_amdgcn_alignbit(w, w, rot + 2) & 0x80008000u;
                v.w ^= __builtin_amdgcn_alignbit(w, w, rot + 3) & 0x80008000u;
                x[0] = bf16_lo(v.x); x[1] = bf16_hi(v.x); x[2] = bf16_lo(v.y); x[3] = bf16_hi(v.y);
                x[4] = bf16_lo(v.z); x[5] = bf16_hi(v.z); x[6] = bf16_lo(v.w); x[7] = bf16_hi(v.w);
#pragma unroll
                for (int h = 1; h < 8; h <<= 1)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (!(i & h)) {
                            const float p = x[i], q = x[i + h];
                            x[i] = p + q;
                            x[i + h] = p - q;
                        }
                // stride 8: the even lane of the pair holds positions 0..7 (sum), the odd lane 8..15 (difference)
                const uint32_t flip = (uint32_t)(tid & 1) << 31;
                uint32_t hm = 0;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float other = u2f(dpp<DPP_QUAD_XOR1>(f2u(x[i])));
                    x[i] = (other + u2f(f2u(x[i]) ^ flip)) * 0.25f;
                    const uint32_t ab = f2u(x[i]) & 0x7FFFFFFFu;
                    hm = hm > ab ? hm : ab;
                }
                const uint32_t o1 = dpp<DPP_QUAD_XOR1>(hm);
                bm = hm > o1 ? hm : o1;
            }
            if (OUTER == 1) {
                uint32_t gm = bm, t;
                t = dpp<DPP_QUAD_XOR2>(gm);       gm = gm > t ? gm : t;
                t = dpp<DPP_ROW_HALF_MIRROR>(gm); gm = gm > t ? gm : t;
                t = dpp<DPP_ROW_MIRROR>(gm);      gm = gm > t ? gm : t;
                os = outer_scale(RHT ? u2f(gm) : u2f(gm << 16));
                if (valid && (tid & 15) == 0) a.gscale[c >> 4] = os.S_g;
            }
            const float amax_b = RHT ? u2f(bm) : u2f(bm << 16);
            const float s = amax_b * os.inv_cg;
            const uint32_t sc = e4m3_round<SUP>(s);
            const float r = os.inv_sg * inv_tab[sc];
            const uint32_t q = quant8<ROUND, SUP>(x, r, (uint32_t)(c * 2), a.k0, a.k1);
            if (valid) a.codes[c] = q;
            // four scale bytes (lanes c, c+2, c+4, c+6) travel to the lane with c % 8 == 0
            const uint32_t s2 = sc | (dpp<DPP_ROW_SHL2>(sc) << 8);
            const uint32_t s4 = s2 | (dpp<DPP_ROW_SHL4>(s2) << 16);
            if (valid && (tid & 7) == 0) {
                if (!CHECK || c + 8 <= nchunks) {
                    reinterpret_cast<uint32_t *>(a.scales)[c >> 3] = s4;
                } else {
                    for (int b = 0; b < 4; ++b)
                        if (c + 2 * b < nchunks) a.scales[(c >> 1) + b] = (uint8_t)(s4 >> (8 * b));
                }
            }
            if (DEQ && reduce_deq) {
                // the group's largest element gets the group's largest code (rounding is monotone)
                const uint32_t mm = e2m1_rtn(amax_b * r) & 7u;
                float val = e2m1_value(mm) * e4m3_value(sc);
                if (OUTER == 1) val = val * os.S_g;
                deq = fmaxf(deq, val);
            }
        }
    };
    if (full) run(std::false_type{});
    else run(std::true_type{});
    if (DEQ && reduce_deq) {
        if (OUTER == 0) deq = deq * os.S_g;
        publish_deq_max(deq, a.amax_deq, red);
    }
}

// ------------------------------------------------------------------------- column-wise ----

constexpr int kTileR = 128;   // source rows per tile = 8 groups of 16
constexpr int kTileC = 64;    // source columns per tile = 32 dwords of bf16 pairs

struct ColArgs {
    const uint4 *src;          // bf16 source
    const uint8_t *src_codes;  // packed source
    const uint8_t *src_scales;
    const float *src_gscale;
    int src_outer;             // packed source: 0 one scale for the tensor, 1 one per row and 128 columns
    int64_t R, C;
    int span;                  // consecutive row tiles (of one column tile) per workgroup
    KArgs k;
    KArgs krow;                // DUAL: the row-wise operand produced from the same read
};

// dword column of the tile, rotated by 4 per 16 rows
__device__ __forceinline__ int tile_pos(int row, int dwcol) { return row * 32 + ((dwcol + 4 * (row >> 4)) & 31); }

// Row-wise AND column-wise operand of one bf16 tensor from a single read of it (Q3 and Q5 of dY).  A workgroup takes
// `span` consecutive 128 x 64 tiles down one column of tiles (blockIdx.x = column tile fastest): the scale set-up is
// paid once and the next tile's loads are in flight while the current one is quantized.  Each tile goes through LDS
// as bf16 pairs (rotated so that the 128-bit row writes and the per-column reads are both conflict free); on the way in,
// while a row passes through registers, it is quantized row-wise (groups along C); after the transpose a lane owns
// two columns x 16 rows = two groups of the column-wise operand.
template <int ROUND, bool SUP>
__global__ __launch_bounds__(kThreads) void quant_dual_kernel(ColArgs a)
{
    __shared__ __attribute__((aligned(16))) uint32_t tile[kTileR * 32];
    __shared__ float inv_tab[128];
    __shared__ float red[4];
    __shared__ float os_sh[4];
    const int tid = threadIdx.x;
    const uint32_t lin0 = blockIdx.x;
    const int64_t R = a.R, C = a.C;
    const uint32_t tiles_r = (uint32_t)((R + kTileR - 1) / kTileR);
    const uint32_t gx = (uint32_t)((C + kTileC - 1) / kTileC);              // column tiles
    // (dealing the tiles to the XCDs in contiguous bands, as the strip kernel does, was measured here: 8 % fewer bytes
    // written, but 65 us against 58.7 on 8192 x 8192)
    const uint32_t lin = lin0;
    // workgroup-uniform: keep them (and everything derived from them) in scalar registers
    const uint32_t by = __builtin_amdgcn_readfirstlane(lin / gx), bx = __builtin_amdgcn_readfirstlane(lin % gx);
    const int64_t C0 = (int64_t)bx * kTileC;
    const uint32_t rt0 = by * (uint32_t)a.span;
    const int ntile = (int)min((uint32_t)a.span, tiles_r - rt0);

    // ---- loads of one tile into registers (nothing here depends on the scale set-up)
    const int64_t ld_row = tid >> 3;
    const int64_t ld_col = C0 + 8 * (tid & 7);
    // element index of the thread's first load: its own part once, the tile's (workgroup-uniform) part per tile
    const int64_t ld_lane = ld_row * C + ld_col;
    struct Fetch { uint4 v[4]; };                                            // 8 elements of rows (tid >> 3) + 32 * pass
    auto fetch = [&](int t, Fetch &f) {
        const int64_t R0 = (int64_t)(rt0 + t) * kTileR;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int64_t r_uni = R0 + pass * 32;                           // uniform
            f.v[pass] = make_uint4(0, 0, 0, 0);
            if (r_uni + ld_row < R && ld_col < C) f.v[pass] = ld_stream(a.src + ((r_uni * C + ld_lane) >> 3));
        }
    };
    Fetch cur;
    fetch(0, cur);

    // ---- set-up, once per workgroup: reciprocal table (waves 0, 1), outer scale (wave 2)
    fill_inv_table(inv_tab);
    const float amax = block_tensor_amax(a.k, red);
    if ((tid >> 6) == 2) {
        const OuterScale o = outer_scale(amax);
        if (tid == 128) {
            os_sh[0] = o.S_g;
            os_sh[1] = o.inv_sg;
            os_sh[2] = o.inv_cg;
            if (lin0 == 0) {
                a.k.gscale[0] = o.S_g;
                a.krow.gscale[0] = o.S_g;
            }
        }
    }
    __syncthreads();
    OuterScale os;
    os.S_g = os_sh[0];
    os.inv_sg = os_sh[1];
    os.inv_cg = os_sh[2];

    // phase-2 ownership: lane = (row group rb, column pair cp): 16 rows down two columns
    const int rb = tid & 7, cp = tid >> 3;
    const int64_t c_first = C0 + 2 * cp;
    const int64_t out_lane = c_first * R + 16 * rb;        // + R0 (+ R for the second column): output element index

    for (int t = 0; t < ntile; ++t) {
        const int64_t R0 = (int64_t)(rt0 + t) * kTileR;
        if (t > 0) __syncthreads();                         // everyone is done reading the previous tile
        // phase 1: tile -> LDS as bf16 pairs, row-major with rotated columns
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int row = pass * 32 + (tid >> 3), q = tid & 7;
            const uint4 v = cur.v[pass];
            *reinterpret_cast<uint4 *>(&tile[tile_pos(row, q * 4)]) = v;
            {
                // row-wise: lanes q, q^1 hold one group of 16 along C
                const int64_t gr = R0 + row;
                const bool valid = gr < R && ld_col < C;
                const uint32_t hm = absmax8_bits(v);
                const uint32_t o1 = dpp<DPP_QUAD_XOR1>(hm);
                const uint32_t bm = hm > o1 ? hm : o1;
                const uint32_t sc = e4m3_round<SUP>(u2f(bm << 16) * os.inv_cg);
                const float r = os.inv_sg * inv_tab[sc];
                const float x[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                                    bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
                const int64_t e0 = (R0 + pass * 32) * C + ld_lane;
                const uint32_t qd = quant8<ROUND, SUP>(x, r, (uint32_t)(e0 >> 2), a.krow.k0, a.krow.k1);
                if (valid) a.krow.codes[e0 >> 3] = qd;
                const uint32_t s2 = sc | (dpp<DPP_ROW_SHL2>(sc) << 8);
                const uint32_t s4 = s2 | (dpp<DPP_ROW_SHL4>(s2) << 16);
                if (valid && q == 0) {
                    if ((C & 63) == 0) {
                        *reinterpret_cast<uint32_t *>(a.krow.scales + (e0 >> 4)) = s4;
                    } else {
                        for (int b = 0; b < 4; ++b)
                            if (ld_col + 16 * b < C) a.krow.scales[(e0 >> 4) + b] = (uint8_t)(s4 >> (8 * b));
                    }
                }
            }
        }
        __syncthreads();
        if (t + 1 < ntile) fetch(t + 1, cur);               // in flight during phase 2

        // phase 2
        uint32_t w[16];
        ushort2_t m2 = {0, 0};                                              // max |.| of the two columns, as bf16 bits
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            w[i] = tile[tile_pos(16 * rb + i, cp)];
            m2 = __builtin_elementwise_max(m2, as_us2(w[i] & 0x7FFF7FFFu));
        }
        if (R0 + 16 * rb >= R) continue;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if (c_first + j >= C) break;
            float x0[8], x1[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                x0[i] = j == 0 ? bf16_lo(w[i]) : bf16_hi(w[i]);
                x1[i] = j == 0 ? bf16_lo(w[8 + i]) : bf16_hi(w[8 + i]);
            }
            float m = u2f((uint32_t)(j == 0 ? m2.x : m2.y) << 16);
            const float s = m * os.inv_cg;
            const uint32_t sc = e4m3_round<SUP>(s);
            const float r = os.inv_sg * inv_tab[sc];
            const int64_t e = out_lane + R0 + (j ? R : 0);
            const uint32_t quad0 = (uint32_t)(e >> 2);
            uint2 q;
            q.x = quant8<ROUND, SUP>(x0, r, quad0, a.k.k0, a.k.k1);
            q.y = quant8<ROUND, SUP>(x1, r, quad0 + 2, a.k.k0, a.k.k1);
            *reinterpret_cast<uint2 *>(reinterpret_cast<uint8_t *>(a.k.codes) + (e >> 1)) = q;
            a.k.scales[e >> 4] = (uint8_t)sc;
        }
    }
}


// ------------------------------------------------------------- column-wise, one strip per wave ----
//
// Groups of 16 run down the columns of the source [R x C]; the output is the transposed operand [C x R].  A wave
// owns a strip of 128 source columns x 128 source rows (8 slabs of 16 rows): lane l holds columns 2 l, 2 l + 1 of a
// slab as 16 registers (one dword of two bf16 per row - a wave load is 256 contiguous bytes of a row; or one byte of
// two codes per row for a packed source), i.e. two complete groups, with no exchange between lanes and no barrier
// while it quantizes.  The four waves of a workgroup take four strips below each other, so for each of the 128
// output rows the workgroup produces 256 contiguous bytes of codes and 32 of scales; these are gathered in LDS and
// written after the workgroup's only barrier, whole runs per store instruction (measured on this chip: 16-byte
// pieces scattered over rows 2.3 TB/s, 64-byte runs 4.2, 256-byte runs 4.6; 8-byte scale pieces cost as much as all
// the codes).  With a 1 x 128 outer block (OUTER = 1) a strip's 128 rows are exactly one outer block of each of its
// output rows: a first pass over the strip takes the column maxima, the second pass (the same addresses again, now
// from cache) quantizes.
constexpr int kStripC = 128, kStripR = 128, kSlabs = kStripR / 16;

// RHT (with OUTER = 1): a lane's 16 values of a column are one block of the random Hadamard transform (Sec. 4.1), all
// in its own registers; the signs depend on the source row only, so they are wave-uniform masks.
template <int ROUND, bool SUP, bool PACKED, int OUTER, bool RHT = false>
__global__ __launch_bounds__(kThreads) void quant_colw_kernel(ColArgs a0, ColArgs a1, unsigned first_second)
{
    static_assert(!RHT || OUTER == 1, "the transform is provided with 1 x 128 outer blocks");
    __shared__ float inv_tab[128];
    __shared__ float red[4];
    const int tid = threadIdx.x, lane = tid & 63;
    const bool second = blockIdx.x >= first_second;
    const ColArgs a = second ? a1 : a0;
    const uint32_t wg0 = second ? blockIdx.x - first_second : blockIdx.x;
    // Workgroup ids are dealt round-robin over the 8 XCDs.  Each XCD gets a contiguous run of this job's strips (column
    // index fastest, so whole bands of strip rows): its strips then cover every column offset - all of the cache's
    // channels, where a strided walk down one column offset would keep hitting the same few - and neighbouring strips,
    // which share cache lines of a packed source, meet in one L2.  Measured on 8192 x 8192 bf16: 6.1 TB/s against 4.0.
    uint32_t wg = wg0;
    {
        const uint32_t nwg = second ? gridDim.x - first_second : (first_second < gridDim.x ? first_second : gridDim.x);
        const uint32_t per_xcd = nwg / 8;
        if (wg < per_xcd * 8) wg = (wg & 7) * per_xcd + (wg >> 3);
    }
    fill_inv_table(inv_tab);
    OuterScale os[2];
    if (OUTER == 0) {
        os[0] = os[1] = outer_scale(block_tensor_amax(a.k, red));
        if (wg0 == 0 && tid == 0) a.k.gscale[0] = os[0].S_g;
    }
    __syncthreads();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t R = a.R, C = a.C;
    constexpr int kWaves = kThreads / 64;
    const uint32_t tiles_c = (uint32_t)((C + kStripC - 1) / kStripC), tiles_r = (uint32_t)((R + kStripR - 1) / kStripR);
    // wave-uniform: keep them (and every address derived from them) in scalar registers
    const uint32_t tc = __builtin_amdgcn_readfirstlane(wg % tiles_c), trg = __builtin_amdgcn_readfirstlane(wg / tiles_c);
    const uint32_t tr = trg * kWaves + wave;
    const bool have = tr < tiles_r;                                // this wave has a strip (all of them reach the barrier)
    // strips of this workgroup that are whole and whose output runs are 16-byte aligned: these go out through LDS
    const int nwide = (R & 127) == 0 ? (int)min((uint32_t)kWaves, tiles_r - trg * kWaves) : 0;
    const int64_t R0 = (int64_t)tr * kStripR, c0 = (int64_t)tc * kStripC + 2 * lane;
    const bool colok = c0 < C;                                     // C is even: both columns or none
    const int nslab = have ? (int)min((int64_t)kSlabs, (R - R0) >> 4) : 0;    // R is a multiple of 16

    // One slab = 16 rows x the lane's two columns.  Every address is a wave-uniform row pointer plus a 32-bit lane
    // index, so the loads need no per-lane address arithmetic and no predication: lanes past the last column read
    // column pair 0 of the strip (valid memory) and are never stored.  fetch() only issues the loads (raw words stay
    // in registers); decode() turns them into binary32, x0[i], x1[i] = source(R0 + 16 s + i, c0), (.., c0 + 1).
    // The next slab is fetched before the current one is decoded, so a wave always has a slab in flight.
    const uint32_t ln = colok ? (uint32_t)lane : 0u;
    const int64_t strip0 = (int64_t)tc * kStripC;                  // first column of the strip (uniform)
    const float src_sg_tensor = (PACKED && a.src_outer == 0) ? a.src_gscale[0] : 1.0f;
    struct Raw {
        uint32_t w[16];                                            // bf16 pairs, or bytes of two codes
        uint32_t sb[PACKED ? 16 : 1];                              // packed: scale bytes
    };
    // packed source: the outer scale of each of the strip's 128 rows, in the wave's own corner of LDS (1 x 128 outer
    // blocks: the strip lies inside one block column, so a row has one; per-tensor scale: 128 copies of it, so that the
    // decode is the same code for both)
    __shared__ float row_sg_all[PACKED ? kThreads / 64 : 1][PACKED ? kStripR : 1];
    float *row_sg = row_sg_all[PACKED ? wave : 0];
    if (PACKED && have) {
        const bool src_blocks = a.src_outer != 0;
        const int64_t nbc = C >> 7;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int64_t row = R0 + lane + 64 * h;
            row_sg[lane + 64 * h] = !src_blocks ? src_sg_tensor : row < R ? a.src_gscale[row * nbc + tc] : 0.0f;
        }
        // same wave writes and reads: the compiler's wait on the LDS counter orders them
    }
    auto fetch = [&](auto stream, int s, Raw &r) {
        constexpr bool STREAM = decltype(stream)::value;          // last use of these bytes: they need not stay cached
        const int64_t e0 = (R0 + 16 * s) * C + strip0;             // uniform
        if constexpr (!PACKED) {
            const uint32_t *p = reinterpret_cast<const uint32_t *>(a.src) + (e0 >> 1);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t *rowp = p + i * (C >> 1);           // uniform
                r.w[i] = STREAM ? __builtin_nontemporal_load(rowp + ln) : rowp[ln];
            }
        } else {
            const uint8_t *pc = a.src_codes + (e0 >> 1);
            const uint8_t *ps = a.src_scales + (e0 >> 4);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                r.w[i] = (pc + i * (C >> 1))[ln];
                r.sb[i] = (ps + i * (C >> 4))[ln >> 3];
            }
        }
    };
    // returns the two column maxima of the slab
    auto decode = [&](const Raw &r, int s, float (&x0)[16], float (&x1)[16], float &m0, float &m1) {
        // RHT: the slab's 16 source rows are positions 16 (s & 1) .. + 15 of sign word (R0 + 16 s) / 32 (R0 is a multiple
        // of 128); the word is the same for the whole wave
        uint32_t sw = 0;
        if (RHT) sw = __builtin_amdgcn_readfirstlane(quad_bits((uint32_t)((R0 + 16 * s) >> 5), a.k.r0, a.k.r1));
        auto flips = [&](int i) { return ((sw >> rht_sign_bit(16 * (s & 1) + i)) & 1u) != 0; };   // uniform
        if constexpr (!PACKED) {
            ushort2_t m2 = {0, 0};
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                uint32_t w = r.w[i];
                if (RHT) w ^= flips(i) ? 0x80008000u : 0u;
                m2 = __builtin_elementwise_max(m2, as_us2(w & 0x7FFF7FFFu));
                x0[i] = bf16_lo(w);
                x1[i] = bf16_hi(w);
            }
            m0 = u2f((uint32_t)m2.x << 16);
            m1 = u2f((uint32_t)m2.y << 16);
        } else {
            m0 = m1 = 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float sg = row_sg[16 * s + i];
                uint32_t cb = r.w[i];
                if (RHT) cb ^= flips(i) ? 0x88u : 0u;               // the sign bits of the two codes
                // P * S_block, exact: the conversion supplies P * 2^120, the scale byte shifted into place is S_block * 2^-120
                const float2_t pv = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(cb, 0x1p120f, 0) * u2f(r.sb[i] << 20);
                x0[i] = pv.x * sg;                                  // the binary32 dequantized value: one rounding
                x1[i] = pv.y * sg;
                m0 = fmaxf(m0, fabsf(x0[i]));
                m1 = fmaxf(m1, fabsf(x1[i]));
            }
        }
        if (RHT) {
            fwht16(x0);
            fwht16(x1);
            m0 = m1 = 0.0f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                m0 = fmaxf(m0, fabsf(x0[i]));
                m1 = fmaxf(m1, fabsf(x1[i]));
            }
        }
    };

    Raw raw[2];                                                    // slab s lives in raw[s % 2] (s is a constant after unrolling)
    if (OUTER == 1 && have) {
        // first pass: the maximum of each column over the strip's 128 rows = one outer block of the output row
        float cm0 = 0.0f, cm1 = 0.0f;
        fetch(std::false_type{}, 0, raw[0]);
#pragma unroll
        for (int s = 0; s < kSlabs; ++s) {
            if (s >= nslab) break;
            const Raw &cur = raw[s & 1];
            if (s + 1 < nslab) fetch(std::false_type{}, s + 1, raw[(s + 1) & 1]);
            if constexpr (!PACKED && !RHT) {
                ushort2_t m2 = {0, 0};
#pragma unroll
                for (int i = 0; i < 16; ++i) m2 = __builtin_elementwise_max(m2, as_us2(cur.w[i] & 0x7FFF7FFFu));
                cm0 = fmaxf(cm0, u2f((uint32_t)m2.x << 16));
                cm1 = fmaxf(cm1, u2f((uint32_t)m2.y << 16));
            } else {
                float x0[16], x1[16], m0, m1;
                decode(cur, s, x0, x1, m0, m1);
                cm0 = fmaxf(cm0, m0);
                cm1 = fmaxf(cm1, m1);
            }
        }
        os[0] = outer_scale(cm0);
        os[1] = outer_scale(cm1);
        if (colok) {
            const int64_t nb = R >> 7;
            a.k.gscale[c0 * nb + tr] = os[0].S_g;
            a.k.gscale[(c0 + 1) * nb + tr] = os[1].S_g;
        }
    }

    // Codes and scale bytes of the workgroup's whole strips are gathered in LDS: [output row][wave][64 + 8 bytes].
    // Code row pitch 264 bytes (256 + 8) spreads the lanes' 8-byte writes over the banks.
    constexpr int kPitch = kWaves * 64 + 8, kScPitch = kWaves * 8;
    __shared__ __attribute__((aligned(16))) uint8_t stage[kStripC * kPitch];
    __shared__ __attribute__((aligned(16))) uint8_t sc_stage[kStripC * kScPitch];
    uint32_t scb[2][2] = {{0, 0}, {0, 0}};                          // scale bytes of slabs 0..3 and 4..7, per column
    const bool wide = (int)wave < nwide;
    if (have) fetch(std::true_type{}, 0, raw[0]);
#pragma unroll
    for (int s = 0; s < kSlabs; ++s) {
        if (s >= nslab) break;
        const Raw &cur = raw[s & 1];
        if (s + 1 < nslab) fetch(std::true_type{}, s + 1, raw[(s + 1) & 1]);
        float x0[16], x1[16], mx[2];
        decode(cur, s, x0, x1, mx[0], mx[1]);
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const float (&x)[16] = j == 0 ? x0 : x1;
            const uint32_t sc = e4m3_round<SUP>(mx[j] * os[j].inv_cg);
            const float r = os[j].inv_sg * inv_tab[sc];
            const int64_t e = (c0 + j) * R + R0 + 16 * s;           // index in the output's [C x R] view
            const uint32_t quad0 = (uint32_t)(e >> 2);
            const float xa[8] = {x[0], x[1], x[2], x[3], x[4], x[5], x[6], x[7]};
            const float xb[8] = {x[8], x[9], x[10], x[11], x[12], x[13], x[14], x[15]};
            uint2 q;
            q.x = quant8<ROUND, SUP>(xa, r, quad0, a.k.k0, a.k.k1);
            q.y = quant8<ROUND, SUP>(xb, r, quad0 + 2, a.k.k0, a.k.k1);
            scb[j][s >> 2] |= sc << (8 * (s & 3));
            if (wide) {
                *reinterpret_cast<uint2 *>(stage + (2 * lane + j) * kPitch + wave * 64 + 8 * s) = q;
            } else if (colok) {
                *reinterpret_cast<uint2 *>(reinterpret_cast<uint8_t *>(a.k.codes) + (e >> 1)) = q;
                a.k.scales[e >> 4] = (uint8_t)sc;
            }
        }
    }
    if (nwide == 0) return;                                         // uniform over the workgroup
    if (wide) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
            *reinterpret_cast<uint2 *>(sc_stage + (2 * lane + j) * kScPitch + wave * 8) = make_uint2(scb[j][0], scb[j][1]);
    }
    __syncthreads();
    {
        // codes: 16 lanes x 16 bytes cover one output row's 256-byte run; 16 rows per pass
        const int64_t Rg = (int64_t)trg * kWaves * kStripR;        // first source row of the workgroup
        const int piece = tid & 15;
        uint8_t *out_codes = reinterpret_cast<uint8_t *>(a.k.codes);
        if (piece < 4 * nwide) {
#pragma unroll
            for (int it = 0; it < kStripC / 16; ++it) {
                const int row = it * 16 + (tid >> 4);
                const uint2 lo = *reinterpret_cast<const uint2 *>(stage + row * kPitch + piece * 16);
                const uint2 hi = *reinterpret_cast<const uint2 *>(stage + row * kPitch + piece * 16 + 8);
                const int64_t c = strip0 + row;
                if (c < C) *reinterpret_cast<uint4 *>(out_codes + ((c * R + Rg) >> 1) + piece * 16) = make_uint4(lo.x, lo.y, hi.x, hi.y);
            }
        }
        // scales: 4 lanes x 8 bytes cover one output row's 32-byte run; 64 rows per pass
        const int sp = tid & 3;
        if (sp < nwide) {
#pragma unroll
            for (int it = 0; it < 2; ++it) {
                const int row = it * 64 + (tid >> 2);
                const uint2 v = *reinterpret_cast<const uint2 *>(sc_stage + row * kScPitch + sp * 8);
                const int64_t c = strip0 + row;
                if (c < C) *reinterpret_cast<uint2 *>(a.k.scales + ((c * R + Rg) >> 4) + sp * 8) = v;
            }
        }
    }
}

inline unsigned colw_grid(const ColArgs &a)
{
    const int64_t tiles_c = (a.C + kStripC - 1) / kStripC, tiles_r = (a.R + kStripR - 1) / kStripR;
    return (unsigned)(tiles_c * ((tiles_r + kThreads / 64 - 1) / (kThreads / 64)));
}

// number of workgroups of a column job (and its span): a workgroup takes several tiles only when there are more than
// 8192 tiles (measured: with fewer workgroups than that the chip is not kept busy)
inline unsigned col_grid(ColArgs &a)
{
    const int64_t tiles_c = (a.C + kTileC - 1) / kTileC, tiles_r = (a.R + kTileR - 1) / kTileR;
    int span = 4;
    while (span > 1 && tiles_c * ((tiles_r + span - 1) / span) < 8192) span >>= 1;
    a.span = span;
    return (unsigned)(tiles_c * ((tiles_r + span - 1) / span));
}

KArgs make_kargs(const QuantParams &p, const QuantOut &o)
{
    KArgs k;
    k.codes = reinterpret_cast<uint32_t *>(o.codes);
    k.scales = o.scales;
    k.gscale = o.gscale;
    k.amax_deq = o.amax_deq;
    k.amax_scalar = p.amax_scalar;
    k.amax_partials = p.amax_partials;
    k.npart = p.npart;
    k.k0 = p.k0;
    k.k1 = p.k1;
    k.r0 = p.r0;
    k.r1 = p.r1;
    return k;
}

template <int ROUND, bool SUP, int OUTER>
void launch_row_t(const RowJob &j0, const RowJob &j1, bool deq, bool rht, hipStream_t st)
{
    const int64_t per_wg = (int64_t)kThreads * kRowIter;
    const unsigned g0 = (unsigned)((j0.nchunks + per_wg - 1) / per_wg), g1 = (unsigned)((j1.nchunks + per_wg - 1) / per_wg);
    const unsigned first_second = g1 ? g0 : 0xFFFFFFFFu;
    if constexpr (OUTER == 1) {
        if (rht) {
            hipLaunchKernelGGL((quant_row_kernel<ROUND, SUP, 1, false, true>), dim3(g0 + g1), dim3(kThreads), 0, st, j0, j1,
                               first_second);
            return;
        }
    }
    if (deq)
        hipLaunchKernelGGL((quant_row_kernel<ROUND, SUP, OUTER, true>), dim3(g0 + g1), dim3(kThreads), 0, st, j0, j1,
                           first_second);
    else
        hipLaunchKernelGGL((quant_row_kernel<ROUND, SUP, OUTER, false>), dim3(g0 + g1), dim3(kThreads), 0, st, j0, j1,
                           first_second);
}

template <bool PACKED, int OUTER, bool RHT>
void launch_colw_t(const ColArgs &a0, const ColArgs &a1, bool pair, int rounding, int scale_up, hipStream_t st)
{
    const unsigned g0 = colw_grid(a0), g1 = pair ? colw_grid(a1) : 0;
    const unsigned first_second = pair ? g0 : 0xFFFFFFFFu;
    const dim3 grid(g0 + g1);
    if (rounding == 0) {
        if (scale_up) hipLaunchKernelGGL((quant_colw_kernel<0, true, PACKED, OUTER, RHT>), grid, dim3(kThreads), 0, st, a0, a1, first_second);
        else          hipLaunchKernelGGL((quant_colw_kernel<0, false, PACKED, OUTER, RHT>), grid, dim3(kThreads), 0, st, a0, a1, first_second);
    } else {
        if (scale_up) hipLaunchKernelGGL((quant_colw_kernel<1, true, PACKED, OUTER, RHT>), grid, dim3(kThreads), 0, st, a0, a1, first_second);
        else          hipLaunchKernelGGL((quant_colw_kernel<1, false, PACKED, OUTER, RHT>), grid, dim3(kThreads), 0, st, a0, a1, first_second);
    }
}

template <bool PACKED>
void launch_colw(const ColArgs &a0, const ColArgs &a1, bool pair, const QuantParams &p, hipStream_t st)
{
    if (p.outer == 0) launch_colw_t<PACKED, 0, false>(a0, a1, pair, p.rounding, p.scale_up, st);
    else if (!p.rht) launch_colw_t<PACKED, 1, false>(a0, a1, pair, p.rounding, p.scale_up, st);
    else launch_colw_t<PACKED, 1, true>(a0, a1, pair, p.rounding, p.scale_up, st);
}

}  // namespace

static int amax_grid(int64_t nchunks)
{
    const int64_t want = (nchunks + (int64_t)kThreads * 8 - 1) / ((int64_t)kThreads * 8);
    return (int)(want < 1 ? 1 : (want > kMaxAmaxPartials ? kMaxAmaxPartials : want));
}

int launch_amax_partials(const void *src, int64_t n, float *partials, float *zero_me, hipStream_t st)
{
    AmaxJob j0{reinterpret_cast<const uint4 *>(src), n / 8, partials, zero_me, (unsigned)amax_grid(n / 8)};
    AmaxJob j1{};
    hipLaunchKernelGGL(amax_partials_kernel, dim3(j0.nblocks), dim3(kThreads), 0, st, j0, j1);
    return (int)j0.nblocks;
}

void launch_amax_partials_pair(const void *src0, int64_t n0, float *partials0, float *zero0, int *npart0,
                               const void *src1, int64_t n1, float *partials1, float *zero1, int *npart1,
                               hipStream_t st)
{
    AmaxJob j0{reinterpret_cast<const uint4 *>(src0), n0 / 8, partials0, zero0, (unsigned)amax_grid(n0 / 8)};
    AmaxJob j1{reinterpret_cast<const uint4 *>(src1), n1 / 8, partials1, zero1, (unsigned)amax_grid(n1 / 8)};
    hipLaunchKernelGGL(amax_partials_kernel, dim3(j0.nblocks + j1.nblocks), dim3(kThreads), 0, st, j0, j1);
    *npart0 = (int)j0.nblocks;
    *npart1 = (int)j1.nblocks;
}

void launch_amax_final(const float *partials, int npart, float *out, hipStream_t st)
{
    hipLaunchKernelGGL(amax_final_kernel, dim3(1), dim3(kThreads), 0, st, partials, npart, out);
}

void launch_zero_scalar(float *p, hipStream_t st)
{
    hipLaunchKernelGGL(zero_scalar_kernel, dim3(1), dim3(1), 0, st, p);
}

static void launch_row_sel(const RowJob &j0, const RowJob &j1, const QuantParams &p, bool deq, hipStream_t st)
{
    const int sel = (p.rounding << 2) | (p.scale_up << 1) | p.outer;
    const bool rht = p.rht != 0;
    switch (sel) {
        case 0: launch_row_t<0, false, 0>(j0, j1, deq, rht, st); break;
        case 1: launch_row_t<0, false, 1>(j0, j1, deq, rht, st); break;
        case 2: launch_row_t<0, true, 0>(j0, j1, deq, rht, st); break;
        case 3: launch_row_t<0, true, 1>(j0, j1, deq, rht, st); break;
        case 4: launch_row_t<1, false, 0>(j0, j1, false, rht, st); break;
        case 5: launch_row_t<1, false, 1>(j0, j1, false, rht, st); break;
        case 6: launch_row_t<1, true, 0>(j0, j1, false, rht, st); break;
        default: launch_row_t<1, true, 1>(j0, j1, false, rht, st); break;
    }
}

hipError_t launch_quant_row_bf16(const void *src, int64_t rows, int64_t K, const QuantParams &p, const QuantOut &o,
                                 hipStream_t st)
{
    const int64_t nchunks = rows * K / 8;
    if (nchunks == 0) return hipSuccess;
    RowJob j0{reinterpret_cast<const uint4 *>(src), nchunks, make_kargs(p, o), (uint32_t)(K / 128)}, j1{};
    launch_row_sel(j0, j1, p, o.amax_deq != nullptr && p.rounding == 0 && !p.rht, st);
    return hipGetLastError();
}

hipError_t launch_quant_row_bf16_pair(const void *src0, int64_t rows0, int64_t K0, const QuantParams &p0,
                                      const QuantOut &o0, const void *src1, int64_t rows1, int64_t K1,
                                      const QuantParams &p1, const QuantOut &o1, hipStream_t st)
{
    if (rows0 * K0 == 0) return launch_quant_row_bf16(src1, rows1, K1, p1, o1, st);
    if (rows1 * K1 == 0) return launch_quant_row_bf16(src0, rows0, K0, p0, o0, st);
    RowJob j0{reinterpret_cast<const uint4 *>(src0), rows0 * K0 / 8, make_kargs(p0, o0), (uint32_t)(K0 / 128)};
    RowJob j1{reinterpret_cast<const uint4 *>(src1), rows1 * K1 / 8, make_kargs(p1, o1), (uint32_t)(K1 / 128)};
    launch_row_sel(j0, j1, p0, (o0.amax_deq != nullptr || o1.amax_deq != nullptr) && p0.rounding == 0, st);
    return hipGetLastError();
}

hipError_t launch_quant_col_bf16(const void *src, int64_t R, int64_t C, const QuantParams &p, const QuantOut &o,
                                 hipStream_t st)
{
    if (R == 0 || C == 0) return hipSuccess;
    ColArgs a{};
    a.src = reinterpret_cast<const uint4 *>(src);
    a.R = R;
    a.C = C;
    a.k = make_kargs(p, o);
    ColArgs none{};
    launch_colw<false>(a, none, false, p, st);
    return hipGetLastError();
}

hipError_t launch_quant_dual_bf16(const void *src, int64_t R, int64_t C, const QuantParams &prow, const QuantOut &orow,
                                  const QuantParams &pcol, const QuantOut &ocol, hipStream_t st)
{
    if (R == 0 || C == 0) return hipSuccess;
    ColArgs a{};
    a.src = reinterpret_cast<const uint4 *>(src);
    a.R = R;
    a.C = C;
    a.k = make_kargs(pcol, ocol);
    a.krow = make_kargs(prow, orow);
    const dim3 grid(col_grid(a));
    const int sel = (pcol.rounding << 1) | pcol.scale_up;
    switch (sel) {
        case 0: hipLaunchKernelGGL((quant_dual_kernel<0, false>), grid, dim3(kThreads), 0, st, a); break;
        case 1: hipLaunchKernelGGL((quant_dual_kernel<0, true>), grid, dim3(kThreads), 0, st, a); break;
        case 2: hipLaunchKernelGGL((quant_dual_kernel<1, false>), grid, dim3(kThreads), 0, st, a); break;
        default: hipLaunchKernelGGL((quant_dual_kernel<1, true>), grid, dim3(kThreads), 0, st, a); break;
    }
    return hipGetLastError();
}

static ColArgs packed_args(const PackedSrc &src, int64_t R, int64_t C, const QuantParams &p, const QuantOut &o)
{
    ColArgs a{};
    a.src_codes = src.codes;
    a.src_scales = src.scales;
    a.src_gscale = src.gscale;
    a.src_outer = src.outer;
    a.R = R;
    a.C = C;
    a.k = make_kargs(p, o);
    return a;
}

hipError_t launch_requant_col(const PackedSrc &src, int64_t R, int64_t C, const QuantParams &p, const QuantOut &o,
                              hipStream_t st)
{
    if (R == 0 || C == 0) return hipSuccess;
    ColArgs a = packed_args(src, R, C, p, o), none{};
    launch_colw<true>(a, none, false, p, st);
    return hipGetLastError();
}

hipError_t launch_requant_col_pair(const PackedSrc &src0, int64_t R0, int64_t C0, const QuantParams &p0,
                                   const QuantOut &o0, const PackedSrc &src1, int64_t R1, int64_t C1,
                                   const QuantParams &p1, const QuantOut &o1, hipStream_t st)
{
    if (R0 == 0 || C0 == 0) return launch_requant_col(src1, R1, C1, p1, o1, st);
    if (R1 == 0 || C1 == 0) return launch_requant_col(src0, R0, C0, p0, o0, st);
    ColArgs a0 = packed_args(src0, R0, C0, p0, o0), a1 = packed_args(src1, R1, C1, p1, o1);
    launch_colw<true>(a0, a1, true, p0, st);
    return hipGetLastError();
}

}  // namespace tj
