// NVFP4 double-block quantizer kernels for gfx950 (TetraJet-v2 Sec. 2.1-2.2, the six
// quantizers of Sec. 2.3).  All of them are bandwidth-bound streaming kernels:
//   amax_partials   per-tensor max|x| of a bf16 array (TENSOR outer mode only)
//   quant_row       groups of 16 along the contiguous axis; 8 elements (one 128-bit load) per
//                   lane, two lanes per group, group maximum exchanged by DPP
//   quant_col       groups of 16 down the columns: a 128 x 64 tile goes through LDS (rotated so
//                   both the 128-bit row writes and the per-column reads are conflict free), each
//                   lane then owns two columns x 16 rows; the output is the transposed operand
//   requant_col     same, the source being a packed NVFP4 tensor (Q4 / Q6)
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

// reciprocals of all E4M3 values (entry 0 = 0, so a zero scale gives all-zero codes)
__device__ __forceinline__ void fill_inv_table(float *tab)
{
    if (threadIdx.x < 128) {
        float v = e4m3_value(threadIdx.x);
        tab[threadIdx.x] = (threadIdx.x == 0 || threadIdx.x == 127) ? 0.0f : 1.0f / v;
    }
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
};

// first_second: first workgroup of the second job (0xFFFFFFFF when the launch has one job)
template <int ROUND, bool SUP, int OUTER, bool DEQ>
__global__ __launch_bounds__(kThreads) void quant_row_kernel(RowJob j0, RowJob j1, unsigned first_second)
{
    __shared__ float inv_tab[128];
    __shared__ float red[4];
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
            const uint4 v = vs[it];
            const uint32_t hm = absmax8_bits(v);
            const uint32_t o1 = dpp<DPP_QUAD_XOR1>(hm);
            const uint32_t bm = hm > o1 ? hm : o1;
            if (OUTER == 1) {
                uint32_t gm = bm, t;
                t = dpp<DPP_QUAD_XOR2>(gm);       gm = gm > t ? gm : t;
                t = dpp<DPP_ROW_HALF_MIRROR>(gm); gm = gm > t ? gm : t;
                t = dpp<DPP_ROW_MIRROR>(gm);      gm = gm > t ? gm : t;
                os = outer_scale(u2f(gm << 16));
                if (valid && (tid & 15) == 0) a.gscale[c >> 4] = os.S_g;
            }
            const float amax_b = u2f(bm << 16);
            const float s = amax_b * os.inv_cg;
            const uint32_t sc = e4m3_round<SUP>(s);
            const float r = os.inv_sg * inv_tab[sc];
            const float x[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                                bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
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
    int64_t R, C;
    int span;                  // consecutive row tiles (of one column tile) per workgroup
    KArgs k;
    KArgs krow;                // DUAL: the row-wise operand produced from the same read
};

// dword column of the tile, rotated by 4 per 16 rows
__device__ __forceinline__ int tile_pos(int row, int dwcol) { return row * 32 + ((dwcol + 4 * (row >> 4)) & 31); }

// 16 packed codes of one source group times its scale, as 8 dwords of bf16 pairs (exact: 6 significant bits).
// The hardware conversion turns a byte into two binary32 values (signed zeros included); the product with the scale
// is exact, and its upper half is the bf16 value.
__device__ __forceinline__ void decode_group_bf16(uint2 codes, uint32_t sc, uint32_t (&out)[8])
{
    const float sb = e4m3_value(sc);
    const float2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes.x, 1.0f, 0) * sb;
    const float2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes.x, 1.0f, 1) * sb;
    const float2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes.x, 1.0f, 2) * sb;
    const float2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes.x, 1.0f, 3) * sb;
    const float2_t p4 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes.y, 1.0f, 0) * sb;
    const float2_t p5 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes.y, 1.0f, 1) * sb;
    const float2_t p6 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes.y, 1.0f, 2) * sb;
    const float2_t p7 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes.y, 1.0f, 3) * sb;
    const float2_t p[8] = {p0, p1, p2, p3, p4, p5, p6, p7};
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = __builtin_amdgcn_perm(f2u(p[i].y), f2u(p[i].x), 0x07060302u);
}

// what one thread brings in for one tile
template <bool PACKED>
struct ColFetch {
    uint4 v[4];                // bf16: 8 elements of rows (tid >> 3) + 32 * pass
};
template <>
struct ColFetch<true> {
    uint2 cw[2];               // packed: two groups of 16 codes of row tid >> 1 ...
    uint32_t sc[2];            // ... and their scale bytes
};

// A workgroup takes `span` consecutive row tiles of one column tile (blockIdx.x = column tile, blockIdx.y = run of
// row tiles): the scale set-up is paid once, the next tile's loads are in flight while the current one is quantized,
// and the halves of an output line (128 source rows give 64 bytes of codes per column) are written close in time.
// DUAL (bf16 source only): the tile's rows are also quantized row-wise (groups along C) while they pass through
// registers on the way into LDS, so one read of the source yields both backward operands of dY (Q3 and Q5).
template <int ROUND, bool SUP, bool PACKED, bool DUAL = false>
__global__ __launch_bounds__(kThreads) void quant_col_kernel(ColArgs a0, ColArgs a1, unsigned first_second)
{
    __shared__ __attribute__((aligned(16))) uint32_t tile[kTileR * 32];
    __shared__ float inv_tab[128];
    __shared__ float red[4];
    __shared__ float os_sh[4];
    const int tid = threadIdx.x;
    // one launch can serve two tensors: workgroups from first_second on take the second job
    const bool second = blockIdx.x >= first_second;
    const ColArgs a = second ? a1 : a0;
    const uint32_t lin0 = second ? blockIdx.x - first_second : blockIdx.x;
    const int64_t R = a.R, C = a.C;
    const uint32_t tiles_r = (uint32_t)((R + kTileR - 1) / kTileR);
    const uint32_t gx = (uint32_t)((C + kTileC - 1) / kTileC);              // column tiles
    const uint32_t gy = (tiles_r + (uint32_t)a.span - 1) / (uint32_t)a.span; // runs of row tiles
    uint32_t lin = lin0;
    if (PACKED) {
        // Workgroup ids are dealt round-robin over the 8 XCDs.  A packed source has only 32 bytes of codes per row and
        // tile, so there each XCD gets a contiguous run of workgroups (column tile fastest): neighbouring column
        // tiles, which share the source's cache lines, then meet in one L2.
        const uint32_t per_xcd = gx * gy / 8;
        if (lin < per_xcd * 8) lin = (lin & 7) * per_xcd + (lin >> 3);
    }
    // workgroup-uniform: keep them (and everything derived from them) in scalar registers
    const uint32_t by = __builtin_amdgcn_readfirstlane(lin / gx), bx = __builtin_amdgcn_readfirstlane(lin % gx);
    const int64_t C0 = (int64_t)bx * kTileC;
    const uint32_t rt0 = by * (uint32_t)a.span;
    const int ntile = (int)min((uint32_t)a.span, tiles_r - rt0);

    // ---- loads of one tile into registers (nothing here depends on the scale set-up)
    const int64_t ld_row = PACKED ? (tid >> 1) : (tid >> 3);
    const int64_t ld_col = C0 + (PACKED ? 32 * (tid & 1) : 8 * (tid & 7));
    // element index of the thread's first load: its own part once, the tile's (workgroup-uniform) part per tile
    const int64_t ld_lane = ld_row * C + ld_col;
    auto fetch = [&](int t, ColFetch<PACKED> &f) {
        const int64_t R0 = (int64_t)(rt0 + t) * kTileR;
        if constexpr (!PACKED) {
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int64_t r_uni = R0 + pass * 32;                       // uniform
                f.v[pass] = make_uint4(0, 0, 0, 0);
                if (r_uni + ld_row < R && ld_col < C) f.v[pass] = ld_stream(a.src + ((r_uni * C + ld_lane) >> 3));
            }
        } else {
            const int64_t e_uni = R0 * C;                                   // uniform
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int64_t gc = ld_col + 16 * b;
                f.cw[b] = make_uint2(0, 0);
                f.sc[b] = 0;
                if (R0 + ld_row < R && gc < C) {
                    const int64_t e = e_uni + ld_lane + 16 * b;
                    f.cw[b] = *reinterpret_cast<const uint2 *>(a.src_codes + (e >> 1));
                    f.sc[b] = a.src_scales[e >> 4];
                }
            }
        }
    };
    ColFetch<PACKED> cur;
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
                if (DUAL) a.krow.gscale[0] = o.S_g;
            }
        }
    }
    const float src_sg = PACKED ? a.src_gscale[0] : 1.0f;
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
        if constexpr (!PACKED) {
#pragma unroll
            for (int pass = 0; pass < 4; ++pass) {
                const int row = pass * 32 + (tid >> 3), q = tid & 7;
                const uint4 v = cur.v[pass];
                *reinterpret_cast<uint4 *>(&tile[tile_pos(row, q * 4)]) = v;
                if (DUAL) {
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
        } else {
            const int row = tid >> 1, half = tid & 1;
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                uint32_t d[8];
                decode_group_bf16(cur.cw[b], cur.sc[b], d);
                const int dw = 16 * half + 8 * b;
                *reinterpret_cast<uint4 *>(&tile[tile_pos(row, dw)]) = make_uint4(d[0], d[1], d[2], d[3]);
                *reinterpret_cast<uint4 *>(&tile[tile_pos(row, dw + 4)]) = make_uint4(d[4], d[5], d[6], d[7]);
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
                if (PACKED) { x0[i] = x0[i] * src_sg; x1[i] = x1[i] * src_sg; }
            }
            float m = u2f((uint32_t)(j == 0 ? m2.x : m2.y) << 16);
            if (PACKED) m = m * src_sg;                                     // rounding is monotone: = max |x|
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
    return k;
}

template <int ROUND, bool SUP, int OUTER>
void launch_row_t(const RowJob &j0, const RowJob &j1, bool deq, hipStream_t st)
{
    const int64_t per_wg = (int64_t)kThreads * kRowIter;
    const unsigned g0 = (unsigned)((j0.nchunks + per_wg - 1) / per_wg), g1 = (unsigned)((j1.nchunks + per_wg - 1) / per_wg);
    const unsigned first_second = g1 ? g0 : 0xFFFFFFFFu;
    if (deq)
        hipLaunchKernelGGL((quant_row_kernel<ROUND, SUP, OUTER, true>), dim3(g0 + g1), dim3(kThreads), 0, st, j0, j1,
                           first_second);
    else
        hipLaunchKernelGGL((quant_row_kernel<ROUND, SUP, OUTER, false>), dim3(g0 + g1), dim3(kThreads), 0, st, j0, j1,
                           first_second);
}

template <bool PACKED>
void launch_col_t(ColArgs &a0, ColArgs &a1, bool pair, int rounding, int scale_up, hipStream_t st)
{
    const unsigned g0 = col_grid(a0), g1 = pair ? col_grid(a1) : 0;
    const unsigned first_second = pair ? g0 : 0xFFFFFFFFu;
    const dim3 grid(g0 + g1);
    if (rounding == 0) {
        if (scale_up) hipLaunchKernelGGL((quant_col_kernel<0, true, PACKED>), grid, dim3(kThreads), 0, st, a0, a1, first_second);
        else          hipLaunchKernelGGL((quant_col_kernel<0, false, PACKED>), grid, dim3(kThreads), 0, st, a0, a1, first_second);
    } else {
        if (scale_up) hipLaunchKernelGGL((quant_col_kernel<1, true, PACKED>), grid, dim3(kThreads), 0, st, a0, a1, first_second);
        else          hipLaunchKernelGGL((quant_col_kernel<1, false, PACKED>), grid, dim3(kThreads), 0, st, a0, a1, first_second);
    }
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
    switch (sel) {
        case 0: launch_row_t<0, false, 0>(j0, j1, deq, st); break;
        case 1: launch_row_t<0, false, 1>(j0, j1, deq, st); break;
        case 2: launch_row_t<0, true, 0>(j0, j1, deq, st); break;
        case 3: launch_row_t<0, true, 1>(j0, j1, deq, st); break;
        case 4: launch_row_t<1, false, 0>(j0, j1, false, st); break;
        case 5: launch_row_t<1, false, 1>(j0, j1, false, st); break;
        case 6: launch_row_t<1, true, 0>(j0, j1, false, st); break;
        default: launch_row_t<1, true, 1>(j0, j1, false, st); break;
    }
}

hipError_t launch_quant_row_bf16(const void *src, int64_t rows, int64_t K, const QuantParams &p, const QuantOut &o,
                                 hipStream_t st)
{
    const int64_t nchunks = rows * K / 8;
    if (nchunks == 0) return hipSuccess;
    RowJob j0{reinterpret_cast<const uint4 *>(src), nchunks, make_kargs(p, o)}, j1{};
    launch_row_sel(j0, j1, p, o.amax_deq != nullptr && p.rounding == 0, st);
    return hipGetLastError();
}

hipError_t launch_quant_row_bf16_pair(const void *src0, int64_t rows0, int64_t K0, const QuantParams &p0,
                                      const QuantOut &o0, const void *src1, int64_t rows1, int64_t K1,
                                      const QuantParams &p1, const QuantOut &o1, hipStream_t st)
{
    if (rows0 * K0 == 0) return launch_quant_row_bf16(src1, rows1, K1, p1, o1, st);
    if (rows1 * K1 == 0) return launch_quant_row_bf16(src0, rows0, K0, p0, o0, st);
    RowJob j0{reinterpret_cast<const uint4 *>(src0), rows0 * K0 / 8, make_kargs(p0, o0)};
    RowJob j1{reinterpret_cast<const uint4 *>(src1), rows1 * K1 / 8, make_kargs(p1, o1)};
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
    launch_col_t<false>(a, none, false, p.rounding, p.scale_up, st);
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
    const ColArgs none{};
    const unsigned fs = 0xFFFFFFFFu;
    const int sel = (pcol.rounding << 1) | pcol.scale_up;
    switch (sel) {
        case 0: hipLaunchKernelGGL((quant_col_kernel<0, false, false, true>), grid, dim3(kThreads), 0, st, a, none, fs); break;
        case 1: hipLaunchKernelGGL((quant_col_kernel<0, true, false, true>), grid, dim3(kThreads), 0, st, a, none, fs); break;
        case 2: hipLaunchKernelGGL((quant_col_kernel<1, false, false, true>), grid, dim3(kThreads), 0, st, a, none, fs); break;
        default: hipLaunchKernelGGL((quant_col_kernel<1, true, false, true>), grid, dim3(kThreads), 0, st, a, none, fs); break;
    }
    return hipGetLastError();
}

static ColArgs packed_args(const PackedSrc &src, int64_t R, int64_t C, const QuantParams &p, const QuantOut &o)
{
    ColArgs a{};
    a.src_codes = src.codes;
    a.src_scales = src.scales;
    a.src_gscale = src.gscale;
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
    launch_col_t<true>(a, none, false, p.rounding, p.scale_up, st);
    return hipGetLastError();
}

hipError_t launch_requant_col_pair(const PackedSrc &src0, int64_t R0, int64_t C0, const QuantParams &p0,
                                   const QuantOut &o0, const PackedSrc &src1, int64_t R1, int64_t C1,
                                   const QuantParams &p1, const QuantOut &o1, hipStream_t st)
{
    if (R0 == 0 || C0 == 0) return launch_requant_col(src1, R1, C1, p1, o1, st);
    if (R1 == 0 || C1 == 0) return launch_requant_col(src0, R0, C0, p0, o0, st);
    ColArgs a0 = packed_args(src0, R0, C0, p0, o0), a1 = packed_args(src1, R1, C1, p1, o1);
    launch_col_t<true>(a0, a1, true, p0.rounding, p0.scale_up, st);
    return hipGetLastError();
}

}  // namespace tj
