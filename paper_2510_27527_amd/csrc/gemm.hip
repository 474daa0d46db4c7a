// NT GEMM on two packed NVFP4 operands for gfx950 (the three products of TetraJet-v2 Sec. 2.3
// all reduce to Out[M x N] = A[M x K] * B[N x K]^T once each operand is grouped along K).
//
// CDNA4's block-scaled MFMA takes E8M0 scales per 32 elements, NVFP4 has E4M3 scales per 16, so
// the exact route is: stage the packed tiles (codes + scale bytes) in LDS, expand
// code * S_block to FP16 in registers (6 significant bits, 2^-14 <= |v| <= 168 after a 2^-4
// pre-scale: exact and normal in FP16), feed v_mfma_f32_32x32x16_f16 with FP32 accumulation and
// multiply by the two FP32 outer scales (and 2^8) in the epilogue.
//
// Work split: 256 threads = 2 x 2 waves; each wave owns TM x TN tiles of 32 x 32.  Within one
// 64-wide K chunk a lane (row r = lane % 32, kg = lane / 32) holds the 32 codes k = 32 kg .. 32 kg + 31
// of its row (one 128-bit LDS read) and uses 8 of them per MFMA; A and B use the same assignment,
// so the order of k inside a chunk does not matter.  Small outputs with a long reduction (the
// weight gradient) are split along K into FP32 partials that a second kernel sums in a fixed order.
#include "device_fmt.h"
#include "internal.h"

namespace tj {

namespace {

constexpr int kThreads = 256;

struct GemmArgs {
    const uint8_t *a_codes, *a_scales;
    const uint8_t *b_codes, *b_scales;
    const float *a_gscale, *b_gscale;
    void *out;          // bf16 / f32 [M x N], or f32 partials [split][M x N]
    int64_t M, N, K;
    int chunks_per_split;   // 64-wide K chunks per split
    int out_f32;
    int tiles_m, tiles_n;
};

__device__ __forceinline__ half2_t scale_pair(uint32_t sc)
{
    // E4M3 byte << 7 is the FP16 pattern of S_block * 2^-8 (same field layout, bias 15 vs 7);
    // times 16 gives S_block * 2^-4, normal in FP16 for every code
    const uint32_t bits = sc * 0x00800080u;
    const half2_t sixteen = {(_Float16)16.0f, (_Float16)16.0f};
    return __builtin_bit_cast(half2_t, bits) * sixteen;
}

// eight codes (one dword) times the block scale -> eight FP16
__device__ __forceinline__ half8_t expand8(uint32_t q, half2_t f)
{
    const half2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q, 1.0f, 0) * f;
    const half2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q, 1.0f, 1) * f;
    const half2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q, 1.0f, 2) * f;
    const half2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(q, 1.0f, 3) * f;
    half8_t r;
    r[0] = p0.x; r[1] = p0.y; r[2] = p1.x; r[3] = p1.y;
    r[4] = p2.x; r[5] = p2.y; r[6] = p3.x; r[7] = p3.y;
    return r;
}

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t b = f2u(f);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ uint32_t pick(uint4 v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// Tile TM*64 x TN*64 per workgroup (2 x 2 waves, TM x TN MFMA tiles of 32 x 32 each), NC chunks of
// 64 k per pipeline stage, two stages in LDS.  Codes go global -> LDS directly (128 bits per lane, a
// wave fills 1 KB = 64 consecutive 16-byte slots); scale bytes pass through registers.
// LDS slot of (row, 16-byte piece p of the stage's row segment) = row * SLOTS + (p ^ f(row)).
template <int TM, int TN, int NC, int OUT>   // OUT: 0 bf16, 1 f32, 2 raw f32 split-K partial
__global__ __launch_bounds__(kThreads, (TM * TN >= 16 ? 1 : 2)) void gemm_nt_kernel(GemmArgs g)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int SLOTS = 2 * NC;                       // 16-byte pieces per row per stage
    constexpr int A_SLOTS = BM * SLOTS, B_SLOTS = BN * SLOTS;
    constexpr int LA = A_SLOTS / kThreads, LB = B_SLOTS / kThreads;
    constexpr int STAGE_U4 = A_SLOTS + B_SLOTS;          // uint4 per stage (codes)
    constexpr int STAGE_SC = (BM + BN) * NC;             // dwords per stage (scales)
    static_assert(BM <= kThreads && BN <= kThreads, "one scale row per thread");
    static_assert(LA >= 1 && LB >= 1, "tile too small");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem_raw[];
    uint4 *codes_lds = reinterpret_cast<uint4 *>(smem_raw);                            // [2][STAGE_U4]
    uint32_t *scales_lds = reinterpret_cast<uint32_t *>(smem_raw + 2 * STAGE_U4 * 16); // [2][STAGE_SC]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int lr = lane & 31, kg = lane >> 5;

    // workgroup -> tile: consecutive ids of one XCD (ids are dealt round-robin over 8 XCDs) walk
    // down a column of tiles, in groups of 8 tile rows
    const int total = g.tiles_m * g.tiles_n;
    int pid = blockIdx.x;
    {
        const int per_xcd = total / 8;
        if (pid < per_xcd * 8) pid = (pid & 7) * per_xcd + (pid >> 3);
    }
    constexpr int GROUP = 8;
    const int group_sz = GROUP * g.tiles_n;
    const int gid = pid / group_sz;
    const int first_m = gid * GROUP;
    const int gm = (g.tiles_m - first_m) < GROUP ? (g.tiles_m - first_m) : GROUP;
    const int tile_m = first_m + (pid % group_sz) % gm;
    const int tile_n = (pid % group_sz) / gm;

    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;
    const int64_t chunks_total = g.K / 64;
    const int64_t cbeg = (int64_t)blockIdx.z * g.chunks_per_split;
    int64_t cend = cbeg + g.chunks_per_split;
    if (cend > chunks_total) cend = chunks_total;
    const int nchunks = (int)(cend - cbeg);
    const int nk = (nchunks + NC - 1) / NC;
    const int64_t cstride = g.K / 2, sstride = g.K / 16;

    // per-thread constants of the code loads: global row pointer and piece index of each slot
    const uint8_t *arow[LA];
    int apiece[LA];
#pragma unroll
    for (int u = 0; u < LA; ++u) {
        const int slot = (u * 4 + wave) * 64 + lane, row = slot / SLOTS, pos = slot % SLOTS;
        int64_t gr = m0 + row;
        if (gr >= g.M) gr = g.M - 1;
        arow[u] = g.a_codes + gr * cstride;
        apiece[u] = pos ^ ((row >> 1) & (SLOTS - 1));
    }
    const uint8_t *brow[LB];
    int bpiece[LB];
#pragma unroll
    for (int u = 0; u < LB; ++u) {
        const int slot = (u * 4 + wave) * 64 + lane, row = slot / SLOTS, pos = slot % SLOTS;
        int64_t gr = n0 + row;
        if (gr >= g.N) gr = g.N - 1;
        brow[u] = g.b_codes + gr * cstride;
        bpiece[u] = pos ^ ((row >> 1) & (SLOTS - 1));
    }
    const bool a_row_ok = tid < BM && m0 + tid < g.M;
    const bool b_row_ok = tid < BN && n0 + tid < g.N;
    const uint8_t *a_srow = g.a_scales + (a_row_ok ? (m0 + tid) : 0) * sstride;
    const uint8_t *b_srow = g.b_scales + (b_row_ok ? (n0 + tid) : 0) * sstride;

    uint32_t sa[NC], sb[NC];

    auto issue_loads = [&](int kt, int buf) {
        const int64_t c0 = cbeg + (int64_t)kt * NC;           // first chunk of the stage
        uint4 *dst = codes_lds + buf * STAGE_U4;
#pragma unroll
        for (int u = 0; u < LA; ++u) {
            int64_t half_chunk = c0 * 2 + apiece[u];          // units of 32 k = 16 bytes
            if (half_chunk >= cend * 2) half_chunk = cend * 2 - 1;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(arow[u] + half_chunk * 16),
                (__attribute__((address_space(3))) void *)(dst + (u * 4 + wave) * 64), 16, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < LB; ++u) {
            int64_t half_chunk = c0 * 2 + bpiece[u];
            if (half_chunk >= cend * 2) half_chunk = cend * 2 - 1;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(brow[u] + half_chunk * 16),
                (__attribute__((address_space(3))) void *)(dst + A_SLOTS + (u * 4 + wave) * 64), 16, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const bool in = c0 + c < cend;
            sa[c] = (a_row_ok && in) ? *reinterpret_cast<const uint32_t *>(a_srow + (c0 + c) * 4) : 0u;
            sb[c] = (b_row_ok && in) ? *reinterpret_cast<const uint32_t *>(b_srow + (c0 + c) * 4) : 0u;
        }
    };
    auto write_scales = [&](int buf) {
        uint32_t *dst = scales_lds + buf * STAGE_SC;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (tid < BM) dst[tid * NC + c] = sa[c];
            if (tid < BN) dst[BM * NC + tid * NC + c] = sb[c];
        }
    };

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    if (nk > 0) {
        issue_loads(0, 0);
        write_scales(0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the direct-to-LDS loads have landed
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) issue_loads(kt + 1, buf ^ 1);
        const uint4 *ac = codes_lds + buf * STAGE_U4;
        const uint4 *bc = ac + A_SLOTS;
        const uint32_t *as = scales_lds + buf * STAGE_SC;
        const uint32_t *bs = as + BM * NC;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            // this lane's 32 codes (k = 32 kg .. 32 kg + 31 of the chunk) and 2 scale bytes per fragment
            uint4 qa[TM], qb[TN];
            half2_t fa[TM][2], fb[TN][2];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = (wm * TM + i) * 32 + lr;
                qa[i] = ac[row * SLOTS + ((2 * c + kg) ^ ((row >> 1) & (SLOTS - 1)))];
                const uint32_t s = as[row * NC + c] >> (16 * kg);
                fa[i][0] = scale_pair(s & 0xFFu);
                fa[i][1] = scale_pair((s >> 8) & 0xFFu);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = (wn * TN + j) * 32 + lr;
                qb[j] = bc[row * SLOTS + ((2 * c + kg) ^ ((row >> 1) & (SLOTS - 1)))];
                const uint32_t s = bs[row * NC + c] >> (16 * kg);
                fb[j][0] = scale_pair(s & 0xFFu);
                fb[j][1] = scale_pair((s >> 8) & 0xFFu);
            }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                half8_t av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) av[i] = expand8(pick(qa[i], ks), fa[i][ks >> 1]);
#pragma unroll
                for (int j = 0; j < TN; ++j) bv[j] = expand8(pick(qb[j], ks), fb[j][ks >> 1]);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
        }
        if (kt + 1 < nk) write_scales(buf ^ 1);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
    }

    // epilogue: acc element e of lane: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
    constexpr bool SPLIT = OUT == 2;
    float alpha = 1.0f;
    if (!SPLIT) alpha = g.a_gscale[0] * g.b_gscale[0] * 256.0f;
    float *outf = reinterpret_cast<float *>(g.out);
    if (SPLIT) outf += (int64_t)blockIdx.z * g.M * g.N;
    uint16_t *outh = reinterpret_cast<uint16_t *>(g.out);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int64_t n = n0 + (wn * TN + j) * 32 + lr;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m0 + (wm * TM + i) * 32 + 8 * (e >> 2) + 4 * kg + (e & 3);
                if (m < g.M && n < g.N) {
                    const float v = acc[i][j][e] * alpha;
                    if (OUT != 0) outf[m * g.N + n] = v;
                    else outh[m * g.N + n] = (uint16_t)f32_to_bf16_bits(v);
                }
            }
            asm volatile("" ::: "memory");       // one tile at a time: keeps the accumulator copies out of VGPRs
        }
}

// sum the split-K partials in split order, scale, convert
__global__ __launch_bounds__(kThreads) void splitk_reduce_kernel(const float *__restrict__ part, int split,
                                                                 int64_t mn, const float *a_gscale,
                                                                 const float *b_gscale, void *out, int out_f32)
{
    const float alpha = a_gscale[0] * b_gscale[0] * 256.0f;
    const int64_t i4 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (i4 >= mn) return;
    if ((mn & 3) == 0) {
        float4 s = *reinterpret_cast<const float4 *>(part + i4);
        for (int z = 1; z < split; ++z) {
            const float4 t = *reinterpret_cast<const float4 *>(part + (int64_t)z * mn + i4);
            s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
        }
        s.x *= alpha; s.y *= alpha; s.z *= alpha; s.w *= alpha;
        if (out_f32) {
            *reinterpret_cast<float4 *>(reinterpret_cast<float *>(out) + i4) = s;
        } else {
            uint2 p;
            p.x = f32_to_bf16_bits(s.x) | (f32_to_bf16_bits(s.y) << 16);
            p.y = f32_to_bf16_bits(s.z) | (f32_to_bf16_bits(s.w) << 16);
            *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + i4) = p;
        }
    } else {
        for (int64_t i = i4; i < mn && i < i4 + 4; ++i) {
            float s = part[i];
            for (int z = 1; z < split; ++z) s += part[(int64_t)z * mn + i];
            s *= alpha;
            if (out_f32) reinterpret_cast<float *>(out)[i] = s;
            else reinterpret_cast<uint16_t *>(out)[i] = (uint16_t)f32_to_bf16_bits(s);
        }
    }
}

// ---- host side: tile shape and split choice ---------------------------------------------------

struct TileCfg { int tm, tn; double eff; };
// relative MFMA efficiency of a workgroup tile: the FP4 -> FP16 expansion is per fragment, the MFMA
// work per fragment pair, so larger wave tiles amortise the expansion better
const TileCfg kTiles[] = {{4, 4, 1.00}, {4, 2, 0.80}, {2, 4, 0.80}, {2, 2, 0.55}};
constexpr int kNumCU = 256;
constexpr int kNC = 2;

struct Plan { int tile; int split; int chunks_per_split; };

Plan make_plan(int64_t M, int64_t N, int64_t K)
{
    const int64_t chunks = K / 64;
    Plan best{3, 1, (int)chunks};
    double best_t = 1e300;
    for (int t = 0; t < 4; ++t) {
        const int64_t bm = 64 * kTiles[t].tm, bn = 64 * kTiles[t].tn;
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        for (int split = 1; split <= 16; split *= 2) {
            if (split > 1 && chunks / split < 8) break;
            const int64_t cps = (chunks + split - 1) / split;
            const int64_t wgs = tiles * split;
            const int64_t rounds = (wgs + kNumCU - 1) / kNumCU;
            // time ~ rounds * work of one workgroup / efficiency (+ fixed cost per round, + the reduction pass)
            double time = (double)rounds * ((double)(bm * bn) * (double)(cps * 64) / kTiles[t].eff + 4.0e6);
            if (split > 1) time += (double)(M * N) * (double)split * 6.0 / kNumCU * 4.0;
            if (time < best_t) { best_t = time; best = Plan{t, split, (int)cps}; }
        }
    }
    if (chunks == 0) best = Plan{3, 1, 0};
    return best;
}

template <int TM, int TN, int OUT>
hipError_t launch_cfg(const GemmArgs &g, dim3 grid, hipStream_t st)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int lds = 2 * ((BM + BN) * 2 * kNC * 16 + (BM + BN) * kNC * 4);
    auto kern = gemm_nt_kernel<TM, TN, kNC, OUT>;
    static bool attr_set = false;
    if (!attr_set) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, grid, dim3(kThreads), lds, st, g);
    return hipGetLastError();
}

template <int OUT>
hipError_t launch_tile(int tile, const GemmArgs &g, dim3 grid, hipStream_t st)
{
    switch (tile) {
        case 0: return launch_cfg<4, 4, OUT>(g, grid, st);
        case 1: return launch_cfg<4, 2, OUT>(g, grid, st);
        case 2: return launch_cfg<2, 4, OUT>(g, grid, st);
        default: return launch_cfg<2, 2, OUT>(g, grid, st);
    }
}

}  // namespace

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    const Plan p = make_plan(M, N, K);
    return p.split > 1 ? (size_t)p.split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

hipError_t launch_gemm_nt(const GemmOperand &A, const GemmOperand &B, int64_t K, void *out, int out_f32,
                          void *ws, size_t ws_bytes, hipStream_t st)
{
    const int64_t M = A.rows, N = B.rows;
    if (M == 0 || N == 0) return hipSuccess;
    Plan p = make_plan(M, N, K);
    if (p.split > 1 && (ws == nullptr || ws_bytes < (size_t)p.split * M * N * sizeof(float))) return hipErrorInvalidValue;
    GemmArgs g;
    g.a_codes = A.codes; g.a_scales = A.scales; g.a_gscale = A.gscale;
    g.b_codes = B.codes; g.b_scales = B.scales; g.b_gscale = B.gscale;
    g.M = M; g.N = N; g.K = K;
    const int bm = 64 * kTiles[p.tile].tm, bn = 64 * kTiles[p.tile].tn;
    g.tiles_m = (int)((M + bm - 1) / bm);
    g.tiles_n = (int)((N + bn - 1) / bn);
    g.chunks_per_split = p.chunks_per_split;
    g.out_f32 = out_f32;
    const int64_t chunks = K / 64;
    const int split = p.split > 1 ? (int)((chunks + p.chunks_per_split - 1) / p.chunks_per_split) : 1;
    g.out = split > 1 ? ws : out;
    dim3 grid((unsigned)(g.tiles_m * g.tiles_n), 1, (unsigned)split);
    hipError_t e = split > 1 ? launch_tile<2>(p.tile, g, grid, st)
                   : out_f32 ? launch_tile<1>(p.tile, g, grid, st) : launch_tile<0>(p.tile, g, grid, st);
    if (e != hipSuccess) return e;
    if (split > 1) {
        const int64_t mn = M * N;
        const unsigned rgrid = (unsigned)((mn + (int64_t)kThreads * 4 - 1) / ((int64_t)kThreads * 4));
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(rgrid), dim3(kThreads), 0, st,
                           reinterpret_cast<const float *>(ws), split, mn, A.gscale, B.gscale, out, out_f32);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace tj
