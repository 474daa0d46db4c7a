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
// so the order of k inside a chunk does not matter.
#include "device_fmt.h"
#include "internal.h"

namespace tj {

namespace {

constexpr int kThreads = 256;
constexpr int BK = 64;   // K elements per pipeline stage

struct GemmArgs {
    const uint8_t *a_codes, *a_scales;
    const uint8_t *b_codes, *b_scales;
    const float *a_gscale, *b_gscale;
    void *out;          // bf16 / f32 [M x N], or f32 partials [split][M x N]
    int64_t M, N, K;
    int k_per_split;    // multiple of BK
    int out_mode;       // 0 bf16, 1 f32, 2 raw f32 partial (split-K)
    int tiles_m, tiles_n;
};

// 16-byte slot of (row, half) inside a stage: the half index is flipped every 4 rows so that
// 8 consecutive rows of one half hit 8 different 16-byte bank groups
__device__ __forceinline__ int code_slot(int row, int half) { return row * 2 + (half ^ ((row >> 2) & 1)); }

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

template <int TM, int TN>
__global__ __launch_bounds__(kThreads) void gemm_nt_kernel(GemmArgs g)
{
    constexpr int BM = 2 * TM * 32, BN = 2 * TN * 32;
    constexpr int LA = BM * 2 / kThreads, LB = BN * 2 / kThreads;   // 128-bit code loads per thread
    static_assert(LA >= 1 && LB >= 1, "tile too small");
    static_assert(BM <= kThreads && BN <= kThreads, "one scale dword per thread");

    __shared__ __attribute__((aligned(16))) uint4 a_codes[2][BM * 2];
    __shared__ __attribute__((aligned(16))) uint4 b_codes[2][BN * 2];
    __shared__ uint32_t a_scales[2][BM];
    __shared__ uint32_t b_scales[2][BN];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

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
    const int64_t kbeg = (int64_t)blockIdx.z * g.k_per_split;
    int64_t kend = kbeg + g.k_per_split;
    if (kend > g.K) kend = g.K;
    const int nk = (int)((kend - kbeg) / BK);
    const int64_t cstride = g.K / 2, sstride = g.K / 16;

    uint4 ra[LA], rb[LB];
    uint32_t rs = 0;

    auto load_global = [&](int kt) {
        const int64_t k0 = kbeg + (int64_t)kt * BK;
#pragma unroll
        for (int u = 0; u < LA; ++u) {
            const int idx = tid + u * kThreads, row = idx >> 1, half = idx & 1;
            ra[u] = make_uint4(0, 0, 0, 0);
            if (m0 + row < g.M)
                ra[u] = *reinterpret_cast<const uint4 *>(g.a_codes + (m0 + row) * cstride + k0 / 2 + 16 * half);
        }
#pragma unroll
        for (int u = 0; u < LB; ++u) {
            const int idx = tid + u * kThreads, row = idx >> 1, half = idx & 1;
            rb[u] = make_uint4(0, 0, 0, 0);
            if (n0 + row < g.N)
                rb[u] = *reinterpret_cast<const uint4 *>(g.b_codes + (n0 + row) * cstride + k0 / 2 + 16 * half);
        }
        rs = 0;
        if (tid < BM) {
            if (m0 + tid < g.M) rs = *reinterpret_cast<const uint32_t *>(g.a_scales + (m0 + tid) * sstride + k0 / 16);
        }
        if (BM + BN <= kThreads) {
            if (tid >= BM && tid < BM + BN && n0 + (tid - BM) < g.N)
                rs = *reinterpret_cast<const uint32_t *>(g.b_scales + (n0 + tid - BM) * sstride + k0 / 16);
        }
    };
    uint32_t rs2 = 0;   // second scale register when BM + BN > 256
    auto load_global_s2 = [&](int kt) {
        if (BM + BN > kThreads) {
            const int64_t k0 = kbeg + (int64_t)kt * BK;
            rs2 = 0;
            if (tid < BN && n0 + tid < g.N)
                rs2 = *reinterpret_cast<const uint32_t *>(g.b_scales + (n0 + tid) * sstride + k0 / 16);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int u = 0; u < LA; ++u) {
            const int idx = tid + u * kThreads;
            a_codes[buf][code_slot(idx >> 1, idx & 1)] = ra[u];
        }
#pragma unroll
        for (int u = 0; u < LB; ++u) {
            const int idx = tid + u * kThreads;
            b_codes[buf][code_slot(idx >> 1, idx & 1)] = rb[u];
        }
        if (tid < BM) a_scales[buf][tid] = rs;
        if (BM + BN <= kThreads) {
            if (tid >= BM && tid < BM + BN) b_scales[buf][tid - BM] = rs;
        } else {
            if (tid < BN) b_scales[buf][tid] = rs2;
        }
    };

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    const int lr = lane & 31, kg = lane >> 5;

    if (nk > 0) {
        load_global(0);
        load_global_s2(0);
        store_lds(0);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) {
            load_global(kt + 1);
            load_global_s2(kt + 1);
        }
        // this lane's 32 codes and 2 scale bytes per fragment
        uint4 qa[TM], qb[TN];
        half2_t fa[TM][2], fb[TN][2];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row = (wm * TM + i) * 32 + lr;
            qa[i] = a_codes[buf][code_slot(row, kg)];
            const uint32_t s = a_scales[buf][row] >> (16 * kg);
            fa[i][0] = scale_pair(s & 0xFFu);
            fa[i][1] = scale_pair((s >> 8) & 0xFFu);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int row = (wn * TN + j) * 32 + lr;
            qb[j] = b_codes[buf][code_slot(row, kg)];
            const uint32_t s = b_scales[buf][row] >> (16 * kg);
            fb[j][0] = scale_pair(s & 0xFFu);
            fb[j][1] = scale_pair((s >> 8) & 0xFFu);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            half8_t av[TM], bv[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const uint32_t q = ks == 0 ? qa[i].x : ks == 1 ? qa[i].y : ks == 2 ? qa[i].z : qa[i].w;
                av[i] = expand8(q, fa[i][ks >> 1]);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const uint32_t q = ks == 0 ? qb[j].x : ks == 1 ? qb[j].y : ks == 2 ? qb[j].z : qb[j].w;
                bv[j] = expand8(q, fb[j][ks >> 1]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_lds(buf ^ 1);
        __syncthreads();
    }

    // epilogue: acc element e of lane: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
    float alpha = 1.0f;
    if (g.out_mode != 2) alpha = g.a_gscale[0] * g.b_gscale[0] * 256.0f;
    float *outf = reinterpret_cast<float *>(g.out);
    if (g.out_mode == 2) outf += (int64_t)blockIdx.z * g.M * g.N;
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
                    if (g.out_mode == 0) outh[m * g.N + n] = (uint16_t)f32_to_bf16_bits(v);
                    else outf[m * g.N + n] = v;
                }
            }
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
        for (int64_t i = i4; i < mn; ++i) {
            float s = part[i];
            for (int z = 1; z < split; ++z) s += part[(int64_t)z * mn + i];
            s *= alpha;
            if (out_f32) reinterpret_cast<float *>(out)[i] = s;
            else reinterpret_cast<uint16_t *>(out)[i] = (uint16_t)f32_to_bf16_bits(s);
        }
    }
}

constexpr int kTM = 2, kTN = 2;
constexpr int kBM = 2 * kTM * 32, kBN = 2 * kTN * 32;

int choose_split(int64_t M, int64_t N, int64_t K)
{
    const int64_t tiles = ((M + kBM - 1) / kBM) * ((N + kBN - 1) / kBN);
    const int64_t chunks = K / BK;
    if (tiles >= 384 || chunks < 16) return 1;
    int64_t split = (768 + tiles - 1) / tiles;          // aim at ~3 workgroups per CU
    if (split > chunks / 8) split = chunks / 8;          // at least 8 chunks (512 k) per split
    if (split > 32) split = 32;
    return split < 1 ? 1 : (int)split;
}

}  // namespace

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K)
{
    const int split = choose_split(M, N, K);
    return split > 1 ? (size_t)split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

hipError_t launch_gemm_nt(const GemmOperand &A, const GemmOperand &B, int64_t K, void *out, int out_f32,
                          void *ws, size_t ws_bytes, hipStream_t st)
{
    const int64_t M = A.rows, N = B.rows;
    if (M == 0 || N == 0) return hipSuccess;
    GemmArgs g;
    g.a_codes = A.codes; g.a_scales = A.scales; g.a_gscale = A.gscale;
    g.b_codes = B.codes; g.b_scales = B.scales; g.b_gscale = B.gscale;
    g.M = M; g.N = N; g.K = K;
    g.tiles_m = (int)((M + kBM - 1) / kBM);
    g.tiles_n = (int)((N + kBN - 1) / kBN);
    int split = choose_split(M, N, K);
    if (split > 1 && (ws == nullptr || ws_bytes < (size_t)split * M * N * sizeof(float))) split = 1;
    const int64_t chunks = K / BK;
    const int64_t cps = (chunks + split - 1) / split;
    g.k_per_split = (int)(cps * BK);
    if (K == 0) { g.k_per_split = 0; split = 1; }
    split = cps > 0 ? (int)((chunks + cps - 1) / cps) : 1;
    if (split > 1) {
        g.out = ws;
        g.out_mode = 2;
    } else {
        g.out = out;
        g.out_mode = out_f32 ? 1 : 0;
    }
    dim3 grid((unsigned)(g.tiles_m * g.tiles_n), 1, (unsigned)split);
    hipLaunchKernelGGL((gemm_nt_kernel<kTM, kTN>), grid, dim3(kThreads), 0, st, g);
    if (split > 1) {
        const int64_t mn = M * N;
        const unsigned rgrid = (unsigned)((mn + (int64_t)kThreads * 4 - 1) / ((int64_t)kThreads * 4));
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(rgrid), dim3(kThreads), 0, st,
                           reinterpret_cast<const float *>(ws), split, mn, A.gscale, B.gscale, out, out_f32);
    }
    return hipGetLastError();
}

}  // namespace tj
