// High-precision side of the OutControl split linear (TetraJet-v2 Sec. 4.2): the few outlier channels of the
// activation stay in bf16 and their products run on the bf16 MFMA path with FP32 accumulation:
//   hp_gemm_nt    Out[M x N] = Addend + A[M x K] * B[N x K]^T, A and B bf16 with K contiguous (the forward term
//                 X_A W_A^T added to the FP4 product, and dW_A = dY^T X_A on transposed copies)
//   transpose     bf16 [R x C] -> [C x R] (dY^T and X_A^T for the weight-gradient term: its reduction runs over tokens)
// These carry about a tenth of the layer's flops.  The product kernel has the structure of the NVFP4 one without the
// expansion: 2 x 2 waves of TM x TN MFMA tiles (32 x 32 each), a pipeline stage of 32 k = 64 bytes per tile row copied
// global -> LDS directly (three stages in flight in a ring of three buffers, the same 16-row swizzle), fragments read
// with one 128-bit LDS read per MFMA operand, one barrier per stage placed between the stage's two 16-k steps so that
// the next stage's first fragments are read under the second step's MFMAs.
#include <type_traits>

#include "device_fmt.h"
#include "gemm_args.h"
#include "internal.h"

namespace tj {

namespace {

constexpr int kThreads = 256;

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

struct HpArgs {
    const uint16_t *A, *B;     // bf16 [M x K], [N x K]
    const float *addend;       // optional f32 [M x N]
    void *out;                 // bf16 or f32 [M x N]
    int64_t M, N, K;
    int out_f32;
    int tiles_n;
};

// global -> LDS copy that bypasses registers (16 bytes per lane, the wave's data lands at lds_addr + lane * 16); inline
// assembly so that completion is tracked only by the explicit s_waitcnt vmcnt(n) below
__device__ __forceinline__ void hp_dma16(const void *base, uint32_t off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(off), "s"(base) : "memory", "m0");
}

template <int TM, int TN>
__global__ __launch_bounds__(kThreads, (TM * TN >= 16 ? 1 : 2)) void hp_gemm_nt_kernel(HpArgs g)
{
    constexpr int BM = 64 * TM, BN = 64 * TN, ROWS = BM + BN;
    constexpr int SLOTS = 4;                               // 16-byte pieces per tile row and stage (32 k of bf16)
    constexpr int LA = BM * SLOTS / kThreads, LB = BN * SLOTS / kThreads, L = LA + LB;   // copies per thread and stage
    constexpr int STAGE_BYTES = ROWS * SLOTS * 16;
    static_assert(L <= 15, "vmcnt immediate");
    extern __shared__ __attribute__((aligned(16))) uint8_t hp_smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1, lr = lane & 31, kg = lane >> 5;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)hp_smem;
    const int64_t m0 = (int64_t)(blockIdx.x / g.tiles_n) * BM, n0 = (int64_t)(blockIdx.x % g.tiles_n) * BN;
    const int nk = (int)(g.K / 32);

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    if (nk > 0) {
        // copy u of a stage: slot (4 u + wave) * 64 + lane of the A part (u < LA) or the B part; slot = row * 4 + position,
        // position p holds piece p ^ ((row / 4) % 4) of the row.  Rows past the end of the operand read its last row
        // (valid memory; their products are never stored).
        uint32_t off[L];
#pragma unroll
        for (int u = 0; u < L; ++u) {
            const bool isA = u < LA;
            const int slot = ((isA ? u : u - LA) * 4 + wave) * 64 + lane, row = slot / SLOTS, pos = slot % SLOTS;
            const int piece = pos ^ ((row >> 2) & (SLOTS - 1));
            const int64_t last = (isA ? g.M - m0 : g.N - n0) - 1;
            const int64_t r = row < last ? row : last;
            off[u] = (uint32_t)(r * g.K * 2) + (uint32_t)piece * 16u;
        }
        const uint8_t *a_base = reinterpret_cast<const uint8_t *>(g.A + m0 * g.K);
        const uint8_t *b_base = reinterpret_cast<const uint8_t *>(g.B + n0 * g.K);
        // every call issues exactly L copies (the waits below count them); stages past the end repeat the last one
        auto issue = [&](int kt, int buf) {
            const int64_t ko = (int64_t)(kt < nk ? kt : nk - 1) * 64;
#pragma unroll
            for (int u = 0; u < L; ++u) {
                const bool isA = u < LA;
                const int wslot = (isA ? 0 : BM * SLOTS) + ((isA ? u : u - LA) * 4 + wave) * 64;
                hp_dma16((isA ? a_base : b_base) + ko, off[u], lds_base + buf * STAGE_BYTES + wslot * 16);
            }
        };
        struct Frags { bf16x8_t a[TM], b[TN]; };
        // operands of 16-k step ks of the stage in buffer buf: a lane feeds row lr of each 32 x 32 tile with the eight k
        // of its half (kg) of the step
        auto read = [&](Frags &f, int buf, int ks) {
            const uint8_t *base = hp_smem + buf * STAGE_BYTES;
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int row = (wm * TM + i) * 32 + lr;
                f.a[i] = *reinterpret_cast<const bf16x8_t *>(base + (row * SLOTS + ((2 * ks + kg) ^ ((row >> 2) & (SLOTS - 1)))) * 16);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int row = (wn * TN + j) * 32 + lr;
                f.b[j] = *reinterpret_cast<const bf16x8_t *>(base + ((BM + row) * SLOTS + ((2 * ks + kg) ^ ((row >> 2) & (SLOTS - 1)))) * 16);
            }
        };
        issue(0, 0);
        issue(1, 1);
        issue(2, 2);
        __builtin_amdgcn_s_waitcnt(0x0F70 | ((2 * L) & 15) | (((2 * L) >> 4) << 14));   // vmcnt(2 L): stage 0 has landed
        __syncthreads();
        Frags f0, f1;
        read(f0, 0, 0);
        int buf = 0;
        for (int kt = 0; kt < nk; ++kt) {
            const int nbuf = buf == 2 ? 0 : buf + 1;
            read(f1, buf, 1);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f0.a[i], f0.b[j], acc[i][j], 0, 0, 0);
            // every read of this stage's buffer has returned (this wave's), stage kt + 1 has landed (this wave's copies):
            // after the barrier both hold for the workgroup, so the buffer can take stage kt + 3
            __builtin_amdgcn_s_waitcnt(0x0070 | L);            // vmcnt(L), lgkmcnt(0)
            __syncthreads();
            issue(kt + 3, buf);
            read(f0, nbuf, 0);                                  // (after the last stage: stale bytes, never used)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f1.a[i], f1.b[j], acc[i][j], 0, 0, 0);
            buf = nbuf;
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);                     // drain the copies before the LDS is released
    }

    // accumulator element e of a lane: row 8 * (e / 4) + 4 * (lane / 32) + e % 4, column lane % 32.  An element's index is
    // a wave-uniform part (tile, block, e) plus one per-lane offset that is the same for all of them, so the stores and
    // addend loads take a scalar base and that one vector offset.  One copy of the loop nest per (addend, output type,
    // whole tile) so that each is branch-free inside and unrolls completely.
    const uint32_t lane_off = (uint32_t)(4 * kg) * (uint32_t)g.N + (uint32_t)lr;      // N < 2^29 (checked on the host)
    auto emit = [&](auto add_c, auto f32_c, auto full_c) {
        constexpr bool ADD = decltype(add_c)::value, F32 = decltype(f32_c)::value, FULL = decltype(full_c)::value;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int64_t mb = m0 + (wm * TM + i) * 32, nb = n0 + (wn * TN + j) * 32;      // uniform
                const bool n_ok = FULL || nb + lr < g.N;
                // the block's sixteen addends first (loads in flight together), then element by element
                float ad[16];
                if (ADD) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int64_t mu = mb + 8 * (e >> 2) + (e & 3);                          // uniform part of the row
                        ad[e] = 0.0f;
                        if (FULL || (n_ok && mu + 4 * kg < g.M)) ad[e] = (g.addend + (mu * g.N + nb))[lane_off];
                    }
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int64_t mu = mb + 8 * (e >> 2) + (e & 3);
                    const int64_t base = mu * g.N + nb;
                    if (FULL || (n_ok && mu + 4 * kg < g.M)) {
                        // the accumulators stay in their accumulation registers until the element is written: read
                        // here, not hoisted above the choice of the epilogue variant
                        float v;
                        asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(acc[i][j][e]));
                        if (ADD) v = ad[e] + v;
                        if (F32) (reinterpret_cast<float *>(g.out) + base)[lane_off] = v;
                        else (reinterpret_cast<uint16_t *>(g.out) + base)[lane_off] = (uint16_t)f32_to_bf16_bits(v);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);          // one 32 x 32 block on its way out at a time
            }
    };
    auto emit2 = [&](auto add_c, auto f32_c) {
        if (m0 + BM <= g.M && n0 + BN <= g.N) emit(add_c, f32_c, std::true_type{});
        else emit(add_c, f32_c, std::false_type{});
    };
    if (g.addend) {
        if (g.out_f32) emit2(std::true_type{}, std::true_type{});
        else emit2(std::true_type{}, std::false_type{});
    } else {
        if (g.out_f32) emit2(std::false_type{}, std::true_type{});
        else emit2(std::false_type{}, std::false_type{});
    }
}

// 64 x 64 tile through LDS (one padding element per row); R and C arbitrary
__global__ __launch_bounds__(kThreads) void transpose_bf16_kernel(const uint16_t *src, uint16_t *dst, int64_t R, int64_t C, int tiles_c)
{
    __shared__ uint16_t tile[64][66];
    const int64_t r0 = (int64_t)(blockIdx.x / tiles_c) * 64, c0 = (int64_t)(blockIdx.x % tiles_c) * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t r = r0 + ty + 4 * i, c = c0 + tx;
        if (r < R && c < C) tile[ty + 4 * i][tx] = src[r * C + c];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t c = c0 + ty + 4 * i, r = r0 + tx;
        if (r < R && c < C) dst[c * R + r] = tile[tx][ty + 4 * i];
    }
}

// the same for even R and C, 64 x 128 tile, two elements per access: a wave reads 256 contiguous bytes of a source row and
// writes 128 contiguous bytes of a destination row
__global__ __launch_bounds__(kThreads) void transpose_bf16_pairs_kernel(const uint16_t *src, uint16_t *dst, int64_t R, int64_t C,
                                                                        int tiles_c)
{
    __shared__ __attribute__((aligned(4))) uint16_t tile[64][130];
    const int64_t r0 = (int64_t)(blockIdx.x / tiles_c) * 64, c0 = (int64_t)(blockIdx.x % tiles_c) * 128;
    {
        const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t r = r0 + ty + 4 * i, c = c0 + 2 * tx;
            if (r < R && c < C) *reinterpret_cast<uint32_t *>(&tile[ty + 4 * i][2 * tx]) = *reinterpret_cast<const uint32_t *>(src + r * C + c);
        }
    }
    __syncthreads();
    {
        const int rr = threadIdx.x & 31, cc = threadIdx.x >> 5;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int cl = cc + 8 * i;
            const int64_t c = c0 + cl, r = r0 + 2 * rr;
            if (c < C && r < R)
                *reinterpret_cast<uint32_t *>(dst + c * R + r) = (uint32_t)tile[2 * rr][cl] | ((uint32_t)tile[2 * rr + 1][cl] << 16);
        }
    }
}

}  // namespace

template <int TM, int TN>
static hipError_t launch_hp_t(HpArgs g, hipStream_t st)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int lds = 3 * (BM + BN) * 64;
    auto kern = hp_gemm_nt_kernel<TM, TN>;
    // once per instantiation; the initialisation of a function-local static is thread-safe
    static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (attr != hipSuccess) return attr;
    g.tiles_n = (int)((g.N + BN - 1) / BN);
    const int64_t tiles = ((g.M + BM - 1) / BM) * g.tiles_n;
    hipLaunchKernelGGL(kern, dim3((unsigned)tiles), dim3(kThreads), lds, st, g);
    return hipGetLastError();
}

hipError_t launch_hp_gemm_nt(const void *A, const void *B, int64_t M, int64_t N, int64_t K, const float *addend, void *out,
                             int out_f32, hipStream_t st)
{
    if (M == 0 || N == 0) return hipSuccess;
    // 32-bit byte offsets inside a tile's operand rows and element offsets inside four output rows
    if (K % 32 != 0 || K > ((int64_t)1 << 22) || N >= ((int64_t)1 << 29)) return hipErrorInvalidValue;
    HpArgs g;
    g.A = static_cast<const uint16_t *>(A);
    g.B = static_cast<const uint16_t *>(B);
    g.addend = addend;
    g.out = out;
    g.M = M; g.N = N; g.K = K;
    g.out_f32 = out_f32;
    g.tiles_n = 0;
    // 256 x 256 tiles when they fill the chip, else 128 x 128
    const int64_t big = ((M + 255) / 256) * ((N + 255) / 256);
    return big >= 192 ? launch_hp_t<4, 4>(g, st) : launch_hp_t<2, 2>(g, st);
}

hipError_t launch_transpose_bf16(const void *src, void *dst, int64_t R, int64_t C, hipStream_t st)
{
    if (R == 0 || C == 0) return hipSuccess;
    if (R % 2 == 0 && C % 2 == 0) {
        const int tc = (int)((C + 127) / 128);
        hipLaunchKernelGGL(transpose_bf16_pairs_kernel, dim3((unsigned)(((R + 63) / 64) * tc)), dim3(kThreads), 0, st,
                           static_cast<const uint16_t *>(src), static_cast<uint16_t *>(dst), R, C, tc);
        return hipGetLastError();
    }
    const int tiles_c = (int)((C + 63) / 64);
    const int64_t tiles = ((R + 63) / 64) * tiles_c;
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)tiles), dim3(kThreads), 0, st, static_cast<const uint16_t *>(src),
                       static_cast<uint16_t *>(dst), R, C, tiles_c);
    return hipGetLastError();
}

}  // namespace tj
