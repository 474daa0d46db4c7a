// High-precision side of the OutControl split linear (TetraJet-v2 Sec. 4.2): the few outlier channels of the
// activation stay in bf16 and their products run on the bf16 MFMA path with FP32 accumulation:
//   hp_gemm_nt    Out[M x N] = Addend + A[M x K] * B[N x K]^T, A and B bf16 with K contiguous (the forward term
//                 X_A W_A^T added to the FP4 product, and dW_A = dY^T X_A on transposed copies)
//   transpose     bf16 [R x C] -> [C x R] (dY^T and X_A^T for the weight-gradient term: its reduction runs over tokens)
// These carry about a tenth of the layer's flops; the kernel is a plain LDS-tiled one (128 x 128 tile, 2 x 2 waves of
// 2 x 2 MFMA tiles, 32 k per step, the global loads of the next four steps in flight in registers, two LDS buffers so
// that a step costs one barrier).
#include "device_fmt.h"
#include "gemm_args.h"
#include "internal.h"

namespace tj {

namespace {

constexpr int kThreads = 256;
constexpr int kBM = 128, kBN = 128, kBK = 32;
constexpr int kPitch = kBK * 2 + 16;        // bytes per tile row in LDS: 64 of data + 16 of padding (bank spread)

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

struct HpArgs {
    const uint16_t *A, *B;     // bf16 [M x K], [N x K]
    const float *addend;       // optional f32 [M x N]
    void *out;                 // bf16 or f32 [M x N]
    int64_t M, N, K;
    int out_f32;
    int tiles_n;
};

__global__ __launch_bounds__(kThreads) void hp_gemm_nt_kernel(HpArgs g)
{
    constexpr int kBuf = (kBM + kBN) * kPitch, kAhead = 4;
    __shared__ __attribute__((aligned(16))) uint8_t lds_all[2 * kBuf];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1, lr = lane & 31, kg = lane >> 5;
    const int64_t m0 = (int64_t)(blockIdx.x / g.tiles_n) * kBM, n0 = (int64_t)(blockIdx.x % g.tiles_n) * kBN;

    // global -> registers: a tile row is 64 bytes = four 16-byte pieces; thread t takes piece t % 4 of rows t / 4 and
    // t / 4 + 64 of each operand; rows past the end read the last valid row (never stored)
    const int piece = tid & 3, r0 = tid >> 2;
    const int64_t ra0 = m0 + r0 < g.M ? m0 + r0 : g.M - 1, ra1 = m0 + r0 + 64 < g.M ? m0 + r0 + 64 : g.M - 1;
    const int64_t rb0 = n0 + r0 < g.N ? n0 + r0 : g.N - 1, rb1 = n0 + r0 + 64 < g.N ? n0 + r0 + 64 : g.N - 1;
    const uint4 *pa0 = reinterpret_cast<const uint4 *>(g.A + ra0 * g.K) + piece;
    const uint4 *pa1 = reinterpret_cast<const uint4 *>(g.A + ra1 * g.K) + piece;
    const uint4 *pb0 = reinterpret_cast<const uint4 *>(g.B + rb0 * g.K) + piece;
    const uint4 *pb1 = reinterpret_cast<const uint4 *>(g.B + rb1 * g.K) + piece;
    const int nk = (int)(g.K / kBK);
    // one step's share of a thread: four 16-byte pieces (two rows of each operand); four such sets are in flight
    struct Stage { uint4 a0, a1, b0, b1; };
    auto fetch = [&](int kt) {
        const int64_t o = (int64_t)kt * (kBK / 8);
        return Stage{pa0[o], pa1[o], pb0[o], pb1[o]};
    };
    auto put = [&](const Stage &st, uint8_t *lds) {
        *reinterpret_cast<uint4 *>(lds + r0 * kPitch + piece * 16) = st.a0;
        *reinterpret_cast<uint4 *>(lds + (r0 + 64) * kPitch + piece * 16) = st.a1;
        *reinterpret_cast<uint4 *>(lds + (kBM + r0) * kPitch + piece * 16) = st.b0;
        *reinterpret_cast<uint4 *>(lds + (kBM + r0 + 64) * kPitch + piece * 16) = st.b1;
    };

    float16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // one 32-k step from register set st, through LDS buffer `odd`
    auto step = [&](int kt, Stage &st, int odd) {
        uint8_t *lds = lds_all + odd * kBuf;
        // this buffer was last read two steps ago; the barrier of the step in between separates the two uses
        put(st, lds);
        __syncthreads();
        if (kt + kAhead < nk) st = fetch(kt + kAhead);
#pragma unroll
        for (int ks = 0; ks < kBK / 16; ++ks) {
            bf16x8_t a[2], b[2];
            // a lane feeds row lr of a 32 x 32 tile with the 8 consecutive k of its half (kg) of the 16-wide step
#pragma unroll
            for (int i = 0; i < 2; ++i)
                a[i] = *reinterpret_cast<const bf16x8_t *>(lds + ((wm * 2 + i) * 32 + lr) * kPitch + ks * 32 + kg * 16);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                b[j] = *reinterpret_cast<const bf16x8_t *>(lds + (kBM + (wn * 2 + j) * 32 + lr) * kPitch + ks * 32 + kg * 16);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };
    Stage s0{}, s1{}, s2{}, s3{};
    if (0 < nk) s0 = fetch(0);
    if (1 < nk) s1 = fetch(1);
    if (2 < nk) s2 = fetch(2);
    if (3 < nk) s3 = fetch(3);
    for (int kt = 0; kt < nk; kt += kAhead) {          // all conditions are uniform over the workgroup
        step(kt, s0, 0);
        if (kt + 1 < nk) step(kt + 1, s1, 1);
        if (kt + 2 < nk) step(kt + 2, s2, 0);
        if (kt + 3 < nk) step(kt + 3, s3, 1);
    }

    // accumulator element e of a lane: row 8 * (e / 4) + 4 * (lane / 32) + e % 4, column lane % 32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + (wn * 2 + j) * 32 + lr;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int64_t m = m0 + (wm * 2 + i) * 32 + 8 * (e >> 2) + 4 * kg + (e & 3);
                if (m < g.M && n < g.N) {
                    float v = acc[i][j][e];
                    if (g.addend) v = g.addend[m * g.N + n] + v;
                    if (g.out_f32) reinterpret_cast<float *>(g.out)[m * g.N + n] = v;
                    else reinterpret_cast<uint16_t *>(g.out)[m * g.N + n] = (uint16_t)f32_to_bf16_bits(v);
                }
            }
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

}  // namespace

hipError_t launch_hp_gemm_nt(const void *A, const void *B, int64_t M, int64_t N, int64_t K, const float *addend, void *out,
                             int out_f32, hipStream_t st)
{
    if (M == 0 || N == 0) return hipSuccess;
    HpArgs g;
    g.A = static_cast<const uint16_t *>(A);
    g.B = static_cast<const uint16_t *>(B);
    g.addend = addend;
    g.out = out;
    g.M = M; g.N = N; g.K = K;
    g.out_f32 = out_f32;
    g.tiles_n = (int)((N + kBN - 1) / kBN);
    const int64_t tiles = ((M + kBM - 1) / kBM) * g.tiles_n;
    hipLaunchKernelGGL(hp_gemm_nt_kernel, dim3((unsigned)tiles), dim3(kThreads), 0, st, g);
    return hipGetLastError();
}

hipError_t launch_transpose_bf16(const void *src, void *dst, int64_t R, int64_t C, hipStream_t st)
{
    if (R == 0 || C == 0) return hipSuccess;
    const int tiles_c = (int)((C + 63) / 64);
    const int64_t tiles = ((R + 63) / 64) * tiles_c;
    hipLaunchKernelGGL(transpose_bf16_kernel, dim3((unsigned)tiles), dim3(kThreads), 0, st, static_cast<const uint16_t *>(src),
                       static_cast<uint16_t *>(dst), R, C, tiles_c);
    return hipGetLastError();
}

}  // namespace tj
