// Host side of the NT GEMM on two packed NVFP4 operands (tile / split planner, launcher) and the split-K reduction.
// The product kernel itself lives in gemm_kernel.h and is instantiated slice by slice in gemm_inst.hip.
#include "gemm_args.h"
#include "internal.h"

namespace tj {

namespace {

constexpr int kThreads = kGemmThreads;
constexpr int kNC = 2;

// K = 0: the product is all zeros (no operand, and no outer scale, is looked at)
__global__ __launch_bounds__(kThreads) void zero_out_kernel(uint16_t *out, int64_t n16)
{
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += stride) out[i] = 0;
}

// partials are read exactly once: streaming load
__device__ __forceinline__ float4 ld4(const float *p)
{
    const float4_t v = __builtin_nontemporal_load(reinterpret_cast<const float4_t *>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

// sum the split-K partials in split order, scale, convert
__global__ __launch_bounds__(kThreads) void splitk_reduce_kernel(const float *__restrict__ part, int split,
                                                                 int64_t mn, const float *a_gscale,
                                                                 const float *b_gscale, int outer, void *out, int out_f32)
{
    // block mode: the partial sums already carry the outer scales
    const float alpha = outer ? 256.0f : a_gscale[0] * b_gscale[0] * 256.0f;
    const int64_t i4 = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (i4 >= mn) return;
    if ((mn & 3) == 0) {
        float4 s = ld4(part + i4);
        for (int z = 1; z < split; ++z) {
            const float4 t = ld4(part + (int64_t)z * mn + i4);
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

// Tile shapes and a small cost model (microseconds, from timings of this kernel on MI355X) that picks
// the tile and the number of K splits for a problem.
struct TileCfg { int tm, tn; double t_stage; double t_fixed; int occupancy; };
// t_stage: one 128-k pipeline stage of one workgroup with the CU to itself; t_fixed: prologue + epilogue
// the 128 x 192 tile exists for the paired scale fetch only (K a multiple of 256)
const TileCfg kTiles[] = {{4, 4, 3.2, 6.0, 1}, {4, 2, 2.0, 5.0, 1}, {2, 4, 2.0, 5.0, 1}, {2, 2, 1.5, 5.0, 3}, {2, 3, 1.4, 5.0, 2}};
constexpr int kNumTiles = 5;
constexpr int kNumCU = 256;

struct Plan { int tile; int split; int chunks_per_split; };

Plan make_plan(int64_t M, int64_t N, int64_t K, int outer)
{
    const int64_t chunks = K / 64;
    Plan best{3, 1, (int)chunks};
    if (M <= 0 || N <= 0 || chunks == 0) return best;      // nothing to tile (empty output or empty reduction)
    double best_t = 1e300;
    for (int t = 0; t < kNumTiles; ++t) {
        if (t == 4 && K % 256 != 0) continue;
        if (t == 0 && outer) continue;                      // block mode keeps two accumulator sets: at most 2 x 4 tiles per wave
        const int64_t bm = 64 * kTiles[t].tm, bn = 64 * kTiles[t].tn;
        const int64_t tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
        for (int split = 1; split <= 16; ++split) {
            if (split > 1 && chunks / split < 8) break;
            int64_t cps = (chunks + split - 1) / split;
            if (chunks % 4 == 0) cps = (cps + 3) / 4 * 4;                       // splits on 256-k boundaries
            else if (outer) cps = (cps + 1) / 2 * 2;                            // block mode: on 128-k boundaries
            if (split > 1 && (chunks + cps - 1) / cps != split) continue;      // same launch as a smaller split
            const int64_t wgs = tiles * split;
            const double stages = (double)((cps + kNC - 1) / kNC);
            // workgroups sharing a CU slow each other down (128 x 128 tiles: up to three per CU)
            const int64_t per_cu = (wgs + kNumCU - 1) / kNumCU;
            const int64_t conc = per_cu < kTiles[t].occupancy ? per_cu : kTiles[t].occupancy;
            const double slow = conc == 1 ? 1.0 : conc == 2 ? 1.75 : 2.35;
            const int64_t waves = (wgs + kNumCU * conc - 1) / (kNumCU * conc);
            // block mode: the per-block rescale of the accumulators makes a stage about a third longer
            double time = (double)waves * (stages * kTiles[t].t_stage * (outer ? 1.35 : 1.0) * slow + kTiles[t].t_fixed);
            if (split > 1) time += 4.0 + (double)(split + 1) * (double)(M * N) * 4.0 / 3.5e6;   // partials out and back in
            if (time < best_t) { best_t = time; best = Plan{t, split, (int)cps}; }
        }
    }
    return best;
}

}  // namespace

void gemm_plan(int64_t M, int64_t N, int64_t K, int outer, int *bm, int *bn, int *split)
{
    const Plan p = make_plan(M, N, K, outer);
    *bm = 64 * kTiles[p.tile].tm;
    *bn = 64 * kTiles[p.tile].tn;
    *split = p.split;
}

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int outer)
{
    const Plan p = make_plan(M, N, K, outer);
    return p.split > 1 ? (size_t)p.split * (size_t)M * (size_t)N * sizeof(float) : 0;
}

hipError_t launch_gemm_nt(const GemmOperand &A, const GemmOperand &B, int64_t K, void *out, int out_f32,
                          void *ws, size_t ws_bytes, hipStream_t st)
{
    const int64_t M = A.rows, N = B.rows;
    if (M == 0 || N == 0) return hipSuccess;
    if (K == 0) {
        const int64_t n16 = M * N * (out_f32 ? 2 : 1);
        const int64_t want = (n16 + kThreads - 1) / kThreads;
        hipLaunchKernelGGL(zero_out_kernel, dim3((unsigned)(want > 4096 ? 4096 : want)), dim3(kThreads), 0, st,
                           static_cast<uint16_t *>(out), n16);
        return hipGetLastError();
    }
    const int outer = A.outer;
    Plan p = make_plan(M, N, K, outer);
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
    g.outer = outer;
    const int64_t chunks = K / 64;
    const int split = p.split > 1 ? (int)((chunks + p.chunks_per_split - 1) / p.chunks_per_split) : 1;
    g.out = split > 1 ? ws : out;
    dim3 grid((unsigned)(g.tiles_m * g.tiles_n), 1, (unsigned)split);
    // K a multiple of 256 with splits on 256-boundaries: scale bytes are fetched 16 per row
    const bool ps = K % 256 == 0 && p.chunks_per_split % 4 == 0;
    typedef hipError_t (*InstFn)(int, const GemmArgs &, dim3, hipStream_t);
    static const InstFn inst[2][2][3] = {
        {{launch_gemm_inst_ps0_out0_outer0, launch_gemm_inst_ps0_out1_outer0, launch_gemm_inst_ps0_out2_outer0},
         {launch_gemm_inst_ps1_out0_outer0, launch_gemm_inst_ps1_out1_outer0, launch_gemm_inst_ps1_out2_outer0}},
        {{launch_gemm_inst_ps0_out0_outer1, launch_gemm_inst_ps0_out1_outer1, launch_gemm_inst_ps0_out2_outer1},
         {launch_gemm_inst_ps1_out0_outer1, launch_gemm_inst_ps1_out1_outer1, launch_gemm_inst_ps1_out2_outer1}}};
    hipError_t e = inst[outer ? 1 : 0][ps ? 1 : 0][split > 1 ? 2 : (out_f32 ? 1 : 0)](p.tile, g, grid, st);
    if (e != hipSuccess) return e;
    if (split > 1) {
        const int64_t mn = M * N;
        const unsigned rgrid = (unsigned)((mn + (int64_t)kThreads * 4 - 1) / ((int64_t)kThreads * 4));
        hipLaunchKernelGGL(splitk_reduce_kernel, dim3(rgrid), dim3(kThreads), 0, st,
                           reinterpret_cast<const float *>(ws), split, mn, A.gscale, B.gscale, outer, out, out_f32);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace tj
