// Shared between the translation units of the NT GEMM: kernel arguments, the per-instantiation launch entry points
// and the bf16 rounding both the product kernel and the split-K reduction use.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_fmt.h"

namespace tj {

constexpr int kGemmThreads = 256;

struct GemmArgs {
    const uint8_t *a_codes, *a_scales;
    const uint8_t *b_codes, *b_scales;
    const float *a_gscale, *b_gscale;   // one float (tensor mode) or [rows][K/128] (block mode)
    void *out;          // bf16 / f32 [M x N], or f32 partials [split][M x N]
    int64_t M, N, K;
    int chunks_per_split;   // 64-wide K chunks per split
    int out_f32;
    int tiles_m, tiles_n;
    int outer;              // 0 one outer scale per operand, 1 one per row and 128 k
};

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f)
{
    const uint32_t b = f2u(f);
    return (b + 0x7FFFu + ((b >> 16) & 1u)) >> 16;
}

// One translation unit per (output kind, scale-fetch variant, outer mode) instantiates the product kernel for every
// tile shape: out 0 bf16, 1 f32, 2 raw f32 split-K partial; ps = paired scale fetch (K a multiple of 256); outer = 1:
// one FP32 outer scale per row and 128 k.  tile: 0 256x256 (outer 0 only), 1 256x128, 2 128x256, 3 128x128,
// 4 128x192 (ps only).
#define TJ_DECL_GEMM_INST(ps, out, outer) \
    hipError_t launch_gemm_inst_ps##ps##_out##out##_outer##outer(int tile, const GemmArgs &g, dim3 grid, hipStream_t st);
TJ_DECL_GEMM_INST(0, 0, 0) TJ_DECL_GEMM_INST(0, 1, 0) TJ_DECL_GEMM_INST(0, 2, 0)
TJ_DECL_GEMM_INST(1, 0, 0) TJ_DECL_GEMM_INST(1, 1, 0) TJ_DECL_GEMM_INST(1, 2, 0)
TJ_DECL_GEMM_INST(0, 0, 1) TJ_DECL_GEMM_INST(0, 1, 1) TJ_DECL_GEMM_INST(0, 2, 1)
TJ_DECL_GEMM_INST(1, 0, 1) TJ_DECL_GEMM_INST(1, 1, 1) TJ_DECL_GEMM_INST(1, 2, 1)
#undef TJ_DECL_GEMM_INST

}  // namespace tj
