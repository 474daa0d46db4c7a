// One (output kind, scale-fetch variant) slice of the product kernel's instantiations; compiled once per slice with
// -DTJ_GEMM_PS=0|1 -DTJ_GEMM_OUT=0|1|2 so that the slices build in parallel.
#include "gemm_kernel.h"

#define TJ_CAT2(a, b, c, d) a##b##c##d
#define TJ_CAT(a, b, c, d) TJ_CAT2(a, b, c, d)

namespace tj {

hipError_t TJ_CAT(launch_gemm_inst_ps, TJ_GEMM_PS, _out, TJ_GEMM_OUT)(int tile, const GemmArgs &g, dim3 grid, hipStream_t st)
{
    return launch_tile<TJ_GEMM_OUT, (TJ_GEMM_PS != 0)>(tile, g, grid, st);
}

}  // namespace tj
