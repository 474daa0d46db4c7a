// One (output kind, scale-fetch variant, outer mode) slice of the product kernel's instantiations; compiled once per
// slice with -DTJ_GEMM_PS=0|1 -DTJ_GEMM_OUT=0|1|2 -DTJ_GEMM_OUTER=0|1 so that the slices build in parallel.
#include "gemm_kernel.h"

#define TJ_CAT2(a, b, c, d, e, f) a##b##c##d##e##f
#define TJ_CAT(a, b, c, d, e, f) TJ_CAT2(a, b, c, d, e, f)

namespace tj {

hipError_t TJ_CAT(launch_gemm_inst_ps, TJ_GEMM_PS, _out, TJ_GEMM_OUT, _outer, TJ_GEMM_OUTER)(int tile, const GemmArgs &g, dim3 grid,
                                                                                         hipStream_t st)
{
    return launch_tile<TJ_GEMM_OUT, (TJ_GEMM_PS != 0), TJ_GEMM_OUTER>(tile, g, grid, st);
}

}  // namespace tj
