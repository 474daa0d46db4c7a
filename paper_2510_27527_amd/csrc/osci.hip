// OsciReset kernels (TetraJet-v2 Sec. 3.2-3.3: Alg. 1 OscillationSuppress; Appendix Alg. 2 UpdateOscillationStats)
// for one weight matrix of binary32 master weights [C x D].  Q(W) is the forward weight quantizer - groups of 16 along
// D, round-to-nearest, nearest-even E4M3 scales, 1 x 128 FP32 outer blocks - followed by the binary32 dequantization
// (P * S_block) * S_global.  Both kernels are elementwise streams: a lane owns 8 consecutive weights (two 128-bit
// loads per array), two lanes a group of 16, sixteen lanes an outer block; maxima travel by DPP.
#include "device_fmt.h"
#include "internal.h"

namespace tj {

namespace {

constexpr int kThreads = 256;

struct F8 { float v[8]; };

__device__ __forceinline__ F8 load8(const float *p)
{
    const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    return F8{{a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w}};
}
__device__ __forceinline__ void store8(float *p, const F8 &x)
{
    *reinterpret_cast<float4 *>(p) = make_float4(x.v[0], x.v[1], x.v[2], x.v[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(x.v[4], x.v[5], x.v[6], x.v[7]);
}

// Q(x) for the lane's 8 weights; all 16 lanes of the outer block must be active
__device__ __forceinline__ F8 quant_dequant8(const F8 &x, const float *inv_tab)
{
    uint32_t hm = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t ab = f2u(x.v[i]) & 0x7FFFFFFFu;
        hm = hm > ab ? hm : ab;
    }
    const uint32_t o1 = dpp<DPP_QUAD_XOR1>(hm);
    const uint32_t bm = hm > o1 ? hm : o1;                  // group of 16
    uint32_t gm = bm, t;
    t = dpp<DPP_QUAD_XOR2>(gm);       gm = gm > t ? gm : t;
    t = dpp<DPP_ROW_HALF_MIRROR>(gm); gm = gm > t ? gm : t;
    t = dpp<DPP_ROW_MIRROR>(gm);      gm = gm > t ? gm : t;  // outer block of 128
    const OuterScale os = outer_scale(u2f(gm));
    const uint32_t sc = e4m3_round<false>(u2f(bm) * os.inv_cg);
    const float r = os.inv_sg * inv_tab[sc];
    uint32_t codes = 0;
    codes = e2m1_rtn_pair<0>(codes, x.v[0] * r, x.v[1] * r);
    codes = e2m1_rtn_pair<1>(codes, x.v[2] * r, x.v[3] * r);
    codes = e2m1_rtn_pair<2>(codes, x.v[4] * r, x.v[5] * r);
    codes = e2m1_rtn_pair<3>(codes, x.v[6] * r, x.v[7] * r);
    const float sb = e4m3_value(sc);
    const float2_t p0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 0) * sb;   // exact: 6 significant bits
    const float2_t p1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 1) * sb;
    const float2_t p2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 2) * sb;
    const float2_t p3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 3) * sb;
    return F8{{p0.x * os.S_g, p0.y * os.S_g, p1.x * os.S_g, p1.y * os.S_g, p2.x * os.S_g, p2.y * os.S_g, p3.x * os.S_g,
               p3.y * os.S_g}};
}

// nchunks = C * D / 8 is a multiple of 16 (D % 128 == 0), so a 16-lane row is either whole or absent
__global__ __launch_bounds__(kThreads) void osci_update_kernel(const float *W, float *W_prev, float *dist_m, float *dist_q,
                                                               int64_t nchunks, int first)
{
    __shared__ float inv_tab[128];
    fill_inv_table(inv_tab);
    __syncthreads();
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (c >= nchunks) return;
    const int64_t e = c * 8;
    const F8 w = load8(W + e);
    if (first) {
        const F8 z{{0, 0, 0, 0, 0, 0, 0, 0}};
        store8(W_prev + e, w);
        store8(dist_m + e, z);
        store8(dist_q + e, z);
        return;
    }
    const F8 wp = load8(W_prev + e);
    F8 dm = load8(dist_m + e), dq = load8(dist_q + e);
    const F8 q = quant_dequant8(w, inv_tab), qp = quant_dequant8(wp, inv_tab);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        dm.v[i] = dm.v[i] + fabsf(w.v[i] - wp.v[i]);
        dq.v[i] = dq.v[i] + fabsf(q.v[i] - qp.v[i]);
    }
    store8(W_prev + e, w);
    store8(dist_m + e, dm);
    store8(dist_q + e, dq);
}

__global__ __launch_bounds__(kThreads) void osci_suppress_kernel(float *W, const float *dist_m, const float *dist_q, float tau,
                                                                 int64_t nchunks, unsigned long long *n_reset)
{
    __shared__ float inv_tab[128];
    __shared__ unsigned int wg_count;
    fill_inv_table(inv_tab);
    if (threadIdx.x == 0) wg_count = 0;
    __syncthreads();
    unsigned int mine = 0;
    // a workgroup walks over several chunks per thread: one atomic per workgroup at the end, and few workgroups
    const int64_t stride = (int64_t)gridDim.x * kThreads;      // a multiple of 16: rows of 16 lanes stay whole
    for (int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x; c < nchunks; c += stride) {
        const int64_t e = c * 8;
        F8 w = load8(W + e);
        const F8 dm = load8(dist_m + e), dq = load8(dist_q + e);
        const F8 q = quant_dequant8(w, inv_tab);
        unsigned int here = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float risk = dq.v[i] / dm.v[i];          // IEEE quotient; 0 / 0 is NaN and compares false
            if (risk >= tau) {
                w.v[i] = q.v[i];
                ++here;
            }
        }
        if (here) store8(W + e, w);
        mine += here;
    }
    if (n_reset) {
        for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
        if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&wg_count, mine);
        __syncthreads();
        if (threadIdx.x == 0 && wg_count) atomicAdd(n_reset, (unsigned long long)wg_count);
    }
}

}  // namespace

hipError_t launch_osci_update(const float *W, float *W_prev, float *dist_m, float *dist_q, int64_t n, int first, hipStream_t st)
{
    const int64_t nchunks = n / 8;
    if (nchunks == 0) return hipSuccess;
    const unsigned grid = (unsigned)((nchunks + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(osci_update_kernel, dim3(grid), dim3(kThreads), 0, st, W, W_prev, dist_m, dist_q, nchunks, first);
    return hipGetLastError();
}

hipError_t launch_osci_suppress(float *W, const float *dist_m, const float *dist_q, float tau, int64_t n,
                                unsigned long long *n_reset, hipStream_t st)
{
    const int64_t nchunks = n / 8;
    if (nchunks == 0) return hipSuccess;
    const int64_t want = (nchunks + kThreads - 1) / kThreads;
    const unsigned grid = (unsigned)(want < 4096 ? want : 4096);
    hipLaunchKernelGGL(osci_suppress_kernel, dim3(grid), dim3(kThreads), 0, st, W, dist_m, dist_q, tau, nchunks, n_reset);
    return hipGetLastError();
}

}  // namespace tj
