// OsciReset kernels (TetraJet-v2 Sec. 3.2-3.3: Alg. 1 OscillationSuppress; Appendix Alg. 2 UpdateOscillationStats and
// Alg. 3, its memory-efficient form that tracks only the k weights closest to a rounding threshold)
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

// Q(x) for the lane's 8 weights; all 16 lanes of the outer block must be active.  SCORE: also the sensitivity score of
// Appendix Alg. 3, |x - Q(x)| / binwidth(Q(x)), binwidth = (length of the interval of scaled values that round to the
// code's magnitude) * RN(S_block * S_global); 0 in a block whose scale is 0.
template <bool SCORE>
__device__ __forceinline__ F8 quant_dequant8_t(const F8 &x, const float *inv_tab, F8 *score)
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
    const F8 q{{p0.x * os.S_g, p0.y * os.S_g, p1.x * os.S_g, p1.y * os.S_g, p2.x * os.S_g, p2.y * os.S_g, p3.x * os.S_g,
                p3.y * os.S_g}};
    if (SCORE) {
        const float unit = sb * os.S_g;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t m = (codes >> (4 * i)) & 7u;
            const float bin = m < 4 ? 0.5f : m == 4 ? 0.75f : m == 6 ? 1.5f : 1.0f;
            const float width = bin * unit;
            const float num = fabsf(x.v[i] - q.v[i]);
            score->v[i] = width == 0.0f ? 0.0f : num / width;
        }
    }
    return q;
}
__device__ __forceinline__ F8 quant_dequant8(const F8 &x, const float *inv_tab) { return quant_dequant8_t<false>(x, inv_tab, nullptr); }

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

// ---- Appendix Alg. 3: selection of the k largest sensitivity scores (equal scores in ascending index order) ----------
//
// Scores are non-negative binary32 values, so they order like their bit patterns.  The k-th largest pattern is found by
// a three-digit radix search (11 + 11 + 10 bits: a histogram pass over the tensor and a pick per digit); the tensor is
// then compacted in index order: a count of (greater, equal) per 2048-element tile, an exclusive scan over the tiles,
// and a pass that ranks every selected element and writes its index and the states of the tracked subset.  Every pass
// recomputes Q(W) (the scores are never stored: the point of the algorithm is to keep no per-element state).
constexpr int kTile = kThreads * 8;

struct SelState {
    uint32_t prefix;      // the digits of the threshold found so far
    uint32_t kneed;       // how many elements are still to be taken among those that match the prefix
    uint32_t thr;         // after the third digit: the k-th largest score (bit pattern)
    uint32_t ties;        // elements equal to thr that belong to the selection (the first ones in index order)
};

__global__ __launch_bounds__(kThreads) void osci_zero_kernel(uint32_t *p, int n)
{
    for (int i = blockIdx.x * kThreads + threadIdx.x; i < n; i += gridDim.x * kThreads) p[i] = 0;
}

template <int PASS>
__global__ __launch_bounds__(kThreads) void osci_hist_kernel(const float *W, int64_t nchunks, const SelState *st, uint32_t *hist)
{
    __shared__ float inv_tab[128];
    __shared__ uint32_t bins[2048];
    fill_inv_table(inv_tab);
    for (int b = threadIdx.x; b < 2048; b += kThreads) bins[b] = 0;
    __syncthreads();
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (c < nchunks) {                                    // whole rows of 16 lanes (nchunks is a multiple of 16)
        const F8 w = load8(W + c * 8);
        F8 sc;
        quant_dequant8_t<true>(w, inv_tab, &sc);
        const uint32_t prefix = PASS == 0 ? 0u : st->prefix;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t b = f2u(sc.v[i]);
            if (PASS == 0) atomicAdd(&bins[b >> 21], 1u);
            else if (PASS == 1) { if ((b >> 21) == prefix) atomicAdd(&bins[(b >> 10) & 2047u], 1u); }
            else { if ((b >> 10) == prefix) atomicAdd(&bins[b & 1023u], 1u); }
        }
    }
    __syncthreads();
    for (int b = threadIdx.x; b < 2048; b += kThreads)
        if (bins[b]) atomicAdd(&hist[b], bins[b]);
}

// one workgroup: the digit whose bin holds the kneed-th largest element; clears the histogram for the next pass
template <int PASS>
__global__ __launch_bounds__(kThreads) void osci_pick_kernel(SelState *st, uint32_t *hist, uint32_t k_total)
{
    __shared__ uint32_t bins[2048];
    for (int b = threadIdx.x; b < 2048; b += kThreads) {
        bins[b] = hist[b];
        hist[b] = 0;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t kneed = PASS == 0 ? k_total : st->kneed;
        uint32_t above = 0;
        int digit = 0;
        for (int b = (PASS == 2 ? 1023 : 2047); b >= 0; --b) {
            if (above + bins[b] >= kneed) { digit = b; break; }
            above += bins[b];
        }
        const uint32_t prefix = PASS == 0 ? (uint32_t)digit : (st->prefix << (PASS == 1 ? 11 : 10)) | (uint32_t)digit;
        st->prefix = prefix;
        st->kneed = kneed - above;
        if (PASS == 2) {
            st->thr = prefix;
            st->ties = kneed - above;
        }
    }
}

// flags of the lane's 8 elements against the threshold: bit i of gt / eq
__device__ __forceinline__ void score_flags(const F8 &sc, uint32_t thr, uint32_t &gt, uint32_t &eq)
{
    gt = eq = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t b = f2u(sc.v[i]);
        gt |= (b > thr ? 1u : 0u) << i;
        eq |= (b == thr ? 1u : 0u) << i;
    }
}

__global__ __launch_bounds__(kThreads) void osci_count_kernel(const float *W, int64_t nchunks, const SelState *st, uint32_t *counts)
{
    __shared__ float inv_tab[128];
    __shared__ uint32_t tot[2];
    fill_inv_table(inv_tab);
    if (threadIdx.x < 2) tot[threadIdx.x] = 0;
    __syncthreads();
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    uint32_t ngt = 0, neq = 0;
    if (c < nchunks) {
        F8 sc;
        quant_dequant8_t<true>(load8(W + c * 8), inv_tab, &sc);
        uint32_t gt, eq;
        score_flags(sc, st->thr, gt, eq);
        ngt = __builtin_popcount(gt);
        neq = __builtin_popcount(eq);
    }
    for (int o = 32; o > 0; o >>= 1) {
        ngt += __shfl_xor(ngt, o, 64);
        neq += __shfl_xor(neq, o, 64);
    }
    if ((threadIdx.x & 63) == 0) {
        atomicAdd(&tot[0], ngt);
        atomicAdd(&tot[1], neq);
    }
    __syncthreads();
    if (threadIdx.x < 2) counts[2 * blockIdx.x + threadIdx.x] = tot[threadIdx.x];
}

// exclusive prefix sums of the per-tile (greater, equal) counts, in place; one workgroup
__global__ __launch_bounds__(kThreads) void osci_scan_kernel(uint32_t *counts, int64_t ntiles)
{
    __shared__ uint32_t part[kThreads][2];
    const int64_t per = (ntiles + kThreads - 1) / kThreads;
    const int64_t lo = per * threadIdx.x, hi = lo + per < ntiles ? lo + per : ntiles;
    uint32_t a = 0, b = 0;
    for (int64_t t = lo; t < hi; ++t) {
        a += counts[2 * t];
        b += counts[2 * t + 1];
    }
    part[threadIdx.x][0] = a;
    part[threadIdx.x][1] = b;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t ra = 0, rb = 0;
        for (int t = 0; t < kThreads; ++t) {
            const uint32_t va = part[t][0], vb = part[t][1];
            part[t][0] = ra;
            part[t][1] = rb;
            ra += va;
            rb += vb;
        }
    }
    __syncthreads();
    a = part[threadIdx.x][0];
    b = part[threadIdx.x][1];
    for (int64_t t = lo; t < hi; ++t) {
        const uint32_t va = counts[2 * t], vb = counts[2 * t + 1];
        counts[2 * t] = a;
        counts[2 * t + 1] = b;
        a += va;
        b += vb;
    }
}

// exclusive prefix sum of v over the workgroup's 256 threads (thread order); red: 4 words of LDS
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t *red)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = v;
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    __syncthreads();                                       // the previous use of red is over
    if (lane == 63) red[wave] = incl;
    __syncthreads();
    uint32_t base = 0;
    for (int w = 0; w < wave; ++w) base += red[w];
    return base + incl - v;
}

__global__ __launch_bounds__(kThreads) void osci_emit_kernel(const float *W, int64_t nchunks, const SelState *st, const uint32_t *offs,
                                                             uint32_t *idx, float *wp, float *qp, float *dm, float *dq)
{
    __shared__ float inv_tab[128];
    __shared__ uint32_t red[4];
    fill_inv_table(inv_tab);
    __syncthreads();
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const uint32_t thr = st->thr, ties = st->ties;
    F8 w{{0, 0, 0, 0, 0, 0, 0, 0}}, q = w;
    uint32_t gt = 0, eq = 0;
    if (c < nchunks) {
        w = load8(W + c * 8);
        F8 sc;
        q = quant_dequant8_t<true>(w, inv_tab, &sc);
        score_flags(sc, thr, gt, eq);
    }
    // equal elements are ranked in index order over the whole tensor; the first `ties` of them are selected
    const uint32_t eq_tiles = offs[2 * blockIdx.x + 1], gt_tiles = offs[2 * blockIdx.x];
    const uint32_t eq_before = eq_tiles + block_exclusive_scan(__builtin_popcount(eq), red);
    uint32_t sel = gt, rank = eq_before;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if ((eq >> i) & 1u) {
            if (rank < ties) sel |= 1u << i;
            ++rank;
        }
    const uint32_t taken_eq_tiles = eq_tiles < ties ? eq_tiles : ties;       // selected equal elements of earlier tiles
    uint32_t pos = gt_tiles + taken_eq_tiles + block_exclusive_scan(__builtin_popcount(sel), red);
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if ((sel >> i) & 1u) {
            idx[pos] = (uint32_t)(c * 8 + i);
            wp[pos] = w.v[i];
            qp[pos] = q.v[i];
            dm[pos] = 0.0f;
            dq[pos] = 0.0f;
            ++pos;
        }
}

// first position j in the ascending list idx[0..k) with idx[j] >= e
__device__ __forceinline__ int64_t lower_bound_u32(const uint32_t *idx, int64_t k, int64_t e)
{
    int64_t lo = 0, hi = k;
    while (lo < hi) {
        const int64_t mid = (lo + hi) >> 1;
        if ((int64_t)idx[mid] < e) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// Alg. 3 at a later step (SUPPRESS = false) and Alg. 1 on the tracked subset (SUPPRESS = true).  A workgroup takes a
// tile of 2048 consecutive weights: Q of the tile goes to LDS, then the tile's entries of the (ascending) index list -
// found by binary search - are updated from it.  Tiles without a tracked element stop after the search.
template <bool SUPPRESS>
__global__ __launch_bounds__(kThreads) void osci_sparse_kernel(float *W, int64_t nchunks, const uint32_t *idx, int64_t k, float *wp,
                                                               float *qp, float *dm, float *dq, float tau,
                                                               unsigned long long *n_reset)
{
    __shared__ float inv_tab[128];
    __shared__ float qt[kTile];
    __shared__ int64_t range[2];
    __shared__ unsigned int wg_count;
    const int64_t tile0 = (int64_t)blockIdx.x * kTile;
    fill_inv_table(inv_tab);
    if (threadIdx.x == 0) {
        range[0] = lower_bound_u32(idx, k, tile0);
        range[1] = lower_bound_u32(idx, k, tile0 + kTile);
        wg_count = 0;
    }
    __syncthreads();
    const int64_t j0 = range[0], j1 = range[1];
    if (j0 == j1) return;                                  // uniform
    const int64_t c = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (c < nchunks) {
        const F8 q = quant_dequant8(load8(W + c * 8), inv_tab);
#pragma unroll
        for (int i = 0; i < 8; ++i) qt[threadIdx.x * 8 + i] = q.v[i];
    }
    __syncthreads();                                       // every weight of the tile has been read: resets may follow
    unsigned int mine = 0;
    for (int64_t j = j0 + threadIdx.x; j < j1; j += kThreads) {
        const int64_t e = idx[j];
        const float q = qt[e - tile0];
        if (SUPPRESS) {
            const float risk = dq[j] / dm[j];              // IEEE quotient; 0 / 0 is NaN and compares false
            if (risk >= tau) {
                W[e] = q;
                ++mine;
            }
        } else {
            const float w = W[e];
            dm[j] = dm[j] + fabsf(w - wp[j]);
            dq[j] = dq[j] + fabsf(q - qp[j]);
            wp[j] = w;
            qp[j] = q;
        }
    }
    if (SUPPRESS && n_reset) {
        for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
        if ((threadIdx.x & 63) == 0 && mine) atomicAdd(&wg_count, mine);
        __syncthreads();
        if (threadIdx.x == 0 && wg_count) atomicAdd(n_reset, (unsigned long long)wg_count);
    }
}

}  // namespace

size_t osci_select_workspace_bytes(int64_t n)
{
    const int64_t ntiles = (n + kTile - 1) / kTile;
    return 256 + 2048 * sizeof(uint32_t) + (size_t)ntiles * 2 * sizeof(uint32_t);
}

hipError_t launch_osci_select(const float *W, int64_t n, int64_t k, uint32_t *idx, float *wp, float *qp, float *dm, float *dq,
                              void *ws, hipStream_t st)
{
    const int64_t nchunks = n / 8;
    if (nchunks == 0 || k == 0) return hipSuccess;
    SelState *state = static_cast<SelState *>(ws);
    uint32_t *hist = reinterpret_cast<uint32_t *>(static_cast<uint8_t *>(ws) + 256);
    uint32_t *counts = hist + 2048;
    const unsigned grid = (unsigned)((nchunks + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(osci_zero_kernel, dim3(8), dim3(kThreads), 0, st, hist, 2048);
    hipLaunchKernelGGL(osci_hist_kernel<0>, dim3(grid), dim3(kThreads), 0, st, W, nchunks, state, hist);
    hipLaunchKernelGGL(osci_pick_kernel<0>, dim3(1), dim3(kThreads), 0, st, state, hist, (uint32_t)k);
    hipLaunchKernelGGL(osci_hist_kernel<1>, dim3(grid), dim3(kThreads), 0, st, W, nchunks, state, hist);
    hipLaunchKernelGGL(osci_pick_kernel<1>, dim3(1), dim3(kThreads), 0, st, state, hist, (uint32_t)k);
    hipLaunchKernelGGL(osci_hist_kernel<2>, dim3(grid), dim3(kThreads), 0, st, W, nchunks, state, hist);
    hipLaunchKernelGGL(osci_pick_kernel<2>, dim3(1), dim3(kThreads), 0, st, state, hist, (uint32_t)k);
    hipLaunchKernelGGL(osci_count_kernel, dim3(grid), dim3(kThreads), 0, st, W, nchunks, state, counts);
    hipLaunchKernelGGL(osci_scan_kernel, dim3(1), dim3(kThreads), 0, st, counts, (int64_t)grid);
    hipLaunchKernelGGL(osci_emit_kernel, dim3(grid), dim3(kThreads), 0, st, W, nchunks, state, counts, idx, wp, qp, dm, dq);
    return hipGetLastError();
}

hipError_t launch_osci_update_sparse(const float *W, int64_t n, const uint32_t *idx, int64_t k, float *wp, float *qp, float *dm,
                                     float *dq, hipStream_t st)
{
    const int64_t nchunks = n / 8;
    if (nchunks == 0 || k == 0) return hipSuccess;
    const unsigned grid = (unsigned)((nchunks + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(osci_sparse_kernel<false>, dim3(grid), dim3(kThreads), 0, st, const_cast<float *>(W), nchunks, idx, k, wp, qp,
                       dm, dq, 0.0f, static_cast<unsigned long long *>(nullptr));
    return hipGetLastError();
}

hipError_t launch_osci_suppress_sparse(float *W, int64_t n, const uint32_t *idx, int64_t k, const float *dm, const float *dq,
                                       float tau, unsigned long long *n_reset, hipStream_t st)
{
    const int64_t nchunks = n / 8;
    if (nchunks == 0 || k == 0) return hipSuccess;
    const unsigned grid = (unsigned)((nchunks + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(osci_sparse_kernel<true>, dim3(grid), dim3(kThreads), 0, st, W, nchunks, idx, k, static_cast<float *>(nullptr),
                       static_cast<float *>(nullptr), const_cast<float *>(dm), const_cast<float *>(dq), tau, n_reset);
    return hipGetLastError();
}

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
