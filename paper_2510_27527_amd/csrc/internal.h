// Host-side launcher interfaces between the C-ABI layer (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tj {

constexpr int kMaxAmaxPartials = 512;   // floats of workspace one tensor-maximum reduction uses

struct QuantOut {
    uint8_t *codes;
    uint8_t *scales;
    float *gscale;
    float *amax_deq;   // may be null
};

struct QuantParams {
    int rounding;      // 0 RTN, 1 SR
    int scale_up;      // 0 nearest-even, 1 upward
    int outer;         // 0 tensor, 1 block128
    uint32_t k0, k1;   // stream key words
    int rht;           // 1: random Hadamard transform (block 16) along the grouped axis first; 1 x 128 outer blocks only
    uint32_t r0, r1;   // key words of the transform's sign stream
    // tensor maximum: either a device scalar, or `npart` partial maxima
    const float *amax_scalar;
    const float *amax_partials;
    int npart;
};

// view of an NVFP4 source tensor [R x C] (grouped along C)
struct PackedSrc {
    const uint8_t *codes;
    const uint8_t *scales;
    const float *gscale;
    int outer;
};

// partial maxima of |x| over a bf16 array of n elements (n % 8 == 0); returns the number of partials written;
// zero_me (optional) is a device float the kernel also clears
int launch_amax_partials(const void *src, int64_t n, float *partials, float *zero_me, hipStream_t st);
// the same for two arrays in one launch
void launch_amax_partials_pair(const void *src0, int64_t n0, float *partials0, float *zero0, int *npart0,
                               const void *src1, int64_t n1, float *partials1, float *zero1, int *npart1,
                               hipStream_t st);
// reduce partials to one scalar
void launch_amax_final(const float *partials, int npart, float *out, hipStream_t st);
// zero one float
void launch_zero_scalar(float *p, hipStream_t st);

// row-wise quantization of a bf16 [rows x K] array (groups along K)
hipError_t launch_quant_row_bf16(const void *src, int64_t rows, int64_t K, const QuantParams &p, const QuantOut &o,
                                 hipStream_t st);
// two such quantizations (same rounding mode, scale rounding and outer mode) in one launch
hipError_t launch_quant_row_bf16_pair(const void *src0, int64_t rows0, int64_t K0, const QuantParams &p0,
                                      const QuantOut &o0, const void *src1, int64_t rows1, int64_t K1,
                                      const QuantParams &p1, const QuantOut &o1, hipStream_t st);
// column-wise quantization of a bf16 [R x C] array: output [C x R] grouped along R
hipError_t launch_quant_col_bf16(const void *src, int64_t R, int64_t C, const QuantParams &p, const QuantOut &o,
                                 hipStream_t st);
// both at once from one read of a bf16 [R x C] array: row-wise [R x C] (prow / orow) and column-wise [C x R]
// (pcol / ocol); the two share rounding mode, scale rounding and the source of the tensor maximum
hipError_t launch_quant_dual_bf16(const void *src, int64_t R, int64_t C, const QuantParams &prow, const QuantOut &orow,
                                  const QuantParams &pcol, const QuantOut &ocol, hipStream_t st);
// column-wise re-quantization of an NVFP4 [R x C] tensor: output [C x R] grouped along R
hipError_t launch_requant_col(const PackedSrc &src, int64_t R, int64_t C, const QuantParams &p, const QuantOut &o,
                              hipStream_t st);

// two such re-quantizations (same rounding mode and scale rounding) in one launch
hipError_t launch_requant_col_pair(const PackedSrc &src0, int64_t R0, int64_t C0, const QuantParams &p0,
                                   const QuantOut &o0, const PackedSrc &src1, int64_t R1, int64_t C1,
                                   const QuantParams &p1, const QuantOut &o1, hipStream_t st);

struct GemmOperand {
    const uint8_t *codes;
    const uint8_t *scales;
    const float *gscale;   // one float, or [rows][K/128] floats
    int64_t rows;
    int outer;             // 0 tensor mode, 1 one outer scale per row and 128 k (both operands alike)
};

// Out[M x N] = A[M x K] * B[N x K]^T; splitk_ws holds split * M * N floats when split > 1
size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int outer);
// workgroup tile and K split the launcher will use for this shape
void gemm_plan(int64_t M, int64_t N, int64_t K, int outer, int *bm, int *bn, int *split);
hipError_t launch_gemm_nt(const GemmOperand &A, const GemmOperand &B, int64_t K, void *out, int out_f32,
                          void *ws, size_t ws_bytes, hipStream_t st);

// bf16 side of the OutControl split linear: Out[M x N] = addend (optional, f32) + A[M x K] * B[N x K]^T with K % 32 == 0;
// transpose of a bf16 [R x C] array
hipError_t launch_hp_gemm_nt(const void *A, const void *B, int64_t M, int64_t N, int64_t K, const float *addend, void *out,
                             int out_f32, hipStream_t st);
hipError_t launch_transpose_bf16(const void *src, void *dst, int64_t R, int64_t C, hipStream_t st);

// OsciReset on a binary32 weight matrix of n elements (rows of a multiple of 128): statistics step and reset
hipError_t launch_osci_update(const float *W, float *W_prev, float *dist_m, float *dist_q, int64_t n, int first, hipStream_t st);
hipError_t launch_osci_suppress(float *W, const float *dist_m, const float *dist_q, float tau, int64_t n,
                                unsigned long long *n_reset, hipStream_t st);
// Appendix Alg. 3 (the k weights closest to a rounding threshold): selection, update and reset on the tracked subset
size_t osci_select_workspace_bytes(int64_t n);
hipError_t launch_osci_select(const float *W, int64_t n, int64_t k, uint32_t *idx, float *wp, float *qp, float *dm, float *dq,
                              void *ws, hipStream_t st);
hipError_t launch_osci_update_sparse(const float *W, int64_t n, const uint32_t *idx, int64_t k, float *wp, float *qp, float *dm,
                                     float *dq, hipStream_t st);
hipError_t launch_osci_suppress_sparse(float *W, int64_t n, const uint32_t *idx, int64_t k, const float *dm, const float *dq,
                                       float tau, unsigned long long *n_reset, hipStream_t st);

uint64_t stream_key(uint64_t seed, uint32_t tensor_id);

}  // namespace tj
