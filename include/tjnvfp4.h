/*
 * tjnvfp4 - NVFP4 fully-quantized linear layer for AMD MI355X (gfx950), C ABI.
 *
 * The operations are those of TetraJet-v2 (arXiv 2510.27527):
 *   Sec. 2.1  E2M1 elements, groups of 16 sharing one E4M3 scale, deterministic
 *             (nearest) and stochastic rounding;
 *   Sec. 2.2  double-block scaling: an FP32 outer scale S_global over an outer
 *             group (the whole tensor, or 128 consecutive elements) and an E4M3
 *             inner scale S_block per 16 elements;
 *   Sec. 2.3  the quantized linear layer
 *               Y  = Q1_D(X)    x Q2_D(W^T)
 *               dX = Q3_S(dY)   x Q4_S(W_hat)
 *               dW = Q5_S(dY^T) x Q6_S(X_hat)
 *             with X [N x D], W [C x D], Y, dY [N x C]; every operand is grouped
 *             along the reduction axis of its product.
 *
 * Conventions
 *   - Every data pointer is DEVICE memory owned by the caller, 16-byte aligned.
 *     The library allocates nothing, frees nothing and never synchronises: each
 *     call validates its arguments on the host, then enqueues kernels on
 *     `stream` (a hipStream_t passed as void*, NULL = default stream) and returns.
 *     Its only state is the per-device address of a static scratch array
 *     (nvfp4_gemm_nt_static), looked up under a lock.
 *   - Descriptor structs (nvfp4_tensor, nvfp4_qcfg) are HOST memory, read during
 *     the call only.
 *   - Return value: 0 on success, a negative NVFP4_ERR_* otherwise; on error
 *     nothing has been enqueued unless the code is NVFP4_ERR_HIP.
 *   - `ws` is a scratch buffer of at least nvfp4_workspace_bytes(...) bytes that
 *     must stay untouched until the enqueued work has finished.  Two calls that
 *     overlap in time need different workspaces.
 *
 * Storage of a quantized operand (K = grouped, contiguous axis, K % 16 == 0):
 *   codes  [rows][K/2]   two E2M1 codes per byte, element 2j in the low nibble;
 *                        code = sign<<3 | index into {0,.5,1,1.5,2,3,4,6}
 *   scales [rows][K/16]  E4M3 (bias 7, no infinity, max 448 = 0x7E), row-major
 *   gscale               FP32 outer scale(s): [1] (NVFP4_OUTER_TENSOR) or
 *                        [rows][K/128] (NVFP4_OUTER_BLOCK128)
 *   value(r,k) = E2M1(code) * E4M3(scales[r][k/16]) * gscale[...]
 *
 * Empty inputs (a size of 0) are accepted everywhere: nothing is launched for an empty tensor, an empty product is
 * skipped, and a product over an empty reduction (K = 0) is written as zeros.  Device pointers of empty tensors are
 * never dereferenced but must still be non-NULL and 16-byte aligned.
 */
#ifndef TJNVFP4_H
#define TJNVFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    NVFP4_OK = 0,
    NVFP4_ERR_NULL = -1,      /* a required pointer is NULL */
    NVFP4_ERR_SHAPE = -2,     /* negative size; grouped axis K % 16 != 0 (K % 128 != 0 in BLOCK128 mode); more than 2^33
                                 elements; C % 8 != 0 for a column-wise bf16 source; for the products: reduction
                                 length not a multiple of 64 or above 2^22 */
    NVFP4_ERR_ENUM = -3,      /* unknown enum value, or a combination this build does not provide */
    NVFP4_ERR_WORKSPACE = -4, /* ws is NULL or smaller than nvfp4_workspace_bytes() */
    NVFP4_ERR_ALIGN = -5,     /* a device pointer is not 16-byte aligned */
    NVFP4_ERR_MISMATCH = -6,  /* operand descriptors disagree with each other or with N, D, C */
    NVFP4_ERR_HIP = -7,       /* a HIP launch failed; see hipGetLastError() */
    NVFP4_ERR_SCRATCH = -8    /* nvfp4_gemm_nt_static: the product needs more than NVFP4_STATIC_SCRATCH_BYTES */
};

/* Size of the library's static device scratch array (one per GPU, held from the first use of
 * nvfp4_gemm_nt_static on that GPU until the process ends). */
#define NVFP4_STATIC_SCRATCH_BYTES (64u << 20)

enum { NVFP4_ROUND_RTN = 0, NVFP4_ROUND_SR = 1 };                 /* Sec. 2.1: deterministic / stochastic   */
enum { NVFP4_SCALE_DEFAULT = 0, NVFP4_SCALE_NE = 1, NVFP4_SCALE_UP = 2 }; /* E4M3 rounding of S_block; DEFAULT = NE for RTN, UP for SR */
enum { NVFP4_OUTER_TENSOR = 0, NVFP4_OUTER_BLOCK128 = 1 };       /* Sec. 2.2 outer group: tensor / 1x128   */
enum { NVFP4_SRC_BF16 = 0, NVFP4_SRC_NVFP4 = 1 };                 /* source kind of nvfp4_quantize         */
enum { NVFP4_OUT_BF16 = 0, NVFP4_OUT_F32 = 1 };                   /* output element type of the products   */
enum { NVFP4_OP_QUANTIZE = 0, NVFP4_OP_GEMM = 1, NVFP4_OP_LINEAR_FWD = 2,
       NVFP4_OP_LINEAR_BWD_DX = 3, NVFP4_OP_LINEAR_BWD_DW = 4, NVFP4_OP_LINEAR_BWD = 5 };

/* One quantized operand.  The caller fills the four pointers with buffers of the
 * sizes given above; the producing call fills rows, K and outer_mode. */
typedef struct nvfp4_tensor {
    uint8_t *codes;      /* device */
    uint8_t *scales;     /* device */
    float   *gscale;     /* device */
    float   *amax_deq;   /* device [1], optional (may be NULL): receives max |value| over the tensor, rounded to
                            FP32; needed when the operand is later re-quantized in TENSOR mode (Q4, Q6) */
    int64_t  rows, K;
    int32_t  outer_mode;
    int32_t  reserved;
} nvfp4_tensor;

/* Parameters of one quantization. */
typedef struct nvfp4_qcfg {
    int32_t  rounding;     /* NVFP4_ROUND_*  */
    int32_t  scale_round;  /* NVFP4_SCALE_*  */
    int32_t  outer_mode;   /* NVFP4_OUTER_*  */
    uint32_t tensor_id;    /* stochastic rounding: stream id; the random bits of output element e (index in the
                              output's own [rows x K] view) depend only on (seed, tensor_id, e) */
    uint64_t seed;
    const float *amax_in;  /* device [1], optional, TENSOR mode: max |src| if the caller already has it */
    int32_t  rht;          /* 1: random Hadamard transform of Sec. 4.1 first: every aligned run of 16 along the grouped
                              axis is multiplied by S H_16 (random signs, then the 16 x 16 Hadamard matrix), and the
                              result is what gets quantized.  Provided with NVFP4_OUTER_BLOCK128 (ENUM otherwise). */
    uint32_t rht_id;       /* stream id of the signs: sign of position k along the grouped axis depends only on
                              (seed, rht_id, k); the two operands of a product must use the same */
} nvfp4_qcfg;

/*
 * Quantize (Sec. 2.1-2.2).  src is a bf16 [R x C] row-major device array (NVFP4_SRC_BF16) or a HOST pointer to an
 * nvfp4_tensor describing an [R x C] operand (NVFP4_SRC_NVFP4, re-quantization of Sec. 2.3's X_hat / W_hat, which
 * starts from the FP32 value code*scale*gscale; axis 1 only; the source may be in either outer mode).
 * axis 0: groups run along C, out describes [R x C] (K = C).
 * axis 1: groups run along R (16 x 1 groups), out describes the transpose [C x R] (K = R); a bf16 source needs
 * C % 8 == 0.  cfg->outer_mode is the outer group of the OUTPUT: the whole tensor, or 128 consecutive elements of
 * its K axis (then K % 128 == 0 and no maximum is needed: the call is a single pass over src).
 * In TENSOR mode the tensor maximum is taken from cfg->amax_in, else from src->amax_deq (NVFP4 source), else by a
 * reduction pass over src.  Errors: NULL, SHAPE, ENUM, WORKSPACE, ALIGN, MISMATCH.
 */
int nvfp4_quantize(const void *src, int src_kind, int64_t R, int64_t C, int axis,
                   const nvfp4_qcfg *cfg, nvfp4_tensor *out, void *ws, size_t ws_bytes, void *stream);

/*
 * Both backward operands of one bf16 [R x C] tensor from a single read of it (Sec. 2.3: Q3 and Q5 both act on dY):
 * out_row describes [R x C] grouped along C (what axis 0 of nvfp4_quantize gives, stream id cfg->tensor_id), out_col
 * the transpose [C x R] grouped along R (axis 1, stream id tensor_id_col).  Rounding, scale rounding, seed and
 * maximum are cfg's and shared; TENSOR outer mode only; R and C multiples of 16.  Every byte equals that of the two
 * separate calls.  ws as for nvfp4_quantize (needed when cfg->amax_in is NULL).
 */
int nvfp4_quantize_dual(const void *src, int64_t R, int64_t C, const nvfp4_qcfg *cfg, uint32_t tensor_id_col,
                        nvfp4_tensor *out_row, nvfp4_tensor *out_col, void *ws, size_t ws_bytes, void *stream);

/*
 * Out[M x N] = A[M x K] * B[N x K]^T on two quantized operands grouped along K (Sec. 2.3: all three products take
 * this form).  Products of dequantized 16-bit values are exact; accumulation is FP32; the outer scales multiply
 * the accumulator at the end (TENSOR mode), or - with the paper's 1 x 128 outer blocks - the sum over each 128-k
 * block is multiplied by the two blocks' FP32 scales before it joins the total; Out is row-major bf16 or f32.  Both
 * operands must be in the same outer mode (MISMATCH otherwise).
 * Limits: A->K == B->K, K % 64 == 0 (K % 128 == 0 in BLOCK128 mode) and K <= 2^22 (SHAPE otherwise); any M = A->rows,
 * N = B->rows.  ws: at least
 * nvfp4_workspace_bytes(NVFP4_OP_GEMM, M, K, N, 0) bytes (0 for most shapes; FP32 partial sums when the planner
 * splits the reduction).  Errors: NULL, SHAPE, ENUM, WORKSPACE, ALIGN, MISMATCH.
 */
int nvfp4_gemm_nt(const nvfp4_tensor *A, const nvfp4_tensor *B, void *Out, int out_dtype,
                  void *ws, size_t ws_bytes, void *stream);

/*
 * nvfp4_gemm_nt for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same kernels and the same bytes
 * in Out as nvfp4_gemm_nt, but the scratch memory a split reduction needs (FP32 partial sums) is a static device array
 * of NVFP4_STATIC_SCRATCH_BYTES inside the library; the call allocates and frees nothing (the array's address is
 * looked up once per device on the first call there).  A product whose nvfp4_workspace_bytes(NVFP4_OP_GEMM, ..)
 * exceeds the array returns NVFP4_ERR_SCRATCH and enqueues nothing.  Every call on one GPU uses that GPU's one array:
 * calls that overlap in time on a GPU (two streams, two threads) race on it; calls on one stream are safe.  Nothing
 * in the array has to be zero at entry (every partial sum that is read has been written by the same call).
 */
int nvfp4_gemm_nt_static(const nvfp4_tensor *A, const nvfp4_tensor *B, void *Out, int out_dtype, void *stream);

/*
 * Forward (Sec. 2.3, first line): quantizes X [N x D] and W [C x D] (bf16, round-to-nearest, groups along D) into
 * Xq_ctx / Wq_ctx, which the caller keeps for the backward calls, and writes Y [N x C].
 * outer_mode: outer group of both operands (NVFP4_OUTER_TENSOR: two maximum passes precede the quantizers;
 * NVFP4_OUTER_BLOCK128: the paper's 1 x 128 blocks, single pass).  The backward calls follow the contexts' mode.
 * Limits: D % 64 == 0 (D % 128 == 0 in BLOCK128 mode) and D <= 2^22 (D is the reduction length); any N, C.  X, W, Y
 * 16-byte aligned.
 */
int nvfp4_linear_fwd(const void *X, const void *W, int64_t N, int64_t D, int64_t C,
                     void *Y, int out_dtype, nvfp4_tensor *Xq_ctx, nvfp4_tensor *Wq_ctx,
                     int outer_mode, void *ws, size_t ws_bytes, void *stream);

/*
 * Input gradient (Sec. 2.3, second line): dX [N x D] = Q3_S(dY) x Q4_S(W_hat); dY [N x C] bf16, W_hat = Wq_ctx of
 * the forward call, both re-grouped along C with stochastic rounding.  Streams: tensor ids layer_id*16+3 and +4.
 * rht = 1 (Sec. 4.1 / 4.2; contexts with 1 x 128 outer blocks only): both operands are first transformed along C,
 * dX = Q3(dY S H) x Q4(H^T S^T W_hat), signs of stream layer_id*16+7.
 */
int nvfp4_linear_bwd_dx(const void *dY, const nvfp4_tensor *Wq_ctx, int64_t N, int64_t D, int64_t C,
                        void *dX, int out_dtype, uint64_t seed, uint32_t layer_id, int rht,
                        void *ws, size_t ws_bytes, void *stream);

/*
 * Weight gradient (Sec. 2.3, third line): dW [C x D] = Q5_S(dY^T) x Q6_S(X_hat); both operands re-grouped along N
 * with stochastic rounding.  Streams: tensor ids layer_id*16+5 and +6.  rht = 1: both operands are first transformed
 * along N, dW = Q5(dY^T S H) x Q6(H^T S^T X_hat), signs of stream layer_id*16+8.
 * Limits: N % 64 == 0 (N % 128 == 0 in BLOCK128 mode) and N <= 2^22 (reduction length); C % 8 == 0; D % 16 == 0.
 */
int nvfp4_linear_bwd_dw(const void *dY, const nvfp4_tensor *Xq_ctx, int64_t N, int64_t D, int64_t C,
                        void *dW, int out_dtype, uint64_t seed, uint32_t layer_id, int rht,
                        void *ws, size_t ws_bytes, void *stream);

/*
 * Both gradients of one layer in one call (Sec. 2.3, second and third line).  Same results, byte for byte, as
 * nvfp4_linear_bwd_dx followed by nvfp4_linear_bwd_dw with the same seed and layer_id, but dY is read once for its
 * maximum and once more for both of its quantizations (Q3 row-wise and Q5 column-wise leave one kernel).
 * Limits: C % 64 == 0, N % 64 == 0 (% 128 in BLOCK128 mode), both <= 2^22 (each is the reduction length of one
 * product); D % 16 == 0.  In BLOCK128 mode dY is read once per operand (no maximum pass, no fused quantizer).
 */
int nvfp4_linear_bwd(const void *dY, const nvfp4_tensor *Xq_ctx, const nvfp4_tensor *Wq_ctx,
                     int64_t N, int64_t D, int64_t C, void *dX, void *dW, int out_dtype,
                     uint64_t seed, uint32_t layer_id, int rht, void *ws, size_t ws_bytes, void *stream);

/*
 * OutControl split linear (Sec. 4.2): a static set A of outlier channels of the activation stays in high precision
 * (bf16 here), the rest runs in NVFP4.  Because the set is fixed once, the caller keeps the two column sets as separate
 * row-major bf16 tensors: X_lo [N x D_lo], W_lo [C x D_lo] (ordinary channels) and X_hp [N x D_hp], W_hp [C x D_hp]
 * (outlier channels; D_hp % 32 == 0, may be 0).
 *   forward:  Y = Q1(X_lo) x Q2(W_lo^T) + X_hp x W_hp^T  (the second product on the bf16 matrix path, FP32 accumulate;
 *             the sum is formed in FP32 and rounded once to out_dtype).  Xq_ctx / Wq_ctx describe the ordinary channels.
 *   backward: dX = Q3(dY) x Q4(W_hat) over ALL input channels in NVFP4: dX_lo [N x D_lo] from the re-quantized context,
 *             dX_hp [N x D_hp] from W_hp quantized column-wise (stream id layer_id*16+9), both against one Q3 operand;
 *             dW_lo [C x D_lo] = Q5(dY^T) x Q6(X_hat_lo) in NVFP4; dW_hp [C x D_hp] = dY^T x X_hp in bf16.
 *             rht as in nvfp4_linear_bwd (on the four NVFP4 operands and on Q4 of W_hp).  With per-tensor outer scales
 *             W_hat's two column sets each get a scale of their own; with 1 x 128 outer blocks (the paper's setting) the
 *             split changes nothing, every output row of Q4 being scaled by itself.
 * ws: nvfp4_outctl_workspace_bytes(backward, ...).  Limits as for nvfp4_linear_fwd / nvfp4_linear_bwd with D = D_lo.
 */
int nvfp4_outctl_fwd(const void *X_lo, const void *W_lo, const void *X_hp, const void *W_hp, int64_t N, int64_t D_lo,
                     int64_t D_hp, int64_t C, void *Y, int out_dtype, nvfp4_tensor *Xq_ctx, nvfp4_tensor *Wq_ctx,
                     int outer_mode, void *ws, size_t ws_bytes, void *stream);
int nvfp4_outctl_bwd(const void *dY, const nvfp4_tensor *Xq_ctx, const nvfp4_tensor *Wq_ctx, const void *X_hp,
                     const void *W_hp, int64_t N, int64_t D_lo, int64_t D_hp, int64_t C, void *dX_lo, void *dX_hp,
                     void *dW_lo, void *dW_hp, int out_dtype, uint64_t seed, uint32_t layer_id, int rht, void *ws,
                     size_t ws_bytes, void *stream);
size_t nvfp4_outctl_workspace_bytes(int backward, int64_t N, int64_t D_lo, int64_t D_hp, int64_t C, int outer_mode,
                                    int out_dtype);

/*
 * OsciReset (Sec. 3.2-3.3) for one weight matrix of binary32 master weights W [C x D], all arrays device memory of
 * C * D floats, 16-byte aligned, D % 128 == 0.  Q(W) below is the forward weight quantizer (groups of 16 along D,
 * round-to-nearest, 1 x 128 outer blocks) followed by dequantization to binary32.
 *
 * nvfp4_osci_update - Appendix Alg. 2 (UpdateOscillationStats), one step of a tracking period.  t0 == 0 opens the
 *   period: dist_m = dist_q = 0 and the snapshot W_prev = W.  t0 > 0: dist_m += |W - W_prev|,
 *   dist_q += |Q(W) - Q(W_prev)|, then W_prev = W.  One pass, 28 bytes of traffic per weight.
 * nvfp4_osci_suppress - Alg. 1 (OscillationSuppress): every element whose risk dist_q / dist_m reaches tau (the paper
 *   uses 8) is reset to the centre of its quantization bin, W = Q(W) there; elements that never moved (0 / 0) are kept.
 *   n_reset (device, optional, 8-byte aligned) is increased by the number of elements reset; the caller clears it.
 * Errors: NULL, SHAPE, ENUM (t0 < 0, tau <= 0), ALIGN.
 */
int nvfp4_osci_update(const float *W, float *W_prev, float *dist_m, float *dist_q, int64_t C, int64_t D, int t0,
                      void *stream);
int nvfp4_osci_suppress(float *W, const float *dist_m, const float *dist_q, float tau, int64_t C, int64_t D,
                        unsigned long long *n_reset, void *stream);

/*
 * The memory-efficient statistics of Appendix Alg. 3: only the k weights closest to a rounding threshold are tracked
 * (the paper tracks the top 5 % of the sensitivity score s = |W - Q(W)| / binwidth(Q(W)); the caller passes
 * k = ceil(p * C * D)).  binwidth = (length of the interval of scaled values that round to the element's FP4 magnitude:
 * 0.5 for 0 .. 1.5, 0.75 for 2, 1 for 3, 1.5 for 4, 1 for 6) * S_block * S_global; equal scores are taken in ascending
 * index order.  State of the subset, all device arrays of k entries owned by the caller: idx (flat indices into W,
 * ascending), W_prev_s / Q_prev_s (master / quantized snapshots), dist_m_s / dist_q_s.  C * D <= 2^31, D % 128 == 0,
 * W 16-byte aligned.
 *
 * nvfp4_osci_select - first step of a period (t0 = 0): finds the k largest scores, writes idx, the two snapshots and
 *   zero distances.  ws: nvfp4_osci_select_workspace_bytes(C, D) bytes, 16-byte aligned.  Ten launches, five reads of W.
 * nvfp4_osci_update_sparse - a later step: dist_m_s += |W[idx] - W_prev_s|, dist_q_s += |Q(W)[idx] - Q_prev_s|, then
 *   the snapshots are replaced.
 * nvfp4_osci_suppress_sparse - Alg. 1 on the subset: W[idx[j]] = Q(W)[idx[j]] where dist_q_s[j] / dist_m_s[j] >= tau;
 *   n_reset as in nvfp4_osci_suppress.
 * With k = C * D the three calls compute exactly what nvfp4_osci_update / nvfp4_osci_suppress compute.
 * Errors: NULL, SHAPE (also k < 0, k > C * D, C * D > 2^31), ENUM (tau <= 0), ALIGN, WORKSPACE.
 */
size_t nvfp4_osci_select_workspace_bytes(int64_t C, int64_t D);
int nvfp4_osci_select(const float *W, int64_t C, int64_t D, int64_t k, uint32_t *idx, float *W_prev_s, float *Q_prev_s,
                      float *dist_m_s, float *dist_q_s, void *ws, size_t ws_bytes, void *stream);
int nvfp4_osci_update_sparse(const float *W, int64_t C, int64_t D, const uint32_t *idx, int64_t k, float *W_prev_s,
                             float *Q_prev_s, float *dist_m_s, float *dist_q_s, void *stream);
int nvfp4_osci_suppress_sparse(float *W, int64_t C, int64_t D, const uint32_t *idx, int64_t k, const float *dist_m_s,
                               const float *dist_q_s, float tau, unsigned long long *n_reset, void *stream);

/*
 * Scratch bytes an operation needs.  op = NVFP4_OP_*.  QUANTIZE: (N, D) = (R, C) of the source, C ignored.
 * GEMM: Out is [N x C] with reduction length D.  LINEAR_*: as in the calls above.  Returns 0 for a bad op.
 */
size_t nvfp4_workspace_bytes(int op, int64_t N, int64_t D, int64_t C, int outer_mode);

/* Launch configuration nvfp4_gemm_nt uses for an [M x K] * [N x K]^T product of operands in outer_mode: workgroup tile (rows x columns of the
 * output) and the number of K splits (> 1 means FP32 partials in ws plus a reduction kernel).  Host-only helper. */
int nvfp4_gemm_plan(int64_t M, int64_t N, int64_t K, int outer_mode, int *tile_m, int *tile_n, int *split);

/* Tensor maximum of |x| of a bf16 device array of n elements (n % 8 == 0) into amax_out (device [1]): the max |X| of
 * Sec. 2.2's S_global = max |X| / (448 * 6) for a per-tensor outer group.  ws: nvfp4_workspace_bytes(NVFP4_OP_QUANTIZE, ..). */
int nvfp4_amax_bf16(const void *src, int64_t n, float *amax_out, void *ws, size_t ws_bytes, void *stream);

/* The 64-bit stream key the stochastic-rounding generator derives from (seed, tensor_id); host-only helper. */
uint64_t nvfp4_stream_key(uint64_t seed, uint32_t tensor_id);

const char *nvfp4_strerror(int code);

/* "tjnvfp4 <version> gfx950" */
const char *nvfp4_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TJNVFP4_H */
