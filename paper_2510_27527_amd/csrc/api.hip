// C-ABI layer of tjnvfp4: host-side argument validation, workspace carving and the composition
// of the kernels into the four calls of the NVFP4 linear layer (TetraJet-v2 Sec. 2.3).
// Validation happens before the first HIP call, so every error path can be exercised on a
// machine without a GPU.
#include <mutex>

#include "../../include/tjnvfp4.h"
#include "internal.h"

// Scratch memory of the entry point that allocates nothing (nvfp4_gemm_nt_static): one copy per GPU, at an address
// of its own on each, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and copies get the address that call returns.
constexpr size_t kStaticScratchBytes = (size_t)NVFP4_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace tj {

// (seed, tensor id) -> 64-bit stream key; low word k0, high word k1
static uint64_t mix64(uint64_t z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

uint64_t stream_key(uint64_t seed, uint32_t tensor_id)
{
    const uint64_t a = mix64(seed + 0x9E3779B97F4A7C15ull);
    const uint64_t b = ((uint64_t)tensor_id + 1ull) * 0xD1B54A32D192ED03ull;
    return mix64(a ^ b);
}

namespace {

constexpr size_t kAlign = 256;
constexpr int64_t kMaxElems = (int64_t)1 << 33;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// sequential carving of the caller's workspace
struct Carver {
    uint8_t *base;
    size_t size, used;
    void *take(size_t bytes)
    {
        const size_t off = used;
        used += align_up(bytes);
        return (base && used <= size) ? base + off : nullptr;
    }
};

size_t partials_bytes() { return align_up(sizeof(float) * kMaxAmaxPartials); }
size_t gscale_bytes(int64_t rows, int64_t K, int outer)
{
    return outer == NVFP4_OUTER_BLOCK128 ? sizeof(float) * (size_t)(rows * (K / 128)) : sizeof(float);
}
size_t packed_bytes(int64_t rows, int64_t K, int outer)
{
    return align_up((size_t)(rows * K / 2)) + align_up((size_t)(rows * K / 16)) + align_up(gscale_bytes(rows, K, outer));
}
bool valid_outer(int outer) { return outer == NVFP4_OUTER_TENSOR || outer == NVFP4_OUTER_BLOCK128; }

int check_shape(int64_t rows, int64_t K, int outer)
{
    if (rows < 0 || K < 0) return NVFP4_ERR_SHAPE;
    if (K % 16 != 0) return NVFP4_ERR_SHAPE;
    if (outer == NVFP4_OUTER_BLOCK128 && K % 128 != 0) return NVFP4_ERR_SHAPE;
    if (rows > 0 && K > kMaxElems / rows) return NVFP4_ERR_SHAPE;
    return NVFP4_OK;
}

int check_tensor_ptrs(const nvfp4_tensor *t)
{
    if (!t || !t->codes || !t->scales || !t->gscale) return NVFP4_ERR_NULL;
    if (!aligned16(t->codes) || !aligned16(t->scales) || (reinterpret_cast<uintptr_t>(t->gscale) & 3u))
        return NVFP4_ERR_ALIGN;
    if (t->amax_deq && (reinterpret_cast<uintptr_t>(t->amax_deq) & 3u)) return NVFP4_ERR_ALIGN;
    return NVFP4_OK;
}

// reduction length of a product: whole 64-wide chunks, and short enough for the kernel's 32-bit per-lane offsets
// (row-in-tile * K / 2 + piece offset, row-in-tile <= 255)
constexpr int64_t kMaxReduction = (int64_t)1 << 22;
int check_reduction(int64_t K) { return (K % 64 != 0 || K > kMaxReduction) ? NVFP4_ERR_SHAPE : NVFP4_OK; }

// a gemm operand must be a finished operand with K % 64 == 0 (K % 128 == 0 with 1 x 128 outer blocks)
int check_gemm_operand(const nvfp4_tensor *t)
{
    int rc = check_tensor_ptrs(t);
    if (rc) return rc;
    if (!valid_outer(t->outer_mode)) return NVFP4_ERR_ENUM;
    rc = check_shape(t->rows, t->K, t->outer_mode);
    if (rc) return rc;
    return check_reduction(t->K);
}

struct QuantPlan {
    int src_kind, axis;
    int64_t R, C;
    int64_t out_rows, out_K;
    int rounding, scale_up, outer, rht;
    bool need_partials;
};

int plan_quantize(const void *src, int src_kind, int64_t R, int64_t C, int axis, const nvfp4_qcfg *cfg,
                  const nvfp4_tensor *out, QuantPlan *pl)
{
    if (!src || !cfg || !out) return NVFP4_ERR_NULL;
    if (src_kind != NVFP4_SRC_BF16 && src_kind != NVFP4_SRC_NVFP4) return NVFP4_ERR_ENUM;
    if (axis != 0 && axis != 1) return NVFP4_ERR_ENUM;
    if (cfg->rounding != NVFP4_ROUND_RTN && cfg->rounding != NVFP4_ROUND_SR) return NVFP4_ERR_ENUM;
    if (cfg->scale_round < NVFP4_SCALE_DEFAULT || cfg->scale_round > NVFP4_SCALE_UP) return NVFP4_ERR_ENUM;
    if (cfg->outer_mode != NVFP4_OUTER_TENSOR && cfg->outer_mode != NVFP4_OUTER_BLOCK128) return NVFP4_ERR_ENUM;
    if (R < 0 || C < 0) return NVFP4_ERR_SHAPE;
    pl->src_kind = src_kind;
    pl->axis = axis;
    pl->R = R;
    pl->C = C;
    pl->out_rows = axis == 0 ? R : C;
    pl->out_K = axis == 0 ? C : R;
    pl->rounding = cfg->rounding;
    pl->scale_up = cfg->scale_round == NVFP4_SCALE_DEFAULT ? (cfg->rounding == NVFP4_ROUND_SR)
                                                           : (cfg->scale_round == NVFP4_SCALE_UP);
    pl->outer = cfg->outer_mode;
    pl->rht = cfg->rht;
    if (cfg->rht != 0 && cfg->rht != 1) return NVFP4_ERR_ENUM;
    if (cfg->rht && pl->outer != NVFP4_OUTER_BLOCK128) return NVFP4_ERR_ENUM;   // the transform comes with 1 x 128 outer blocks
    int rc = check_shape(pl->out_rows, pl->out_K, pl->outer);
    if (rc) return rc;
    rc = check_tensor_ptrs(out);
    if (rc) return rc;
    if (cfg->amax_in && (reinterpret_cast<uintptr_t>(cfg->amax_in) & 3u)) return NVFP4_ERR_ALIGN;
    if (src_kind == NVFP4_SRC_BF16) {
        if (!aligned16(src)) return NVFP4_ERR_ALIGN;
        if (axis == 1 && C % 8 != 0) return NVFP4_ERR_SHAPE;           // 128-bit loads along C
        pl->need_partials = pl->outer == NVFP4_OUTER_TENSOR && cfg->amax_in == nullptr;
    } else {
        const nvfp4_tensor *s = static_cast<const nvfp4_tensor *>(src);
        rc = check_tensor_ptrs(s);
        if (rc) return rc;
        if (s->rows != R || s->K != C) return NVFP4_ERR_MISMATCH;
        rc = check_shape(R, C, s->outer_mode);
        if (rc) return rc;
        // provided: a packed source re-grouped along its other axis (Q4, Q6), in either outer mode on either side
        if (axis != 1) return NVFP4_ERR_ENUM;
        if (s->outer_mode != NVFP4_OUTER_TENSOR && s->outer_mode != NVFP4_OUTER_BLOCK128) return NVFP4_ERR_ENUM;
        if (pl->outer == NVFP4_OUTER_TENSOR && !cfg->amax_in && !s->amax_deq) return NVFP4_ERR_NULL;
        pl->need_partials = false;
    }
    return NVFP4_OK;
}

void set_rht(QuantParams &p, const QuantPlan &pl, const nvfp4_qcfg *cfg)
{
    p.rht = pl.rht;
    const uint64_t key = stream_key(cfg->seed, cfg->rht_id);
    p.r0 = (uint32_t)key;
    p.r1 = (uint32_t)(key >> 32);
}

int run_quantize(const void *src, const QuantPlan &pl, const nvfp4_qcfg *cfg, nvfp4_tensor *out, float *partials,
                 hipStream_t st)
{
    QuantParams p{};
    p.rounding = pl.rounding;
    p.scale_up = pl.scale_up ? 1 : 0;
    p.outer = pl.outer;
    const uint64_t key = stream_key(cfg->seed, cfg->tensor_id);
    p.k0 = (uint32_t)key;
    p.k1 = (uint32_t)(key >> 32);
    set_rht(p, pl, cfg);
    QuantOut o{out->codes, out->scales, out->gscale, out->amax_deq};
    out->rows = pl.out_rows;
    out->K = pl.out_K;
    out->outer_mode = pl.outer;
    if (pl.out_rows == 0 || pl.out_K == 0) return NVFP4_OK;
    hipError_t e;
    if (pl.src_kind == NVFP4_SRC_BF16) {
        if (pl.rounding != NVFP4_ROUND_RTN || pl.rht) o.amax_deq = nullptr;   // only forward operands are re-quantized
        bool zeroed = o.amax_deq == nullptr;
        if (pl.outer == NVFP4_OUTER_TENSOR) {
            if (cfg->amax_in) {
                p.amax_scalar = cfg->amax_in;
            } else {
                p.npart = launch_amax_partials(src, pl.R * pl.C, partials, o.amax_deq, st);
                p.amax_partials = partials;
                zeroed = true;
                if (pl.axis == 1 && pl.R * pl.C >= ((int64_t)1 << 23)) {
                    // many small workgroups follow: one more tiny launch is cheaper than each of them reducing the
                    // partials (the result may overwrite the first partial: it is written after all are read)
                    launch_amax_final(partials, p.npart, partials, st);
                    p.amax_scalar = partials;
                    p.amax_partials = nullptr;
                    p.npart = 0;
                }
            }
        }
        if (!zeroed) launch_zero_scalar(o.amax_deq, st);
        e = pl.axis == 0 ? launch_quant_row_bf16(src, pl.R, pl.C, p, o, st)
                         : launch_quant_col_bf16(src, pl.R, pl.C, p, o, st);
    } else {
        const nvfp4_tensor *s = static_cast<const nvfp4_tensor *>(src);
        p.amax_scalar = pl.outer == NVFP4_OUTER_TENSOR ? (cfg->amax_in ? cfg->amax_in : s->amax_deq) : nullptr;
        o.amax_deq = nullptr;
        PackedSrc ps{s->codes, s->scales, s->gscale, s->outer_mode};
        e = launch_requant_col(ps, pl.R, pl.C, p, o, st);
    }
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

QuantParams params_of(const QuantPlan &pl, const nvfp4_qcfg *cfg)
{
    QuantParams p{};
    p.rounding = pl.rounding;
    p.scale_up = pl.scale_up ? 1 : 0;
    p.outer = pl.outer;
    const uint64_t key = stream_key(cfg->seed, cfg->tensor_id);
    p.k0 = (uint32_t)key;
    p.k1 = (uint32_t)(key >> 32);
    set_rht(p, pl, cfg);
    return p;
}

void stamp(nvfp4_tensor *out, const QuantPlan &pl)
{
    out->rows = pl.out_rows;
    out->K = pl.out_K;
    out->outer_mode = pl.outer;
}

// Two row-wise tensor-mode quantizations of bf16 sources with the same settings (the two operands of a forward
// call): one launch for both maxima, one for both quantizations.
int run_quantize_row_pair(const void *src0, const QuantPlan &pl0, nvfp4_tensor *out0, float *partials0, const void *src1,
                          const QuantPlan &pl1, nvfp4_tensor *out1, float *partials1, const nvfp4_qcfg *cfg,
                          hipStream_t st)
{
    const bool pairable = pl0.src_kind == NVFP4_SRC_BF16 && pl1.src_kind == NVFP4_SRC_BF16 && pl0.axis == 0 &&
                          pl1.axis == 0 && pl0.outer == pl1.outer && cfg->amax_in == nullptr && pl0.R * pl0.C > 0 &&
                          pl1.R * pl1.C > 0;
    if (!pairable) {
        const int rc = run_quantize(src0, pl0, cfg, out0, partials0, st);
        return rc ? rc : run_quantize(src1, pl1, cfg, out1, partials1, st);
    }
    QuantParams p0 = params_of(pl0, cfg), p1 = params_of(pl1, cfg);
    QuantOut o0{out0->codes, out0->scales, out0->gscale, out0->amax_deq};
    QuantOut o1{out1->codes, out1->scales, out1->gscale, out1->amax_deq};
    if (pl0.rounding != NVFP4_ROUND_RTN) o0.amax_deq = o1.amax_deq = nullptr;
    stamp(out0, pl0);
    stamp(out1, pl1);
    if (pl0.outer == NVFP4_OUTER_TENSOR) {
        launch_amax_partials_pair(src0, pl0.R * pl0.C, partials0, o0.amax_deq, &p0.npart, src1, pl1.R * pl1.C, partials1,
                                  o1.amax_deq, &p1.npart, st);
        p0.amax_partials = partials0;
        p1.amax_partials = partials1;
    } else {
        // 1 x 128 outer blocks: no maximum pass; the dequantized maximum (an atomic maximum over the workgroups) is
        // only wanted by a later tensor-mode re-quantization and starts from zero
        if (o0.amax_deq) launch_zero_scalar(o0.amax_deq, st);
        if (o1.amax_deq) launch_zero_scalar(o1.amax_deq, st);
    }
    const hipError_t e = launch_quant_row_bf16_pair(src0, pl0.R, pl0.C, p0, o0, src1, pl1.R, pl1.C, p1, o1, st);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

// Two column-wise re-quantizations of packed tensors (Q4 and Q6 of one backward call) in one launch.
int run_requant_pair(const nvfp4_tensor *s0, const QuantPlan &pl0, const nvfp4_qcfg *c0, nvfp4_tensor *out0,
                     const nvfp4_tensor *s1, const QuantPlan &pl1, const nvfp4_qcfg *c1, nvfp4_tensor *out1,
                     hipStream_t st)
{
    QuantParams p0 = params_of(pl0, c0), p1 = params_of(pl1, c1);
    p0.amax_scalar = pl0.outer == NVFP4_OUTER_TENSOR ? (c0->amax_in ? c0->amax_in : s0->amax_deq) : nullptr;
    p1.amax_scalar = pl1.outer == NVFP4_OUTER_TENSOR ? (c1->amax_in ? c1->amax_in : s1->amax_deq) : nullptr;
    if (p0.rounding != p1.rounding || p0.scale_up != p1.scale_up || p0.outer != p1.outer || p0.rht != p1.rht) {
        const int rc = run_quantize(s0, pl0, c0, out0, nullptr, st);
        return rc ? rc : run_quantize(s1, pl1, c1, out1, nullptr, st);
    }
    stamp(out0, pl0);
    stamp(out1, pl1);
    QuantOut o0{out0->codes, out0->scales, out0->gscale, nullptr}, o1{out1->codes, out1->scales, out1->gscale, nullptr};
    PackedSrc ps0{s0->codes, s0->scales, s0->gscale, s0->outer_mode}, ps1{s1->codes, s1->scales, s1->gscale, s1->outer_mode};
    const hipError_t e = launch_requant_col_pair(ps0, pl0.R, pl0.C, p0, o0, ps1, pl1.R, pl1.C, p1, o1, st);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int run_gemm(const nvfp4_tensor *A, const nvfp4_tensor *B, void *Out, int out_dtype, void *ws, size_t ws_bytes,
             hipStream_t st)
{
    const int outer = A->outer_mode == NVFP4_OUTER_BLOCK128 ? 1 : 0;
    GemmOperand a{A->codes, A->scales, A->gscale, A->rows, outer};
    GemmOperand b{B->codes, B->scales, B->gscale, B->rows, outer};
    const hipError_t e = launch_gemm_nt(a, b, A->K, Out, out_dtype == NVFP4_OUT_F32, ws, ws_bytes, st);
    return e == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int check_out(const void *p, int out_dtype)
{
    if (!p) return NVFP4_ERR_NULL;
    if (out_dtype != NVFP4_OUT_BF16 && out_dtype != NVFP4_OUT_F32) return NVFP4_ERR_ENUM;
    if (!aligned16(p)) return NVFP4_ERR_ALIGN;
    return NVFP4_OK;
}

// device address of the static scratch array on the current device, looked up once per device
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return NVFP4_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return NVFP4_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return NVFP4_OK;
}

// carve a temporary operand [rows x K] out of the workspace
bool carve_tensor(Carver &cv, int64_t rows, int64_t K, int outer, nvfp4_tensor *t)
{
    t->codes = static_cast<uint8_t *>(cv.take((size_t)(rows * K / 2)));
    t->scales = static_cast<uint8_t *>(cv.take((size_t)(rows * K / 16)));
    t->gscale = static_cast<float *>(cv.take(gscale_bytes(rows, K, outer)));
    t->amax_deq = nullptr;
    t->rows = rows;
    t->K = K;
    t->outer_mode = outer;
    t->reserved = 0;
    return t->codes && t->scales && t->gscale;
}

}  // namespace
}  // namespace tj

using namespace tj;

extern "C" {

const char *nvfp4_strerror(int code)
{
    switch (code) {
        case NVFP4_OK: return "ok";
        case NVFP4_ERR_NULL: return "a required pointer is NULL";
        case NVFP4_ERR_SHAPE: return "bad shape (negative, grouped axis not a multiple of 16/64/128, or too large)";
        case NVFP4_ERR_ENUM: return "unknown enum value or unsupported combination";
        case NVFP4_ERR_WORKSPACE: return "workspace missing or too small";
        case NVFP4_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case NVFP4_ERR_MISMATCH: return "operand descriptors disagree";
        case NVFP4_ERR_HIP: return "HIP launch failed";
        case NVFP4_ERR_SCRATCH: return "the product needs more scratch memory than the library's static array holds";
        default: return "unknown error code";
    }
}

const char *nvfp4_version(void) { return "tjnvfp4 0.1 gfx950"; }

uint64_t nvfp4_stream_key(uint64_t seed, uint32_t tensor_id) { return stream_key(seed, tensor_id); }

size_t nvfp4_workspace_bytes(int op, int64_t N, int64_t D, int64_t C, int outer_mode)
{
    if (N < 0 || D < 0 || C < 0 || !valid_outer(outer_mode)) return 0;
    const int o = outer_mode;
    switch (op) {
        case NVFP4_OP_QUANTIZE: return partials_bytes();
        case NVFP4_OP_GEMM: return align_up(gemm_workspace_bytes(N, C, D, o));
        case NVFP4_OP_LINEAR_FWD: return 2 * partials_bytes() + align_up(gemm_workspace_bytes(N, C, D, o));
        case NVFP4_OP_LINEAR_BWD_DX:
            return partials_bytes() + packed_bytes(N, C, o) + packed_bytes(D, C, o) + align_up(gemm_workspace_bytes(N, D, C, o));
        case NVFP4_OP_LINEAR_BWD_DW:
            return partials_bytes() + packed_bytes(C, N, o) + packed_bytes(D, N, o) + align_up(gemm_workspace_bytes(C, D, N, o));
        case NVFP4_OP_LINEAR_BWD: {
            const size_t g1 = align_up(gemm_workspace_bytes(N, D, C, o)), g2 = align_up(gemm_workspace_bytes(C, D, N, o));
            return partials_bytes() + align_up(sizeof(float)) + packed_bytes(N, C, o) + packed_bytes(D, C, o) +
                   packed_bytes(C, N, o) + packed_bytes(D, N, o) + (g1 > g2 ? g1 : g2);
        }
        default: return 0;
    }
}

int nvfp4_gemm_plan(int64_t M, int64_t N, int64_t K, int outer_mode, int *tile_m, int *tile_n, int *split)
{
    if (!tile_m || !tile_n || !split) return NVFP4_ERR_NULL;
    if (!valid_outer(outer_mode)) return NVFP4_ERR_ENUM;
    if (M < 0 || N < 0 || K < 0 || K % 64 != 0) return NVFP4_ERR_SHAPE;
    if (outer_mode == NVFP4_OUTER_BLOCK128 && K % 128 != 0) return NVFP4_ERR_SHAPE;
    gemm_plan(M, N, K, outer_mode, tile_m, tile_n, split);
    return NVFP4_OK;
}

int nvfp4_amax_bf16(const void *src, int64_t n, float *amax_out, void *ws, size_t ws_bytes, void *stream)
{
    if (!src || !amax_out) return NVFP4_ERR_NULL;
    if (n < 0 || n % 8 != 0) return NVFP4_ERR_SHAPE;
    if (!aligned16(src)) return NVFP4_ERR_ALIGN;
    if (!ws || ws_bytes < partials_bytes()) return NVFP4_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int npart = launch_amax_partials(src, n, static_cast<float *>(ws), nullptr, st);
    launch_amax_final(static_cast<float *>(ws), npart, amax_out, st);
    return hipGetLastError() == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_quantize(const void *src, int src_kind, int64_t R, int64_t C, int axis, const nvfp4_qcfg *cfg,
                   nvfp4_tensor *out, void *ws, size_t ws_bytes, void *stream)
{
    QuantPlan pl{};
    const int rc = plan_quantize(src, src_kind, R, C, axis, cfg, out, &pl);
    if (rc) return rc;
    if (pl.need_partials && (!ws || ws_bytes < partials_bytes())) return NVFP4_ERR_WORKSPACE;
    if (ws && !aligned16(ws)) return NVFP4_ERR_ALIGN;
    return run_quantize(src, pl, cfg, out, static_cast<float *>(ws), static_cast<hipStream_t>(stream));
}

int nvfp4_quantize_dual(const void *src, int64_t R, int64_t C, const nvfp4_qcfg *cfg, uint32_t tensor_id_col,
                        nvfp4_tensor *out_row, nvfp4_tensor *out_col, void *ws, size_t ws_bytes, void *stream)
{
    if (!cfg) return NVFP4_ERR_NULL;
    if (cfg->outer_mode != NVFP4_OUTER_TENSOR) return NVFP4_ERR_ENUM;
    nvfp4_qcfg ccol = *cfg;
    ccol.tensor_id = tensor_id_col;
    QuantPlan prow{}, pcol{};
    int rc = plan_quantize(src, NVFP4_SRC_BF16, R, C, 0, cfg, out_row, &prow);
    if (rc) return rc;
    rc = plan_quantize(src, NVFP4_SRC_BF16, R, C, 1, &ccol, out_col, &pcol);
    if (rc) return rc;
    if (prow.need_partials && (!ws || ws_bytes < partials_bytes())) return NVFP4_ERR_WORKSPACE;
    if (ws && !aligned16(ws)) return NVFP4_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    stamp(out_row, prow);
    stamp(out_col, pcol);
    if (R == 0 || C == 0) return NVFP4_OK;
    QuantParams pr = params_of(prow, cfg), pc = params_of(pcol, &ccol);
    if (cfg->amax_in) {
        pr.amax_scalar = pc.amax_scalar = cfg->amax_in;
    } else {
        pr.npart = pc.npart = launch_amax_partials(src, R * C, static_cast<float *>(ws), nullptr, st);
        pr.amax_partials = pc.amax_partials = static_cast<float *>(ws);
    }
    // the dequantized maximum is only produced by the deterministic row-wise quantizer of nvfp4_quantize
    QuantOut orow{out_row->codes, out_row->scales, out_row->gscale, nullptr};
    QuantOut ocol{out_col->codes, out_col->scales, out_col->gscale, nullptr};
    return launch_quant_dual_bf16(src, R, C, pr, orow, pc, ocol, st) == hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

// common validation of the two product entry points; *need = scratch bytes of the split reduction
static int check_gemm_call(const nvfp4_tensor *A, const nvfp4_tensor *B, const void *Out, int out_dtype, size_t *need)
{
    int rc = check_gemm_operand(A);
    if (rc) return rc;
    rc = check_gemm_operand(B);
    if (rc) return rc;
    rc = check_out(Out, out_dtype);
    if (rc) return rc;
    if (A->K != B->K || A->outer_mode != B->outer_mode) return NVFP4_ERR_MISMATCH;
    *need = gemm_workspace_bytes(A->rows, B->rows, A->K, A->outer_mode);
    return NVFP4_OK;
}

int nvfp4_gemm_nt(const nvfp4_tensor *A, const nvfp4_tensor *B, void *Out, int out_dtype, void *ws, size_t ws_bytes,
                  void *stream)
{
    size_t need = 0;
    const int rc = check_gemm_call(A, B, Out, out_dtype, &need);
    if (rc) return rc;
    if (ws && !aligned16(ws)) return NVFP4_ERR_ALIGN;
    if (need > 0 && (!ws || ws_bytes < need)) return NVFP4_ERR_WORKSPACE;
    return run_gemm(A, B, Out, out_dtype, ws, ws_bytes, static_cast<hipStream_t>(stream));
}

int nvfp4_gemm_nt_static(const nvfp4_tensor *A, const nvfp4_tensor *B, void *Out, int out_dtype, void *stream)
{
    size_t need = 0;
    int rc = check_gemm_call(A, B, Out, out_dtype, &need);
    if (rc) return rc;
    if (need > kStaticScratchBytes) return NVFP4_ERR_SCRATCH;
    void *ws = nullptr;
    if (need > 0) {
        rc = static_scratch(&ws);
        if (rc) return rc;
    }
    return run_gemm(A, B, Out, out_dtype, ws, need, static_cast<hipStream_t>(stream));
}

// ---- OutControl split linear (Sec. 4.2) -------------------------------------------------------------------------

static nvfp4_qcfg bwd_cfg(uint64_t seed, uint32_t layer_id, int k, int outer, int rht);

static size_t outctl_fwd_bytes(int64_t N, int64_t D_lo, int64_t C, int outer, int out_dtype)
{
    return nvfp4_workspace_bytes(NVFP4_OP_LINEAR_FWD, N, D_lo, C, outer) +
           (out_dtype == NVFP4_OUT_F32 ? 0 : align_up((size_t)(N * C) * sizeof(float)));
}

static size_t outctl_bwd_bytes(int64_t N, int64_t D_lo, int64_t D_hp, int64_t C, int outer)
{
    const size_t g1 = align_up(gemm_workspace_bytes(N, D_lo, C, outer)), g2 = align_up(gemm_workspace_bytes(C, D_lo, N, outer));
    const size_t g3 = align_up(gemm_workspace_bytes(N, D_hp, C, outer));
    size_t g = g1 > g2 ? g1 : g2;
    g = g > g3 ? g : g3;
    return 2 * partials_bytes() + packed_bytes(N, C, outer) + packed_bytes(D_lo, C, outer) + packed_bytes(D_hp, C, outer) +
           packed_bytes(C, N, outer) + packed_bytes(D_lo, N, outer) + align_up((size_t)(N * C) * 2) +
           align_up((size_t)(N * D_hp) * 2) + g;
}

size_t nvfp4_outctl_workspace_bytes(int backward, int64_t N, int64_t D_lo, int64_t D_hp, int64_t C, int outer_mode, int out_dtype)
{
    if (N < 0 || D_lo < 0 || D_hp < 0 || C < 0 || !valid_outer(outer_mode)) return 0;
    return backward ? outctl_bwd_bytes(N, D_lo, D_hp, C, outer_mode) : outctl_fwd_bytes(N, D_lo, C, outer_mode, out_dtype);
}

int nvfp4_outctl_fwd(const void *X_lo, const void *W_lo, const void *X_hp, const void *W_hp, int64_t N, int64_t D_lo,
                     int64_t D_hp, int64_t C, void *Y, int out_dtype, nvfp4_tensor *Xq_ctx, nvfp4_tensor *Wq_ctx,
                     int outer_mode, void *ws, size_t ws_bytes, void *stream)
{
    if (!X_hp || !W_hp) return NVFP4_ERR_NULL;
    if (D_hp < 0 || D_hp % 32 != 0) return NVFP4_ERR_SHAPE;
    if (!aligned16(X_hp) || !aligned16(W_hp)) return NVFP4_ERR_ALIGN;
    int rc = check_out(Y, out_dtype);
    if (rc) return rc;
    if (N < 0 || D_lo < 0 || C < 0) return NVFP4_ERR_SHAPE;
    if (!valid_outer(outer_mode)) return NVFP4_ERR_ENUM;
    if (!ws || ws_bytes < outctl_fwd_bytes(N, D_lo, C, outer_mode, out_dtype)) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(ws)) return NVFP4_ERR_ALIGN;
    // the FP4 product in FP32 (in Y itself when Y is FP32), then the bf16 term is added and the sum stored
    const size_t fwd_ws = nvfp4_workspace_bytes(NVFP4_OP_LINEAR_FWD, N, D_lo, C, outer_mode);
    float *y32 = out_dtype == NVFP4_OUT_F32 ? static_cast<float *>(Y)
                                            : reinterpret_cast<float *>(static_cast<uint8_t *>(ws) + fwd_ws);
    rc = nvfp4_linear_fwd(X_lo, W_lo, N, D_lo, C, y32, NVFP4_OUT_F32, Xq_ctx, Wq_ctx, outer_mode, ws, fwd_ws, stream);
    if (rc) return rc;
    return launch_hp_gemm_nt(X_hp, W_hp, N, C, D_hp, y32, Y, out_dtype == NVFP4_OUT_F32, static_cast<hipStream_t>(stream)) ==
                   hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_outctl_bwd(const void *dY, const nvfp4_tensor *Xq_ctx, const nvfp4_tensor *Wq_ctx, const void *X_hp,
                     const void *W_hp, int64_t N, int64_t D_lo, int64_t D_hp, int64_t C, void *dX_lo, void *dX_hp,
                     void *dW_lo, void *dW_hp, int out_dtype, uint64_t seed, uint32_t layer_id, int rht, void *ws,
                     size_t ws_bytes, void *stream)
{
    if (!dY || !Xq_ctx || !Wq_ctx || !X_hp || !W_hp) return NVFP4_ERR_NULL;
    if (N < 0 || D_lo < 0 || D_hp < 0 || C < 0) return NVFP4_ERR_SHAPE;
    if (check_reduction(C) || check_reduction(N) || D_hp % 32 != 0) return NVFP4_ERR_SHAPE;
    int rc = check_out(dX_lo, out_dtype);
    if (!rc) rc = check_out(dX_hp, out_dtype);
    if (!rc) rc = check_out(dW_lo, out_dtype);
    if (!rc) rc = check_out(dW_hp, out_dtype);
    if (rc) return rc;
    if (Wq_ctx->rows != C || Wq_ctx->K != D_lo || Xq_ctx->rows != N || Xq_ctx->K != D_lo) return NVFP4_ERR_MISMATCH;
    if (Wq_ctx->outer_mode != Xq_ctx->outer_mode) return NVFP4_ERR_MISMATCH;
    const int outer = Xq_ctx->outer_mode;
    if (!valid_outer(outer)) return NVFP4_ERR_ENUM;
    if (!aligned16(dY) || !aligned16(X_hp) || !aligned16(W_hp)) return NVFP4_ERR_ALIGN;
    if (!ws || ws_bytes < outctl_bwd_bytes(N, D_lo, D_hp, C, outer)) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(ws)) return NVFP4_ERR_ALIGN;
    Carver cv{static_cast<uint8_t *>(ws), ws_bytes, 0};
    float *part = static_cast<float *>(cv.take(sizeof(float) * kMaxAmaxPartials));
    float *part2 = static_cast<float *>(cv.take(sizeof(float) * kMaxAmaxPartials));
    nvfp4_tensor q3{}, q4{}, q4h{}, q5{}, q6{};
    if (!carve_tensor(cv, N, C, outer, &q3) || !carve_tensor(cv, D_lo, C, outer, &q4) || !carve_tensor(cv, D_hp, C, outer, &q4h) ||
        !carve_tensor(cv, C, N, outer, &q5) || !carve_tensor(cv, D_lo, N, outer, &q6))
        return NVFP4_ERR_WORKSPACE;
    void *dYT = cv.take((size_t)(N * C) * 2), *XhT = cv.take((size_t)(N * D_hp) * 2);
    const size_t g1 = gemm_workspace_bytes(N, D_lo, C, outer), g2 = gemm_workspace_bytes(C, D_lo, N, outer),
                 g3 = gemm_workspace_bytes(N, D_hp, C, outer);
    size_t gbytes = g1 > g2 ? g1 : g2;
    gbytes = gbytes > g3 ? gbytes : g3;
    void *gws = gbytes ? cv.take(gbytes) : nullptr;
    if (!dYT || !XhT || (gbytes && !gws)) return NVFP4_ERR_WORKSPACE;

    // the five stochastic quantizers: Q3, Q5 of dY; Q4, Q6 of the forward contexts; Q4 of the outlier channels of W
    nvfp4_qcfg c3 = bwd_cfg(seed, layer_id, 3, outer, rht), c4 = bwd_cfg(seed, layer_id, 4, outer, rht),
               c5 = bwd_cfg(seed, layer_id, 5, outer, rht), c6 = bwd_cfg(seed, layer_id, 6, outer, rht),
               c9 = bwd_cfg(seed, layer_id, 9, outer, rht);
    QuantPlan p3{}, p4{}, p5{}, p6{}, p9{};
    rc = plan_quantize(dY, NVFP4_SRC_BF16, N, C, 0, &c3, &q3, &p3);
    if (!rc) rc = plan_quantize(Wq_ctx, NVFP4_SRC_NVFP4, C, D_lo, 1, &c4, &q4, &p4);
    if (!rc) rc = plan_quantize(dY, NVFP4_SRC_BF16, N, C, 1, &c5, &q5, &p5);
    if (!rc) rc = plan_quantize(Xq_ctx, NVFP4_SRC_NVFP4, N, D_lo, 1, &c6, &q6, &p6);
    if (!rc && D_hp > 0) rc = plan_quantize(W_hp, NVFP4_SRC_BF16, C, D_hp, 1, &c9, &q4h, &p9);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = run_quantize(dY, p3, &c3, &q3, part, st);
    if (!rc) rc = run_quantize(dY, p5, &c5, &q5, part, st);
    if (!rc) rc = run_requant_pair(Wq_ctx, p4, &c4, &q4, Xq_ctx, p6, &c6, &q6, st);
    if (!rc && D_hp > 0) rc = run_quantize(W_hp, p9, &c9, &q4h, part2, st);
    if (rc) return rc;
    // dX over all input channels in FP4 (one Q3 operand serves both column sets); dW of the ordinary channels in FP4
    rc = run_gemm(&q3, &q4, dX_lo, out_dtype, gws, gbytes, st);
    if (!rc && D_hp > 0) rc = run_gemm(&q3, &q4h, dX_hp, out_dtype, gws, gbytes, st);
    if (!rc) rc = run_gemm(&q5, &q6, dW_lo, out_dtype, gws, gbytes, st);
    if (rc) return rc;
    // dW of the outlier channels in bf16: dY^T [C x N] times X_hp^T [D_hp x N]^T, the reduction running over tokens
    if (D_hp > 0 && C > 0) {
        if (launch_transpose_bf16(dY, dYT, N, C, st) != hipSuccess) return NVFP4_ERR_HIP;
        if (launch_transpose_bf16(X_hp, XhT, N, D_hp, st) != hipSuccess) return NVFP4_ERR_HIP;
        if (launch_hp_gemm_nt(dYT, XhT, C, D_hp, N, nullptr, dW_hp, out_dtype == NVFP4_OUT_F32, st) != hipSuccess)
            return NVFP4_ERR_HIP;
    }
    return NVFP4_OK;
}

static int check_osci(const void *W, const void *a, const void *b, int64_t C, int64_t D)
{
    if (!W || !a || !b) return NVFP4_ERR_NULL;
    if (C < 0 || D < 0 || D % 128 != 0) return NVFP4_ERR_SHAPE;
    if (C > 0 && D > kMaxElems / C) return NVFP4_ERR_SHAPE;
    if (!aligned16(W) || !aligned16(a) || !aligned16(b)) return NVFP4_ERR_ALIGN;
    return NVFP4_OK;
}

int nvfp4_osci_update(const float *W, float *W_prev, float *dist_m, float *dist_q, int64_t C, int64_t D, int t0, void *stream)
{
    int rc = check_osci(W, W_prev, dist_m, C, D);
    if (rc) return rc;
    if (!dist_q) return NVFP4_ERR_NULL;
    if (!aligned16(dist_q)) return NVFP4_ERR_ALIGN;
    if (t0 < 0) return NVFP4_ERR_ENUM;
    return launch_osci_update(W, W_prev, dist_m, dist_q, C * D, t0 == 0, static_cast<hipStream_t>(stream)) == hipSuccess
               ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_osci_suppress(float *W, const float *dist_m, const float *dist_q, float tau, int64_t C, int64_t D,
                        unsigned long long *n_reset, void *stream)
{
    const int rc = check_osci(W, dist_m, dist_q, C, D);
    if (rc) return rc;
    if (!(tau > 0.0f)) return NVFP4_ERR_ENUM;
    if (n_reset && (reinterpret_cast<uintptr_t>(n_reset) & 7u)) return NVFP4_ERR_ALIGN;
    return launch_osci_suppress(W, dist_m, dist_q, tau, C * D, n_reset, static_cast<hipStream_t>(stream)) == hipSuccess
               ? NVFP4_OK : NVFP4_ERR_HIP;
}

// the tracked subset of Appendix Alg. 3: 32-bit indices, so at most 2^31 weights per matrix
static int check_osci_sparse(const void *W, int64_t C, int64_t D, const void *idx, int64_t k, const void *a, const void *b)
{
    if (!W) return NVFP4_ERR_NULL;
    if (C < 0 || D < 0 || D % 128 != 0 || k < 0) return NVFP4_ERR_SHAPE;
    if (C > 0 && D > ((int64_t)1 << 31) / C) return NVFP4_ERR_SHAPE;
    if (k > C * D) return NVFP4_ERR_SHAPE;
    if (k > 0 && (!idx || !a || !b)) return NVFP4_ERR_NULL;
    if (!aligned16(W)) return NVFP4_ERR_ALIGN;
    return NVFP4_OK;
}

size_t nvfp4_osci_select_workspace_bytes(int64_t C, int64_t D)
{
    if (C < 0 || D < 0 || (C > 0 && D > ((int64_t)1 << 31) / C)) return 0;
    return osci_select_workspace_bytes(C * D);
}

int nvfp4_osci_select(const float *W, int64_t C, int64_t D, int64_t k, uint32_t *idx, float *W_prev_s, float *Q_prev_s,
                      float *dist_m_s, float *dist_q_s, void *ws, size_t ws_bytes, void *stream)
{
    int rc = check_osci_sparse(W, C, D, idx, k, W_prev_s, Q_prev_s);
    if (rc) return rc;
    if (k > 0 && (!dist_m_s || !dist_q_s)) return NVFP4_ERR_NULL;
    if (k == 0 || C * D == 0) return NVFP4_OK;
    if (!ws || ws_bytes < osci_select_workspace_bytes(C * D)) return NVFP4_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) & 15u) return NVFP4_ERR_ALIGN;
    return launch_osci_select(W, C * D, k, idx, W_prev_s, Q_prev_s, dist_m_s, dist_q_s, ws, static_cast<hipStream_t>(stream)) ==
                   hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_osci_update_sparse(const float *W, int64_t C, int64_t D, const uint32_t *idx, int64_t k, float *W_prev_s,
                             float *Q_prev_s, float *dist_m_s, float *dist_q_s, void *stream)
{
    int rc = check_osci_sparse(W, C, D, idx, k, W_prev_s, Q_prev_s);
    if (rc) return rc;
    if (k > 0 && (!dist_m_s || !dist_q_s)) return NVFP4_ERR_NULL;
    return launch_osci_update_sparse(W, C * D, idx, k, W_prev_s, Q_prev_s, dist_m_s, dist_q_s, static_cast<hipStream_t>(stream)) ==
                   hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_osci_suppress_sparse(float *W, int64_t C, int64_t D, const uint32_t *idx, int64_t k, const float *dist_m_s,
                               const float *dist_q_s, float tau, unsigned long long *n_reset, void *stream)
{
    int rc = check_osci_sparse(W, C, D, idx, k, dist_m_s, dist_q_s);
    if (rc) return rc;
    if (!(tau > 0.0f)) return NVFP4_ERR_ENUM;
    if (n_reset && (reinterpret_cast<uintptr_t>(n_reset) & 7u)) return NVFP4_ERR_ALIGN;
    return launch_osci_suppress_sparse(W, C * D, idx, k, dist_m_s, dist_q_s, tau, n_reset, static_cast<hipStream_t>(stream)) ==
                   hipSuccess ? NVFP4_OK : NVFP4_ERR_HIP;
}

int nvfp4_linear_fwd(const void *X, const void *W, int64_t N, int64_t D, int64_t C, void *Y, int out_dtype,
                     nvfp4_tensor *Xq_ctx, nvfp4_tensor *Wq_ctx, int outer_mode, void *ws, size_t ws_bytes,
                     void *stream)
{
    if (!X || !W) return NVFP4_ERR_NULL;
    if (!valid_outer(outer_mode)) return NVFP4_ERR_ENUM;
    if (N < 0 || D < 0 || C < 0) return NVFP4_ERR_SHAPE;
    if (check_reduction(D)) return NVFP4_ERR_SHAPE;
    int rc = check_out(Y, out_dtype);
    if (rc) return rc;
    nvfp4_qcfg cfg{};
    cfg.rounding = NVFP4_ROUND_RTN;
    cfg.scale_round = NVFP4_SCALE_DEFAULT;
    cfg.outer_mode = outer_mode;
    QuantPlan px{}, pw{};
    rc = plan_quantize(X, NVFP4_SRC_BF16, N, D, 0, &cfg, Xq_ctx, &px);
    if (rc) return rc;
    rc = plan_quantize(W, NVFP4_SRC_BF16, C, D, 0, &cfg, Wq_ctx, &pw);
    if (rc) return rc;
    if (!ws || ws_bytes < nvfp4_workspace_bytes(NVFP4_OP_LINEAR_FWD, N, D, C, outer_mode)) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(ws)) return NVFP4_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    Carver cv{static_cast<uint8_t *>(ws), ws_bytes, 0};
    float *part_x = static_cast<float *>(cv.take(sizeof(float) * kMaxAmaxPartials));
    float *part_w = static_cast<float *>(cv.take(sizeof(float) * kMaxAmaxPartials));
    const size_t gbytes = gemm_workspace_bytes(N, C, D, outer_mode);
    void *gws = gbytes ? cv.take(gbytes) : nullptr;
    rc = run_quantize_row_pair(X, px, Xq_ctx, part_x, W, pw, Wq_ctx, part_w, &cfg, st);
    if (rc) return rc;
    return run_gemm(Xq_ctx, Wq_ctx, Y, out_dtype, gws, gbytes, st);
}

// stochastic-rounding settings of backward quantizer Q<k> of a layer (k = 3..6), in the forward operands' outer mode
static nvfp4_qcfg bwd_cfg(uint64_t seed, uint32_t layer_id, int k, int outer, int rht)
{
    nvfp4_qcfg c{};
    c.rounding = NVFP4_ROUND_SR;
    c.outer_mode = outer;
    c.seed = seed;
    c.tensor_id = layer_id * 16u + (uint32_t)k;
    c.rht = rht;
    c.rht_id = layer_id * 16u + (k == 3 || k == 4 || k == 9 ? 7u : 8u);   // the signs of the dX product (Q3, Q4) / of the dW product
    return c;
}

int nvfp4_linear_bwd_dx(const void *dY, const nvfp4_tensor *Wq_ctx, int64_t N, int64_t D, int64_t C, void *dX,
                        int out_dtype, uint64_t seed, uint32_t layer_id, int rht, void *ws, size_t ws_bytes, void *stream)
{
    if (!dY || !Wq_ctx) return NVFP4_ERR_NULL;
    if (N < 0 || D < 0 || C < 0) return NVFP4_ERR_SHAPE;
    if (check_reduction(C)) return NVFP4_ERR_SHAPE;
    int rc = check_out(dX, out_dtype);
    if (rc) return rc;
    if (Wq_ctx->rows != C || Wq_ctx->K != D) return NVFP4_ERR_MISMATCH;
    const int outer = Wq_ctx->outer_mode;
    if (!valid_outer(outer)) return NVFP4_ERR_ENUM;
    if (!ws || ws_bytes < nvfp4_workspace_bytes(NVFP4_OP_LINEAR_BWD_DX, N, D, C, outer)) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(ws)) return NVFP4_ERR_ALIGN;
    Carver cv{static_cast<uint8_t *>(ws), ws_bytes, 0};
    float *part = static_cast<float *>(cv.take(sizeof(float) * kMaxAmaxPartials));
    nvfp4_tensor dYq{}, Wq2{};
    if (!carve_tensor(cv, N, C, outer, &dYq) || !carve_tensor(cv, D, C, outer, &Wq2)) return NVFP4_ERR_WORKSPACE;
    const size_t gbytes = gemm_workspace_bytes(N, D, C, outer);
    void *gws = gbytes ? cv.take(gbytes) : nullptr;

    nvfp4_qcfg c3 = bwd_cfg(seed, layer_id, 3, outer, rht), c4 = bwd_cfg(seed, layer_id, 4, outer, rht);
    QuantPlan p3{}, p4{};
    rc = plan_quantize(dY, NVFP4_SRC_BF16, N, C, 0, &c3, &dYq, &p3);
    if (rc) return rc;
    rc = plan_quantize(Wq_ctx, NVFP4_SRC_NVFP4, C, D, 1, &c4, &Wq2, &p4);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = run_quantize(dY, p3, &c3, &dYq, part, st);
    if (rc) return rc;
    rc = run_quantize(Wq_ctx, p4, &c4, &Wq2, nullptr, st);
    if (rc) return rc;
    return run_gemm(&dYq, &Wq2, dX, out_dtype, gws, gbytes, st);
}

int nvfp4_linear_bwd_dw(const void *dY, const nvfp4_tensor *Xq_ctx, int64_t N, int64_t D, int64_t C, void *dW,
                        int out_dtype, uint64_t seed, uint32_t layer_id, int rht, void *ws, size_t ws_bytes, void *stream)
{
    if (!dY || !Xq_ctx) return NVFP4_ERR_NULL;
    if (N < 0 || D < 0 || C < 0) return NVFP4_ERR_SHAPE;
    if (check_reduction(N)) return NVFP4_ERR_SHAPE;
    int rc = check_out(dW, out_dtype);
    if (rc) return rc;
    if (Xq_ctx->rows != N || Xq_ctx->K != D) return NVFP4_ERR_MISMATCH;
    const int outer = Xq_ctx->outer_mode;
    if (!valid_outer(outer)) return NVFP4_ERR_ENUM;
    if (!ws || ws_bytes < nvfp4_workspace_bytes(NVFP4_OP_LINEAR_BWD_DW, N, D, C, outer)) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(ws)) return NVFP4_ERR_ALIGN;
    Carver cv{static_cast<uint8_t *>(ws), ws_bytes, 0};
    float *part = static_cast<float *>(cv.take(sizeof(float) * kMaxAmaxPartials));
    nvfp4_tensor dYq{}, Xq2{};
    if (!carve_tensor(cv, C, N, outer, &dYq) || !carve_tensor(cv, D, N, outer, &Xq2)) return NVFP4_ERR_WORKSPACE;
    const size_t gbytes = gemm_workspace_bytes(C, D, N, outer);
    void *gws = gbytes ? cv.take(gbytes) : nullptr;

    nvfp4_qcfg c5 = bwd_cfg(seed, layer_id, 5, outer, rht), c6 = bwd_cfg(seed, layer_id, 6, outer, rht);
    QuantPlan p5{}, p6{};
    rc = plan_quantize(dY, NVFP4_SRC_BF16, N, C, 1, &c5, &dYq, &p5);
    if (rc) return rc;
    rc = plan_quantize(Xq_ctx, NVFP4_SRC_NVFP4, N, D, 1, &c6, &Xq2, &p6);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    rc = run_quantize(dY, p5, &c5, &dYq, part, st);
    if (rc) return rc;
    rc = run_quantize(Xq_ctx, p6, &c6, &Xq2, nullptr, st);
    if (rc) return rc;
    return run_gemm(&dYq, &Xq2, dW, out_dtype, gws, gbytes, st);
}

int nvfp4_linear_bwd(const void *dY, const nvfp4_tensor *Xq_ctx, const nvfp4_tensor *Wq_ctx, int64_t N, int64_t D,
                     int64_t C, void *dX, void *dW, int out_dtype, uint64_t seed, uint32_t layer_id, int rht, void *ws,
                     size_t ws_bytes, void *stream)
{
    if (!dY || !Xq_ctx || !Wq_ctx) return NVFP4_ERR_NULL;
    if (N < 0 || D < 0 || C < 0) return NVFP4_ERR_SHAPE;
    if (check_reduction(C) || check_reduction(N)) return NVFP4_ERR_SHAPE;
    int rc = check_out(dX, out_dtype);
    if (rc) return rc;
    rc = check_out(dW, out_dtype);
    if (rc) return rc;
    if (Wq_ctx->rows != C || Wq_ctx->K != D || Xq_ctx->rows != N || Xq_ctx->K != D) return NVFP4_ERR_MISMATCH;
    if (Wq_ctx->outer_mode != Xq_ctx->outer_mode) return NVFP4_ERR_MISMATCH;
    const int outer = Xq_ctx->outer_mode;
    if (!valid_outer(outer)) return NVFP4_ERR_ENUM;
    if (!aligned16(dY)) return NVFP4_ERR_ALIGN;
    if (!ws || ws_bytes < nvfp4_workspace_bytes(NVFP4_OP_LINEAR_BWD, N, D, C, outer)) return NVFP4_ERR_WORKSPACE;
    if (!aligned16(ws)) return NVFP4_ERR_ALIGN;
    Carver cv{static_cast<uint8_t *>(ws), ws_bytes, 0};
    float *part = static_cast<float *>(cv.take(sizeof(float) * kMaxAmaxPartials));
    float *amax = static_cast<float *>(cv.take(sizeof(float)));
    nvfp4_tensor q3{}, q4{}, q5{}, q6{};
    if (!carve_tensor(cv, N, C, outer, &q3) || !carve_tensor(cv, D, C, outer, &q4) || !carve_tensor(cv, C, N, outer, &q5) ||
        !carve_tensor(cv, D, N, outer, &q6))
        return NVFP4_ERR_WORKSPACE;
    const size_t g1 = gemm_workspace_bytes(N, D, C, outer), g2 = gemm_workspace_bytes(C, D, N, outer);
    const size_t gbytes = g1 > g2 ? g1 : g2;
    void *gws = gbytes ? cv.take(gbytes) : nullptr;

    nvfp4_qcfg c[4];
    for (int k = 0; k < 4; ++k) c[k] = bwd_cfg(seed, layer_id, 3 + k, outer, rht);
    if (outer == NVFP4_OUTER_TENSOR) {
        c[0].amax_in = amax;     // Q3 and Q5 share the maximum of dY
        c[2].amax_in = amax;
    }
    QuantPlan p3{}, p4{}, p5{}, p6{};
    rc = plan_quantize(dY, NVFP4_SRC_BF16, N, C, 0, &c[0], &q3, &p3);
    if (rc) return rc;
    rc = plan_quantize(Wq_ctx, NVFP4_SRC_NVFP4, C, D, 1, &c[1], &q4, &p4);
    if (rc) return rc;
    rc = plan_quantize(dY, NVFP4_SRC_BF16, N, C, 1, &c[2], &q5, &p5);
    if (rc) return rc;
    rc = plan_quantize(Xq_ctx, NVFP4_SRC_NVFP4, N, D, 1, &c[3], &q6, &p6);
    if (rc) return rc;

    hipStream_t st = static_cast<hipStream_t>(stream);
    if (outer == NVFP4_OUTER_TENSOR) {
        if (N > 0 && C > 0) {
            // every workgroup of the quantizer reduces the partial maxima itself: no launch in between
            const int npart = launch_amax_partials(dY, N * C, part, nullptr, st);
            QuantParams pr{}, pc{};
            pr.rounding = pc.rounding = 1;
            pr.scale_up = pc.scale_up = 1;
            pr.amax_partials = pc.amax_partials = part;
            pr.npart = pc.npart = npart;
            const uint64_t k3 = stream_key(seed, c[0].tensor_id), k5 = stream_key(seed, c[2].tensor_id);
            pr.k0 = (uint32_t)k3; pr.k1 = (uint32_t)(k3 >> 32);
            pc.k0 = (uint32_t)k5; pc.k1 = (uint32_t)(k5 >> 32);
            QuantOut orow{q3.codes, q3.scales, q3.gscale, nullptr}, ocol{q5.codes, q5.scales, q5.gscale, nullptr};
            if (launch_quant_dual_bf16(dY, N, C, pr, orow, pc, ocol, st) != hipSuccess) return NVFP4_ERR_HIP;
        }
        q3.rows = N; q3.K = C; q5.rows = C; q5.K = N;
    } else {
        // 1 x 128 outer blocks: no maximum pass at all; dY is read once per operand, each a single pass
        rc = run_quantize(dY, p3, &c[0], &q3, nullptr, st);
        if (rc) return rc;
        rc = run_quantize(dY, p5, &c[2], &q5, nullptr, st);
        if (rc) return rc;
    }
    rc = run_requant_pair(Wq_ctx, p4, &c[1], &q4, Xq_ctx, p6, &c[3], &q6, st);
    if (rc) return rc;
    rc = run_gemm(&q3, &q4, dX, out_dtype, gws, gbytes, st);
    if (rc) return rc;
    return run_gemm(&q5, &q6, dW, out_dtype, gws, gbytes, st);
}

}  // extern "C"
