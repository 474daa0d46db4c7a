"""ctypes binding of libtjnvfp4.so: argument marshalling only.

Every step of the path (maxima, quantizers, re-quantizers, matrix products) runs in the
library's HIP kernels; this module turns torch CUDA tensors into raw device pointers and
the current torch stream into a hipStream_t.  There is no CPU fallback: if the library is
missing the import fails.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtjnvfp4.so")

ROUND_RTN, ROUND_SR = 0, 1
SCALE_DEFAULT, SCALE_NE, SCALE_UP = 0, 1, 2
OUTER_TENSOR, OUTER_BLOCK128 = 0, 1
SRC_BF16, SRC_NVFP4 = 0, 1
OUT_BF16, OUT_F32 = 0, 1
OP_QUANTIZE, OP_GEMM, OP_LINEAR_FWD, OP_LINEAR_BWD_DX, OP_LINEAR_BWD_DW, OP_LINEAR_BWD = 0, 1, 2, 3, 4, 5

EXPORTS = ["nvfp4_quantize", "nvfp4_quantize_dual", "nvfp4_gemm_nt", "nvfp4_gemm_nt_static", "nvfp4_linear_fwd", "nvfp4_linear_bwd_dx", "nvfp4_linear_bwd_dw", "nvfp4_linear_bwd", "nvfp4_osci_update", "nvfp4_osci_suppress", "nvfp4_osci_select", "nvfp4_osci_update_sparse", "nvfp4_osci_suppress_sparse", "nvfp4_osci_select_workspace_bytes", "nvfp4_outctl_fwd", "nvfp4_outctl_bwd", "nvfp4_outctl_workspace_bytes",
           "nvfp4_workspace_bytes", "nvfp4_gemm_plan", "nvfp4_amax_bf16", "nvfp4_stream_key", "nvfp4_strerror", "nvfp4_version"]


class NVFP4Error(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, lib().nvfp4_strerror(code).decode(), code))


class CTensor(C.Structure):
    _fields_ = [("codes", C.c_void_p), ("scales", C.c_void_p), ("gscale", C.c_void_p), ("amax_deq", C.c_void_p),
                ("rows", C.c_int64), ("K", C.c_int64), ("outer_mode", C.c_int32), ("reserved", C.c_int32)]


class CQcfg(C.Structure):
    _fields_ = [("rounding", C.c_int32), ("scale_round", C.c_int32), ("outer_mode", C.c_int32),
                ("tensor_id", C.c_uint32), ("seed", C.c_uint64), ("amax_in", C.c_void_p), ("rht", C.c_int32),
                ("rht_id", C.c_uint32)]


_lib = None


def lib():
    """Load the library (raises OSError if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise OSError("libtjnvfp4.so is not built: run `python -m paper_2510_27527_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, u64, u32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_uint32, C.c_size_t
        L.nvfp4_quantize.restype = i32
        L.nvfp4_quantize.argtypes = [vp, i32, i64, i64, i32, C.POINTER(CQcfg), C.POINTER(CTensor), vp, sz, vp]
        L.nvfp4_quantize_dual.restype = i32
        L.nvfp4_quantize_dual.argtypes = [vp, i64, i64, C.POINTER(CQcfg), u32, C.POINTER(CTensor), C.POINTER(CTensor), vp, sz,
                                          vp]
        L.nvfp4_gemm_nt.restype = i32
        L.nvfp4_gemm_nt.argtypes = [C.POINTER(CTensor), C.POINTER(CTensor), vp, i32, vp, sz, vp]
        L.nvfp4_gemm_nt_static.restype = i32
        L.nvfp4_gemm_nt_static.argtypes = [C.POINTER(CTensor), C.POINTER(CTensor), vp, i32, vp]
        L.nvfp4_linear_fwd.restype = i32
        L.nvfp4_linear_fwd.argtypes = [vp, vp, i64, i64, i64, vp, i32, C.POINTER(CTensor), C.POINTER(CTensor),
                                       i32, vp, sz, vp]
        L.nvfp4_linear_bwd_dx.restype = i32
        L.nvfp4_linear_bwd_dx.argtypes = [vp, C.POINTER(CTensor), i64, i64, i64, vp, i32, u64, u32, i32, vp, sz, vp]
        L.nvfp4_linear_bwd_dw.restype = i32
        L.nvfp4_linear_bwd_dw.argtypes = [vp, C.POINTER(CTensor), i64, i64, i64, vp, i32, u64, u32, i32, vp, sz, vp]
        L.nvfp4_linear_bwd.restype = i32
        L.nvfp4_linear_bwd.argtypes = [vp, C.POINTER(CTensor), C.POINTER(CTensor), i64, i64, i64, vp, vp, i32, u64, u32,
                                       i32, vp, sz, vp]
        L.nvfp4_outctl_fwd.restype = i32
        L.nvfp4_outctl_fwd.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, vp, i32, C.POINTER(CTensor), C.POINTER(CTensor), i32, vp,
                                       sz, vp]
        L.nvfp4_outctl_bwd.restype = i32
        L.nvfp4_outctl_bwd.argtypes = [vp, C.POINTER(CTensor), C.POINTER(CTensor), vp, vp, i64, i64, i64, i64, vp, vp, vp, vp, i32,
                                       u64, u32, i32, vp, sz, vp]
        L.nvfp4_outctl_workspace_bytes.restype = sz
        L.nvfp4_outctl_workspace_bytes.argtypes = [i32, i64, i64, i64, i64, i32, i32]
        L.nvfp4_osci_update.restype = i32
        L.nvfp4_osci_update.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp]
        L.nvfp4_osci_suppress.restype = i32
        L.nvfp4_osci_suppress.argtypes = [vp, vp, vp, C.c_float, i64, i64, vp, vp]
        L.nvfp4_osci_select_workspace_bytes.restype = C.c_size_t
        L.nvfp4_osci_select_workspace_bytes.argtypes = [i64, i64]
        L.nvfp4_osci_select.restype = i32
        L.nvfp4_osci_select.argtypes = [vp, i64, i64, i64, vp, vp, vp, vp, vp, vp, C.c_size_t, vp]
        L.nvfp4_osci_update_sparse.restype = i32
        L.nvfp4_osci_update_sparse.argtypes = [vp, i64, i64, vp, i64, vp, vp, vp, vp, vp]
        L.nvfp4_osci_suppress_sparse.restype = i32
        L.nvfp4_osci_suppress_sparse.argtypes = [vp, i64, i64, vp, i64, vp, vp, C.c_float, vp, vp]
        L.nvfp4_workspace_bytes.restype = sz
        L.nvfp4_workspace_bytes.argtypes = [i32, i64, i64, i64, i32]
        L.nvfp4_gemm_plan.restype = i32
        L.nvfp4_gemm_plan.argtypes = [i64, i64, i64, i32, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)]
        L.nvfp4_amax_bf16.restype = i32
        L.nvfp4_amax_bf16.argtypes = [vp, i64, vp, vp, sz, vp]
        L.nvfp4_stream_key.restype = u64
        L.nvfp4_stream_key.argtypes = [u64, u32]
        L.nvfp4_strerror.restype = C.c_char_p
        L.nvfp4_strerror.argtypes = [i32]
        L.nvfp4_version.restype = C.c_char_p
        L.nvfp4_version.argtypes = []
        _lib = L
    return _lib


def _check(rc: int, where: str):
    if rc != 0:
        raise NVFP4Error(rc, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


_EMPTY = {}


def _ptr(t: Optional[torch.Tensor]):
    """Device address of a tensor.  An empty tensor has no storage; the library still wants a non-NULL, 16-byte
    aligned pointer for it (it never dereferences it), so it gets the address of a small per-device placeholder."""
    if t is None:
        return None
    if t.numel() == 0 and t.is_cuda:
        key = t.device.index
        if key not in _EMPTY:
            _EMPTY[key] = torch.zeros(64, dtype=torch.uint8, device=t.device)
        return _EMPTY[key].data_ptr()
    return t.data_ptr()


@dataclass
class NVFP4Tensor:
    """Device buffers of one quantized operand [rows, K] (K contiguous, grouped axis)."""
    codes: torch.Tensor      # uint8 [rows, K/2]
    scales: torch.Tensor     # uint8 [rows, K/16]
    gscale: torch.Tensor     # float32 [1] or [rows, K/128]
    amax_deq: Optional[torch.Tensor]   # float32 [1] or None
    rows: int
    K: int
    outer: int

    def c_struct(self) -> CTensor:
        return CTensor(_ptr(self.codes), _ptr(self.scales), _ptr(self.gscale), _ptr(self.amax_deq),
                       self.rows, self.K, self.outer, 0)


def alloc_nvfp4(rows: int, K: int, outer: int = OUTER_TENSOR, device="cuda", with_amax: bool = True) -> NVFP4Tensor:
    codes = torch.empty((rows, K // 2), dtype=torch.uint8, device=device)
    scales = torch.empty((rows, K // 16), dtype=torch.uint8, device=device)
    gshape = (1,) if outer == OUTER_TENSOR else (rows, max(K // 128, 1))
    gscale = torch.empty(gshape, dtype=torch.float32, device=device)
    amax = torch.zeros((1,), dtype=torch.float32, device=device) if with_amax else None
    return NVFP4Tensor(codes, scales, gscale, amax, rows, K, outer)


def workspace_bytes(op: int, N: int, D: int, Cc: int, outer: int = OUTER_TENSOR) -> int:
    return int(lib().nvfp4_workspace_bytes(op, N, D, Cc, outer))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty((max(int(nbytes), 16),), dtype=torch.uint8, device=device)


def gemm_plan(M: int, N: int, K: int, outer: int = OUTER_TENSOR):
    """(tile rows, tile columns, K splits) nvfp4_gemm_nt will use for this shape and outer mode."""
    a, b, c = C.c_int(), C.c_int(), C.c_int()
    _check(lib().nvfp4_gemm_plan(M, N, K, outer, C.byref(a), C.byref(b), C.byref(c)), "nvfp4_gemm_plan")
    return a.value, b.value, c.value


def stream_key(seed: int, tensor_id: int) -> int:
    return int(lib().nvfp4_stream_key(seed, tensor_id))


def amax_bf16(src: torch.Tensor, ws: torch.Tensor) -> torch.Tensor:
    out = torch.empty((1,), dtype=torch.float32, device=src.device)
    _check(lib().nvfp4_amax_bf16(_ptr(src), src.numel(), _ptr(out), _ptr(ws), ws.numel(), _stream()), "nvfp4_amax_bf16")
    return out


def quantize(src, axis: int, rounding: int, out: Optional[NVFP4Tensor] = None, *, scale_round: int = SCALE_DEFAULT,
             outer: int = OUTER_TENSOR, seed: int = 0, tensor_id: int = 0, amax_in: Optional[torch.Tensor] = None,
             ws: Optional[torch.Tensor] = None, rht_id: Optional[int] = None) -> NVFP4Tensor:
    """nvfp4_quantize: src is a bf16 [R, C] tensor or an NVFP4Tensor."""
    if isinstance(src, NVFP4Tensor):
        kind, R, Cc = SRC_NVFP4, src.rows, src.K
        cs = src.c_struct()
        src_arg = C.cast(C.pointer(cs), C.c_void_p)
        dev = src.codes.device
    else:
        assert src.dtype == torch.bfloat16 and src.dim() == 2 and src.is_contiguous()
        kind, (R, Cc) = SRC_BF16, src.shape
        src_arg = _ptr(src)
        dev = src.device
    rows, K = (R, Cc) if axis == 0 else (Cc, R)
    if out is None:
        out = alloc_nvfp4(rows, K, outer, dev)
    if ws is None:
        ws = alloc_workspace(workspace_bytes(OP_QUANTIZE, R, Cc, 0, outer), dev)
    cfg = CQcfg(rounding, scale_round, outer, tensor_id, seed, _ptr(amax_in), 0 if rht_id is None else 1, rht_id or 0)
    co = out.c_struct()
    rc = lib().nvfp4_quantize(src_arg, kind, R, Cc, axis, C.byref(cfg), C.byref(co), _ptr(ws), ws.numel(), _stream())
    _check(rc, "nvfp4_quantize")
    out.rows, out.K, out.outer = co.rows, co.K, co.outer_mode
    return out


def quantize_dual(src: torch.Tensor, rounding: int, out_row: Optional[NVFP4Tensor] = None,
                  out_col: Optional[NVFP4Tensor] = None, *, scale_round: int = SCALE_DEFAULT, seed: int = 0,
                  tensor_id_row: int = 0, tensor_id_col: int = 0, amax_in: Optional[torch.Tensor] = None,
                  ws: Optional[torch.Tensor] = None):
    """nvfp4_quantize_dual: row-wise [R, C] and column-wise [C, R] operands of a bf16 [R, C] tensor from one read."""
    assert src.dtype == torch.bfloat16 and src.dim() == 2 and src.is_contiguous()
    R, Cc = src.shape
    dev = src.device
    if out_row is None:
        out_row = alloc_nvfp4(R, Cc, OUTER_TENSOR, dev)
    if out_col is None:
        out_col = alloc_nvfp4(Cc, R, OUTER_TENSOR, dev)
    if ws is None:
        ws = alloc_workspace(workspace_bytes(OP_QUANTIZE, R, Cc, 0, OUTER_TENSOR), dev)
    cfg = CQcfg(rounding, scale_round, OUTER_TENSOR, tensor_id_row, seed, _ptr(amax_in), 0, 0)
    cr, cc = out_row.c_struct(), out_col.c_struct()
    rc = lib().nvfp4_quantize_dual(_ptr(src), R, Cc, C.byref(cfg), tensor_id_col, C.byref(cr), C.byref(cc), _ptr(ws),
                                   ws.numel(), _stream())
    _check(rc, "nvfp4_quantize_dual")
    out_row.rows, out_row.K, out_row.outer = cr.rows, cr.K, cr.outer_mode
    out_col.rows, out_col.K, out_col.outer = cc.rows, cc.K, cc.outer_mode
    return out_row, out_col


def _check_bf16(t: torch.Tensor, what: str):
    assert t.dtype == torch.bfloat16 and t.dim() == 2 and t.is_contiguous() and t.is_cuda, what + ": bf16, 2-D, contiguous, on the GPU"


def _check_out(t: torch.Tensor, shape, out_dtype: int, what: str):
    want = torch.bfloat16 if out_dtype == OUT_BF16 else torch.float32
    assert t.dtype == want and tuple(t.shape) == tuple(shape) and t.is_contiguous() and t.is_cuda, what


def _out_tensor(M, N, out_dtype, device):
    return torch.empty((M, N), dtype=torch.bfloat16 if out_dtype == OUT_BF16 else torch.float32, device=device)


def gemm_nt(A: NVFP4Tensor, B: NVFP4Tensor, out_dtype: int = OUT_BF16, out: Optional[torch.Tensor] = None,
            ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    dev = A.codes.device
    if out is None:
        out = _out_tensor(A.rows, B.rows, out_dtype, dev)
    if ws is None:
        ws = alloc_workspace(workspace_bytes(OP_GEMM, A.rows, A.K, B.rows, A.outer), dev)
    ca, cb = A.c_struct(), B.c_struct()
    rc = lib().nvfp4_gemm_nt(C.byref(ca), C.byref(cb), _ptr(out), out_dtype, _ptr(ws), ws.numel(), _stream())
    _check(rc, "nvfp4_gemm_nt")
    return out


STATIC_SCRATCH_BYTES = 64 << 20
ERR_SCRATCH = -8


def gemm_nt_static(A: NVFP4Tensor, B: NVFP4Tensor, out: torch.Tensor, out_dtype: int = OUT_BF16) -> torch.Tensor:
    """nvfp4_gemm_nt_static: the product with the library's static scratch array; `out` is the caller's."""
    _check_out(out, (A.rows, B.rows), out_dtype, "out")
    ca, cb = A.c_struct(), B.c_struct()
    rc = lib().nvfp4_gemm_nt_static(C.byref(ca), C.byref(cb), _ptr(out), out_dtype, _stream())
    _check(rc, "nvfp4_gemm_nt_static")
    return out


def linear_fwd(X: torch.Tensor, W: torch.Tensor, out_dtype: int = OUT_BF16, *, Y: Optional[torch.Tensor] = None,
               Xq: Optional[NVFP4Tensor] = None, Wq: Optional[NVFP4Tensor] = None,
               ws: Optional[torch.Tensor] = None, outer: int = OUTER_TENSOR):
    _check_bf16(X, "X")
    _check_bf16(W, "W")
    N, D = X.shape
    Cc, D2 = W.shape
    assert D == D2
    dev = X.device
    Y = _out_tensor(N, Cc, out_dtype, dev) if Y is None else Y
    _check_out(Y, (N, Cc), out_dtype, "Y")
    Xq = alloc_nvfp4(N, D, outer, dev) if Xq is None else Xq
    Wq = alloc_nvfp4(Cc, D, outer, dev) if Wq is None else Wq
    ws = alloc_workspace(workspace_bytes(OP_LINEAR_FWD, N, D, Cc, outer), dev) if ws is None else ws
    cx, cw = Xq.c_struct(), Wq.c_struct()
    rc = lib().nvfp4_linear_fwd(_ptr(X), _ptr(W), N, D, Cc, _ptr(Y), out_dtype, C.byref(cx), C.byref(cw), outer,
                                _ptr(ws), ws.numel(), _stream())
    _check(rc, "nvfp4_linear_fwd")
    Xq.rows, Xq.K, Xq.outer = cx.rows, cx.K, cx.outer_mode
    Wq.rows, Wq.K, Wq.outer = cw.rows, cw.K, cw.outer_mode
    return Y, Xq, Wq


def linear_bwd_dx(dY: torch.Tensor, Wq: NVFP4Tensor, seed: int, layer_id: int, out_dtype: int = OUT_BF16, *,
                  dX: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, rht: bool = False) -> torch.Tensor:
    _check_bf16(dY, "dY")
    N, Cc = dY.shape
    D = Wq.K
    dev = dY.device
    dX = _out_tensor(N, D, out_dtype, dev) if dX is None else dX
    _check_out(dX, (N, D), out_dtype, "dX")
    ws = alloc_workspace(workspace_bytes(OP_LINEAR_BWD_DX, N, D, Cc, Wq.outer), dev) if ws is None else ws
    cw = Wq.c_struct()
    rc = lib().nvfp4_linear_bwd_dx(_ptr(dY), C.byref(cw), N, D, Cc, _ptr(dX), out_dtype, seed, layer_id, int(rht),
                                   _ptr(ws), ws.numel(), _stream())
    _check(rc, "nvfp4_linear_bwd_dx")
    return dX


def linear_bwd_dw(dY: torch.Tensor, Xq: NVFP4Tensor, seed: int, layer_id: int, out_dtype: int = OUT_BF16, *,
                  dW: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, rht: bool = False) -> torch.Tensor:
    _check_bf16(dY, "dY")
    N, Cc = dY.shape
    D = Xq.K
    dev = dY.device
    dW = _out_tensor(Cc, D, out_dtype, dev) if dW is None else dW
    _check_out(dW, (Cc, D), out_dtype, "dW")
    ws = alloc_workspace(workspace_bytes(OP_LINEAR_BWD_DW, N, D, Cc, Xq.outer), dev) if ws is None else ws
    cx = Xq.c_struct()
    rc = lib().nvfp4_linear_bwd_dw(_ptr(dY), C.byref(cx), N, D, Cc, _ptr(dW), out_dtype, seed, layer_id, int(rht),
                                   _ptr(ws), ws.numel(), _stream())
    _check(rc, "nvfp4_linear_bwd_dw")
    return dW


def linear_bwd(dY: torch.Tensor, Xq: NVFP4Tensor, Wq: NVFP4Tensor, seed: int, layer_id: int, out_dtype: int = OUT_BF16, *,
               dX: Optional[torch.Tensor] = None, dW: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
               rht: bool = False):
    """nvfp4_linear_bwd: both gradients, dY read once for its maximum and once for both quantizations."""
    _check_bf16(dY, "dY")
    N, Cc = dY.shape
    D = Xq.K
    dev = dY.device
    dX = _out_tensor(N, D, out_dtype, dev) if dX is None else dX
    dW = _out_tensor(Cc, D, out_dtype, dev) if dW is None else dW
    _check_out(dX, (N, D), out_dtype, "dX")
    _check_out(dW, (Cc, D), out_dtype, "dW")
    ws = alloc_workspace(workspace_bytes(OP_LINEAR_BWD, N, D, Cc, Xq.outer), dev) if ws is None else ws
    cx, cw = Xq.c_struct(), Wq.c_struct()
    rc = lib().nvfp4_linear_bwd(_ptr(dY), C.byref(cx), C.byref(cw), N, D, Cc, _ptr(dX), _ptr(dW), out_dtype, seed,
                                layer_id, int(rht), _ptr(ws), ws.numel(), _stream())
    _check(rc, "nvfp4_linear_bwd")
    return dX, dW


def _check_f32(t: torch.Tensor, shape, what: str):
    assert t.dtype == torch.float32 and tuple(t.shape) == tuple(shape) and t.is_contiguous() and t.is_cuda, what


def osci_update(W: torch.Tensor, W_prev: torch.Tensor, dist_m: torch.Tensor, dist_q: torch.Tensor, t0: int):
    """nvfp4_osci_update: one step of the oscillation statistics of a float32 [C, D] weight, in place."""
    Cc, D = W.shape
    for t, n in ((W, "W"), (W_prev, "W_prev"), (dist_m, "dist_m"), (dist_q, "dist_q")):
        _check_f32(t, (Cc, D), n)
    _check(lib().nvfp4_osci_update(_ptr(W), _ptr(W_prev), _ptr(dist_m), _ptr(dist_q), Cc, D, t0, _stream()), "nvfp4_osci_update")


def osci_suppress(W: torch.Tensor, dist_m: torch.Tensor, dist_q: torch.Tensor, tau: float,
                  n_reset: Optional[torch.Tensor] = None):
    """nvfp4_osci_suppress: reset the oscillating elements of W in place; n_reset (int64 [1], optional) accumulates
    their number."""
    Cc, D = W.shape
    for t, n in ((W, "W"), (dist_m, "dist_m"), (dist_q, "dist_q")):
        _check_f32(t, (Cc, D), n)
    if n_reset is not None:
        assert n_reset.dtype == torch.int64 and n_reset.numel() == 1 and n_reset.is_cuda
    _check(lib().nvfp4_osci_suppress(_ptr(W), _ptr(dist_m), _ptr(dist_q), tau, Cc, D, _ptr(n_reset), _stream()),
           "nvfp4_osci_suppress")


def _check_subset(k: int, idx, *states):
    assert idx.dtype == torch.int32 and idx.numel() == k and idx.is_contiguous() and idx.is_cuda, "idx"
    for t in states:
        assert t.dtype == torch.float32 and t.numel() == k and t.is_contiguous() and t.is_cuda, "subset state"


def osci_select(W: torch.Tensor, k: int):
    """nvfp4_osci_select (Appendix Alg. 3, first step of a period): returns (idx, W_prev_s, Q_prev_s, dist_m_s, dist_q_s)
    of the k weights with the largest sensitivity scores; idx holds 32-bit flat indices (int32 storage, read as unsigned)."""
    Cc, D = W.shape
    _check_f32(W, (Cc, D), "W")
    idx = torch.empty(k, dtype=torch.int32, device=W.device)
    st = [torch.empty(k, dtype=torch.float32, device=W.device) for _ in range(4)]
    nbytes = lib().nvfp4_osci_select_workspace_bytes(Cc, D)
    ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=W.device)
    _check(lib().nvfp4_osci_select(_ptr(W), Cc, D, k, _ptr(idx), *[_ptr(t) for t in st], _ptr(ws), ws.numel(), _stream()),
           "nvfp4_osci_select")
    return (idx, *st)


def osci_update_sparse(W, idx, W_prev_s, Q_prev_s, dist_m_s, dist_q_s):
    """nvfp4_osci_update_sparse: a later step of the period, in place on the four subset states."""
    Cc, D = W.shape
    _check_f32(W, (Cc, D), "W")
    _check_subset(idx.numel(), idx, W_prev_s, Q_prev_s, dist_m_s, dist_q_s)
    _check(lib().nvfp4_osci_update_sparse(_ptr(W), Cc, D, _ptr(idx), idx.numel(), _ptr(W_prev_s), _ptr(Q_prev_s), _ptr(dist_m_s),
                                          _ptr(dist_q_s), _stream()), "nvfp4_osci_update_sparse")


def osci_suppress_sparse(W, idx, dist_m_s, dist_q_s, tau: float, n_reset: Optional[torch.Tensor] = None):
    """nvfp4_osci_suppress_sparse: reset the oscillating tracked elements of W in place."""
    Cc, D = W.shape
    _check_f32(W, (Cc, D), "W")
    _check_subset(idx.numel(), idx, dist_m_s, dist_q_s)
    if n_reset is not None:
        assert n_reset.dtype == torch.int64 and n_reset.numel() == 1 and n_reset.is_cuda
    _check(lib().nvfp4_osci_suppress_sparse(_ptr(W), Cc, D, _ptr(idx), idx.numel(), _ptr(dist_m_s), _ptr(dist_q_s), tau,
                                            _ptr(n_reset), _stream()), "nvfp4_osci_suppress_sparse")


def outctl_fwd(X_lo, W_lo, X_hp, W_hp, out_dtype: int = OUT_BF16, *, outer: int = OUTER_TENSOR, Y=None, Xq=None, Wq=None, ws=None):
    """nvfp4_outctl_fwd: Y = Q1(X_lo) Q2(W_lo)^T + X_hp W_hp^T (Sec. 4.2); returns (Y, Xq, Wq) of the ordinary channels."""
    for t, n in ((X_lo, "X_lo"), (W_lo, "W_lo"), (X_hp, "X_hp"), (W_hp, "W_hp")):
        _check_bf16(t, n)
    N, D_lo = X_lo.shape
    Cc, D_hp = W_hp.shape
    assert W_lo.shape == (Cc, D_lo) and X_hp.shape == (N, D_hp)
    dev = X_lo.device
    Y = _out_tensor(N, Cc, out_dtype, dev) if Y is None else Y
    _check_out(Y, (N, Cc), out_dtype, "Y")
    Xq = alloc_nvfp4(N, D_lo, outer, dev) if Xq is None else Xq
    Wq = alloc_nvfp4(Cc, D_lo, outer, dev) if Wq is None else Wq
    if ws is None:
        ws = alloc_workspace(lib().nvfp4_outctl_workspace_bytes(0, N, D_lo, D_hp, Cc, outer, out_dtype), dev)
    cx, cw = Xq.c_struct(), Wq.c_struct()
    rc = lib().nvfp4_outctl_fwd(_ptr(X_lo), _ptr(W_lo), _ptr(X_hp), _ptr(W_hp), N, D_lo, D_hp, Cc, _ptr(Y), out_dtype,
                                C.byref(cx), C.byref(cw), outer, _ptr(ws), ws.numel(), _stream())
    _check(rc, "nvfp4_outctl_fwd")
    Xq.rows, Xq.K, Xq.outer = cx.rows, cx.K, cx.outer_mode
    Wq.rows, Wq.K, Wq.outer = cw.rows, cw.K, cw.outer_mode
    return Y, Xq, Wq


def outctl_bwd(dY, Xq: NVFP4Tensor, Wq: NVFP4Tensor, X_hp, W_hp, seed: int, layer_id: int, out_dtype: int = OUT_BF16, *,
               rht: bool = False, ws=None, outs=None):
    """nvfp4_outctl_bwd: returns (dX_lo, dX_hp, dW_lo, dW_hp) (written into `outs` when given)."""
    for t, n in ((dY, "dY"), (X_hp, "X_hp"), (W_hp, "W_hp")):
        _check_bf16(t, n)
    N, Cc = dY.shape
    D_lo, D_hp = Xq.K, X_hp.shape[1]
    dev = dY.device
    shapes = [(N, D_lo), (N, D_hp), (Cc, D_lo), (Cc, D_hp)]
    if outs is None:
        outs = [_out_tensor(a, b, out_dtype, dev) for a, b in shapes]
    for t, sh in zip(outs, shapes):
        _check_out(t, sh, out_dtype, "gradient output")
    if ws is None:
        ws = alloc_workspace(lib().nvfp4_outctl_workspace_bytes(1, N, D_lo, D_hp, Cc, Xq.outer, out_dtype), dev)
    cx, cw = Xq.c_struct(), Wq.c_struct()
    rc = lib().nvfp4_outctl_bwd(_ptr(dY), C.byref(cx), C.byref(cw), _ptr(X_hp), _ptr(W_hp), N, D_lo, D_hp, Cc, _ptr(outs[0]),
                                _ptr(outs[1]), _ptr(outs[2]), _ptr(outs[3]), out_dtype, seed, layer_id, int(rht), _ptr(ws),
                                ws.numel(), _stream())
    _check(rc, "nvfp4_outctl_bwd")
    return tuple(outs)
