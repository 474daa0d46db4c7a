"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads ``nvfp4_oracle.c`` (built with gcc into ``oracle/libnvfp4_oracle.so``) through
ctypes and composes its primitives into the quantizers and the three matrix
products of the NVFP4 linear layer (TetraJet-v2, Sec. 2.1-2.3).  Only tests/, the
smoke check and the bench's ``cpu_baseline`` leg may import this package; it does
not import the GPU package and the GPU package does not import it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nvfp4_oracle.c")
_SO = os.path.join(_HERE, "libnvfp4_oracle.so")

RTN, SR = 0, 1
SCALE_DEFAULT, SCALE_NE, SCALE_UP = 0, 1, 2
OUTER_TENSOR, OUTER_BLOCK128 = 0, 1

FP4_VALUES = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
               "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        p, i64, i32, u64, u32, f32 = C.c_void_p, C.c_int64, C.c_int, C.c_uint64, C.c_uint32, C.c_float
        L.oracle_e4m3_value.restype = f32
        L.oracle_e4m3_value.argtypes = [C.c_uint8]
        L.oracle_e4m3_round.restype = C.c_uint8
        L.oracle_e4m3_round.argtypes = [f32, i32]
        L.oracle_stream_key.restype = u64
        L.oracle_stream_key.argtypes = [u64, u32]
        L.oracle_quad_bits.restype = u32
        L.oracle_quad_bits.argtypes = [u32, u64]
        L.oracle_rand22.restype = u32
        L.oracle_rand22.argtypes = [u64, u64]
        L.oracle_round_sr_count_up.restype = i64
        L.oracle_round_sr_count_up.argtypes = [f32, C.POINTER(C.c_int)]
        L.oracle_round_rtn.restype = i32
        L.oracle_round_rtn.argtypes = [f32]
        L.oracle_round_sr.restype = i32
        L.oracle_round_sr.argtypes = [f32, u32]
        L.oracle_global_scale.restype = f32
        L.oracle_global_scale.argtypes = [f32]
        L.oracle_quantize_rows.restype = i32
        L.oracle_quantize_rows.argtypes = [p, i64, i64, i32, i32, i32, u64, u32, p, p, p, p]
        L.oracle_quantize_rows_y.restype = i32
        L.oracle_quantize_rows_y.argtypes = [p, i64, i64, i32, i32, i32, u64, u32, p, p, p, p, p]
        L.oracle_quantize_rows_slice.restype = i32
        L.oracle_quantize_rows_slice.argtypes = [p, i64, i64, i32, i32, i32, u64, u32, i64, f32, p, p, p]
        L.oracle_rand22_fill.restype = None
        L.oracle_rand22_fill.argtypes = [u64, i64, p]
        L.oracle_rht_sign.restype = i32
        L.oracle_rht_sign.argtypes = [u64, u64]
        L.oracle_rht16_rows.restype = i32
        L.oracle_rht16_rows.argtypes = [p, i64, i64, u64]
        L.oracle_quant_dequant_weight.restype = i32
        L.oracle_quant_dequant_weight.argtypes = [p, i64, i64, p]
        L.oracle_osci_update.restype = i32
        L.oracle_osci_update.argtypes = [p, p, p, p, i64, i64, i32]
        L.oracle_osci_suppress.restype = i64
        L.oracle_osci_suppress.argtypes = [p, p, p, f32, i64, i64]
        L.oracle_osci_scores.restype = i32
        L.oracle_osci_scores.argtypes = [p, i64, i64, p, p]
        L.oracle_dequant_f32.restype = i32
        L.oracle_dequant_f32.argtypes = [p, p, p, i64, i64, i32, p]
        L.oracle_dequant_f64.restype = i32
        L.oracle_dequant_f64.argtypes = [p, p, p, i64, i64, i32, p]
        L.oracle_gemm_nt_f64.restype = i32
        L.oracle_gemm_nt_f64.argtypes = [p, p, i64, i64, i64, p, p]
        L.oracle_bf16_to_f32.restype = None
        L.oracle_bf16_to_f32.argtypes = [p, i64, p]
        L.oracle_transpose_f32.restype = None
        L.oracle_transpose_f32.argtypes = [p, i64, i64, p]
        L.oracle_abs_max_f32.restype = f32
        L.oracle_abs_max_f32.argtypes = [p, i64]
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


@dataclass
class NVFP4:
    """One quantized operand, K contiguous: codes [rows, K/2], scales [rows, K/16]."""
    codes: np.ndarray
    scales: np.ndarray
    gscale: np.ndarray          # [1] (TENSOR) or [rows, K/128] (BLOCK128)
    amax_deq: float
    rows: int
    K: int
    outer: int


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    out = np.empty(bits.shape, dtype=np.float32)
    lib().oracle_bf16_to_f32(_ptr(bits), bits.size, _ptr(out))
    return out


def transpose_f32(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    R, Cc = x.shape
    out = np.empty((Cc, R), dtype=np.float32)
    lib().oracle_transpose_f32(_ptr(x), R, Cc, _ptr(out))
    return out


def rht16(x: np.ndarray, seed: int, rht_id: int) -> np.ndarray:
    """x S H_16 along the last axis of a float32 [rows, K] array (Sec. 4.1); the signs are those of stream
    (seed, rht_id) and depend on the position along K only."""
    x = np.array(x, dtype=np.float32, order="C", copy=True)
    rows, K = x.shape
    rc = lib().oracle_rht16_rows(_ptr(x), rows, K, lib().oracle_stream_key(seed, rht_id))
    if rc != 0:
        raise ValueError("oracle_rht16_rows: bad shape")
    return x


def quantize_f32(x: np.ndarray, rounding: int, scale_round: int = SCALE_DEFAULT,
                 outer: int = OUTER_TENSOR, seed: int = 0, tensor_id: int = 0, rht_id=None) -> NVFP4:
    """Quantize a float32 [rows, K] view along K (Sec. 2.2); with rht_id, after the random Hadamard transform of
    Sec. 4.1 along K (signs of stream (seed, rht_id))."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if rht_id is not None:
        x = rht16(x, seed, rht_id)
    rows, K = x.shape
    codes = np.zeros((rows, K // 2), dtype=np.uint8)
    scales = np.zeros((rows, K // 16), dtype=np.uint8)
    gscale = np.zeros((1,) if outer == OUTER_TENSOR else (rows, K // 128), dtype=np.float32)
    amax_deq = C.c_float(0.0)
    rc = lib().oracle_quantize_rows(_ptr(x), rows, K, rounding, scale_round, outer,
                                    seed, tensor_id, _ptr(codes), _ptr(scales), _ptr(gscale),
                                    C.cast(C.byref(amax_deq), C.c_void_p))
    if rc != 0:
        raise ValueError("oracle_quantize_rows: bad shape or enum")
    return NVFP4(codes, scales, gscale, float(amax_deq.value), rows, K, outer)


def quantize_f32_slice(x: np.ndarray, row0: int, tensor_amax: float, rounding: int, scale_round: int = SCALE_DEFAULT,
                       seed: int = 0, tensor_id: int = 0) -> NVFP4:
    """Rows row0 .. row0 + len(x) - 1 of a larger [*, K] tensor with max |.| = tensor_amax (per-tensor outer scale):
    the bytes those rows have in the whole tensor's quantization (sampled checks on tensors too large to do whole)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    rows, K = x.shape
    codes = np.zeros((rows, K // 2), dtype=np.uint8)
    scales = np.zeros((rows, K // 16), dtype=np.uint8)
    gscale = np.zeros((1,), dtype=np.float32)
    rc = lib().oracle_quantize_rows_slice(_ptr(x), rows, K, rounding, scale_round, OUTER_TENSOR, seed, tensor_id,
                                          row0, tensor_amax, _ptr(codes), _ptr(scales), _ptr(gscale))
    if rc != 0:
        raise ValueError("oracle_quantize_rows_slice: bad shape or enum")
    return NVFP4(codes, scales, gscale, float("nan"), rows, K, OUTER_TENSOR)


def quantize_bf16(src_bits: np.ndarray, axis: int, rounding: int, **kw) -> NVFP4:
    """Quantize a bf16 [R, C] tensor row-wise (axis=0: K=C) or column-wise
    (axis=1: K=R, the result describes the transpose [C, R]); Sec. 2.3 group shapes."""
    x = bf16_to_f32(src_bits)
    if axis == 1:
        x = transpose_f32(x)
    return quantize_f32(x, rounding, **kw)


def dequant_f32(q: NVFP4) -> np.ndarray:
    out = np.empty((q.rows, q.K), dtype=np.float32)
    rc = lib().oracle_dequant_f32(_ptr(q.codes), _ptr(q.scales), _ptr(q.gscale), q.rows, q.K, q.outer, _ptr(out))
    assert rc == 0
    return out


def dequant_f64(q: NVFP4, rows=None) -> np.ndarray:
    """Exact dequantized values; ``rows`` optionally selects a subset of rows."""
    if rows is not None:
        rows = np.asarray(rows)
        gs = q.gscale if q.outer == OUTER_TENSOR else np.ascontiguousarray(q.gscale[rows])
        q = NVFP4(np.ascontiguousarray(q.codes[rows]), np.ascontiguousarray(q.scales[rows]), gs,
                  q.amax_deq, len(rows), q.K, q.outer)
    out = np.empty((q.rows, q.K), dtype=np.float64)
    rc = lib().oracle_dequant_f64(_ptr(q.codes), _ptr(q.scales), _ptr(q.gscale), q.rows, q.K, q.outer, _ptr(out))
    assert rc == 0
    return out


def requantize(q: NVFP4, axis: int, rounding: int, **kw) -> NVFP4:
    """Quantize an NVFP4 tensor again (Q4 / Q6 of Sec. 2.3) from its binary32 dequantized value."""
    x = dequant_f32(q)
    if axis == 1:
        x = transpose_f32(x)
    return quantize_f32(x, rounding, **kw)


def gemm_nt_f64(A: np.ndarray, B: np.ndarray):
    """C = A @ B.T in binary64 with sequential k; also returns sum_k |a||b|."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    B = np.ascontiguousarray(B, dtype=np.float64)
    M, K = A.shape
    N, K2 = B.shape
    assert K == K2
    Cm = np.empty((M, N), dtype=np.float64)
    Ab = np.empty((M, N), dtype=np.float64)
    lib().oracle_gemm_nt_f64(_ptr(A), _ptr(B), M, N, K, _ptr(Cm), _ptr(Ab))
    return Cm, Ab


def gemm_nt(qa: NVFP4, qb: NVFP4, rows_a=None, rows_b=None):
    """Quantized NT product of two operands (optionally on sampled rows of A and / or B)."""
    assert qa.K == qb.K
    return gemm_nt_f64(dequant_f64(qa, rows_a), dequant_f64(qb, rows_b))


def tensor_id(layer_id: int, quantizer_index: int) -> int:
    """Stream id of quantizer Q^(k) of a layer (k = 1..6 as numbered in Sec. 2.3)."""
    return layer_id * 16 + quantizer_index


# ----- the linear layer of Sec. 2.3 ------------------------------------------------------

def linear_fwd(X_bits, W_bits, outer: int = OUTER_TENSOR):
    """Y = Q1_D(X) x Q2_D(W^T): returns (Xq, Wq); both are grouped along D."""
    Xq = quantize_bf16(X_bits, 0, RTN, outer=outer)
    Wq = quantize_bf16(W_bits, 0, RTN, outer=outer)
    return Xq, Wq


def rht_id(layer_id: int, product: str):
    """Stream id of the random signs of a layer's backward product (Sec. 4.1): "dx" (signs along C) or "dw" (along N)."""
    return layer_id * 16 + (7 if product == "dx" else 8)


def linear_bwd_dx_operands(dY_bits, Wq: NVFP4, seed: int, layer_id: int, outer: int = OUTER_TENSOR, rht: bool = False):
    """dX = Q3_S(dY) x Q4_S(W_hat): returns (dYq [N, C], Wq' [D, C]), both grouped along C; with rht, both operands
    are transformed along C with the same signs first (Sec. 4.1/4.2: Q3(dY S H), Q4(H^T S^T W_hat))."""
    rid = rht_id(layer_id, "dx") if rht else None
    dYq = quantize_bf16(dY_bits, 0, SR, outer=outer, seed=seed, tensor_id=tensor_id(layer_id, 3), rht_id=rid)
    Wq2 = requantize(Wq, 1, SR, outer=outer, seed=seed, tensor_id=tensor_id(layer_id, 4), rht_id=rid)
    return dYq, Wq2


def linear_bwd_dw_operands(dY_bits, Xq: NVFP4, seed: int, layer_id: int, outer: int = OUTER_TENSOR, rht: bool = False):
    """dW = Q5_S(dY^T) x Q6_S(X_hat): returns (dYq' [C, N], Xq' [D, N]), both grouped along N; with rht, both are
    transformed along N with the same signs first."""
    rid = rht_id(layer_id, "dw") if rht else None
    dYq = quantize_bf16(dY_bits, 1, SR, outer=outer, seed=seed, tensor_id=tensor_id(layer_id, 5), rht_id=rid)
    Xq2 = requantize(Xq, 1, SR, outer=outer, seed=seed, tensor_id=tensor_id(layer_id, 6), rht_id=rid)
    return dYq, Xq2


# ----- OsciReset (Sec. 3.2-3.3; Alg. 1 and Appendix Alg. 2) ---------------------------------

def quant_dequant_weight(W: np.ndarray) -> np.ndarray:
    """Q(W): a binary32 [C, D] weight through the forward weight quantizer (groups along D, nearest, 1 x 128 outer
    blocks) and back to binary32."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    out = np.empty_like(W)
    if lib().oracle_quant_dequant_weight(_ptr(W), W.shape[0], W.shape[1], _ptr(out)) != 0:
        raise ValueError("oracle_quant_dequant_weight: bad shape")
    return out


def osci_update(W, W_prev, dist_m, dist_q, t0: int):
    """Appendix Alg. 2, in place on W_prev, dist_m, dist_q (float32, C-contiguous [C, D])."""
    for a in (W, W_prev, dist_m, dist_q):
        assert a.dtype == np.float32 and a.flags.c_contiguous and a.shape == W.shape
    if lib().oracle_osci_update(_ptr(W), _ptr(W_prev), _ptr(dist_m), _ptr(dist_q), W.shape[0], W.shape[1], t0) != 0:
        raise ValueError("oracle_osci_update: bad shape")


def osci_suppress(W, dist_m, dist_q, tau: float) -> int:
    """Alg. 1, in place on W; returns the number of elements reset."""
    for a in (W, dist_m, dist_q):
        assert a.dtype == np.float32 and a.flags.c_contiguous and a.shape == W.shape
    n = lib().oracle_osci_suppress(_ptr(W), _ptr(dist_m), _ptr(dist_q), tau, W.shape[0], W.shape[1])
    if n < 0:
        raise ValueError("oracle_osci_suppress: bad shape")
    return int(n)


def osci_scores(W):
    """Appendix Alg. 3: (Q(W), sensitivity score |W - Q(W)| / binwidth(Q(W))) of every element, binary32."""
    assert W.dtype == np.float32 and W.flags.c_contiguous and W.ndim == 2
    q, s = np.empty_like(W), np.empty_like(W)
    if lib().oracle_osci_scores(_ptr(W), W.shape[0], W.shape[1], _ptr(q), _ptr(s)) != 0:
        raise ValueError("oracle_osci_scores: bad shape")
    return q, s


def osci_select(W, k: int):
    """Appendix Alg. 3 at the first step of a period: the k elements with the largest sensitivity scores (equal scores in
    ascending index order), as an ascending list of flat indices, with the states of the tracked subset:
    (idx u32 [k], master snapshot, quantized snapshot, dist_M = 0, dist_Q = 0)."""
    q, s = osci_scores(W)
    order = np.argsort(-s.reshape(-1), kind="stable")[:k]         # stable: equal scores keep ascending index order
    idx = np.sort(order).astype(np.uint32)
    z = np.zeros(k, np.float32)
    return idx, W.reshape(-1)[idx].copy(), q.reshape(-1)[idx].copy(), z, z.copy()


def osci_update_sparse(W, idx, W_prev_s, Q_prev_s, dist_m_s, dist_q_s) -> None:
    """Appendix Alg. 3 at a later step, in place on the four subset states: the distances grow by the moves of the
    tracked master weights and of their quantized values, then the snapshots are replaced."""
    q = quant_dequant_weight(W).reshape(-1)[idx]
    w = W.reshape(-1)[idx]
    dist_m_s += np.abs(w - W_prev_s)                              # binary32 throughout: one rounding per operation
    dist_q_s += np.abs(q - Q_prev_s)
    W_prev_s[:] = w
    Q_prev_s[:] = q


def osci_suppress_sparse(W, idx, dist_m_s, dist_q_s, tau: float) -> int:
    """Alg. 1 on the tracked subset, in place on W: a tracked element whose risk dist_Q / dist_M reaches tau is reset to
    Q(W) at that element; returns the number of resets."""
    q = quant_dequant_weight(W).reshape(-1)
    with np.errstate(divide="ignore", invalid="ignore"):
        risk = dist_q_s / dist_m_s                                # binary32 quotient; 0 / 0 is NaN and compares false
        hit = risk >= np.float32(tau)
    flat = W.reshape(-1)
    flat[idx[hit]] = q[idx[hit]]
    return int(hit.sum())


# ----- OutControl split linear (Sec. 4.2) -------------------------------------------------------

def outctl_fwd(X_lo_bits, W_lo_bits, X_hp_bits, W_hp_bits, outer: int = OUTER_TENSOR):
    """Y = Q1(X_lo) x Q2(W_lo^T) + X_hp x W_hp^T: returns (Xq, Wq, Y, abs) with Y in binary64 (the bf16 values of the
    outlier channels are exact there) and abs = sum_k |a||b| over both terms (for tolerance scaling)."""
    Xq, Wq = linear_fwd(X_lo_bits, W_lo_bits, outer=outer)
    Y, Ab = gemm_nt(Xq, Wq)
    Xh, Wh = bf16_to_f32(X_hp_bits).astype(np.float64), bf16_to_f32(W_hp_bits).astype(np.float64)
    if Xh.shape[1]:
        Yh, Abh = gemm_nt_f64(Xh, Wh)
        Y, Ab = Y + Yh, Ab + Abh
    return Xq, Wq, Y, Ab


def outctl_bwd(dY_bits, Xq: NVFP4, Wq: NVFP4, X_hp_bits, W_hp_bits, seed: int, layer_id: int, rht: bool = False):
    """The four gradients of the split layer, each as (value, abs) in binary64:
    dX_lo = Q3(dY) x Q4(W_hat_lo), dX_hp = Q3(dY) x Q4(W_hp) (NVFP4, one Q3 operand),
    dW_lo = Q5(dY^T) x Q6(X_hat_lo) (NVFP4), dW_hp = dY^T x X_hp (bf16 values, exact products)."""
    outer = Xq.outer
    o3, o4 = linear_bwd_dx_operands(dY_bits, Wq, seed, layer_id, outer=outer, rht=rht)
    o5, o6 = linear_bwd_dw_operands(dY_bits, Xq, seed, layer_id, outer=outer, rht=rht)
    res = {"dX_lo": gemm_nt(o3, o4), "dW_lo": gemm_nt(o5, o6)}
    if X_hp_bits.shape[1]:
        o4h = quantize_bf16(W_hp_bits, 1, SR, outer=outer, seed=seed, tensor_id=tensor_id(layer_id, 9),
                            rht_id=rht_id(layer_id, "dx") if rht else None)
        res["dX_hp"] = gemm_nt(o3, o4h)
        dYT = np.ascontiguousarray(bf16_to_f32(dY_bits).astype(np.float64).T)
        XhT = np.ascontiguousarray(bf16_to_f32(X_hp_bits).astype(np.float64).T)
        res["dW_hp"] = gemm_nt_f64(dYT, XhT)
    return res
