"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times.

Every linear of a workload runs as nvfp4_linear_fwd + the fused nvfp4_linear_bwd with bf16 outputs and a
caller-supplied workspace.  Checked against the CPU oracle:
  * the forward operands Q1(X), Q2(W): every code, scale byte, outer scale and the dequantized maximum, bit for bit;
  * the backward operands Q3..Q6 (nvfp4_quantize with the layer's stream ids): every byte;
  * the fused backward's dX, dW are the bytes of the separate nvfp4_linear_bwd_dx / _dw calls;
  * Y, dX, dW on sampled rows (all columns), within 2^-8 |ref| + 1e-6 sum_k |a||b| of the oracle's float64 product of
    the same dequantized operands (bf16 output: its rounding alone is up to 2^-9 relative);
  * the first linear of every workload once more with FP32 outputs, held to the stated bound 1e-3 |ref| + 1e-6 sum_k |a||b|.
The quantizer stress tensor is compared in full.
"""
import sys

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

tj = None
SAMPLE_ROWS = 256


@pytest.fixture(scope="module", autouse=True)
def _load():
    global tj
    import paper_2510_27527_amd as mod
    tj = mod
    mod.binding.lib()          # fails loudly if the HIP library is missing
    yield


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def same_bytes(q_gpu, q_ref: oracle.NVFP4, what, check_amax=False):
    torch.cuda.synchronize()
    assert (q_gpu.rows, q_gpu.K) == (q_ref.rows, q_ref.K), what
    assert np.array_equal(q_gpu.gscale.cpu().numpy().view(np.uint32).ravel(), q_ref.gscale.view(np.uint32).ravel()), what
    sc = q_gpu.scales.cpu().numpy()
    assert np.array_equal(sc, q_ref.scales), "%s: %d scale bytes differ" % (what, int((sc != q_ref.scales).sum()))
    cd = q_gpu.codes.cpu().numpy()
    assert np.array_equal(cd, q_ref.codes), "%s: %d code bytes differ" % (what, int((cd != q_ref.codes).sum()))
    if check_amax:
        assert np.float32(q_gpu.amax_deq.cpu().numpy()[0]) == np.float32(q_ref.amax_deq), what


def product_ok(got_rows: torch.Tensor, ref, absref, what):
    g = got_rows.double().cpu().numpy()
    err = np.abs(g - ref)
    rel = 1e-3 if got_rows.dtype == torch.float32 else 2.0 ** -8
    tol = rel * np.abs(ref) + 1e-6 * absref + 1e-30
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), "%s: err %.3e tol %.3e at %s" % (what, err[worst], tol[worst], worst)


def run_full_linear(cfg, name, N, D, C, seed, kind, li, sr_seed, outer=0, rht=False):
    B = tj.binding
    cfg = cfg + ("/block128" if outer else "") + ("/rht" if rht else "")
    rid = (lambda prod: li * 16 + (7 if prod == "dx" else 8)) if rht else (lambda prod: None)
    say("[%s %s] N=%d D=%d C=%d: inputs" % (cfg, name, N, D, C))
    Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed, kind)
    X, W, dY = dev_bf16(Xb), dev_bf16(Wb), dev_bf16(dYb)
    ws = tj.alloc_workspace(max(tj.workspace_bytes(op, N, D, C, outer) for op in (B.OP_LINEAR_FWD, B.OP_LINEAR_BWD)))
    Xq, Wq = tj.alloc_nvfp4(N, D, outer), tj.alloc_nvfp4(C, D, outer)
    Y = torch.empty((N, C), dtype=torch.bfloat16, device="cuda")
    dX = torch.empty((N, D), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((C, D), dtype=torch.bfloat16, device="cuda")
    tj.linear_fwd(X, W, B.OUT_BF16, Y=Y, Xq=Xq, Wq=Wq, ws=ws, outer=outer)
    tj.linear_bwd(dY, Xq, Wq, sr_seed, li, B.OUT_BF16, dX=dX, dW=dW, ws=ws, rht=rht)
    torch.cuda.synchronize()

    say("[%s %s] oracle forward operands" % (cfg, name))
    oXq, oWq = oracle.linear_fwd(Xb, Wb, outer=outer)
    same_bytes(Xq, oXq, "Q1(X)", check_amax=True)
    same_bytes(Wq, oWq, "Q2(W)", check_amax=True)
    say("[%s %s] oracle backward operands" % (cfg, name))
    o3, o4 = oracle.linear_bwd_dx_operands(dYb, oWq, sr_seed, li, outer=outer, rht=rht)
    same_bytes(tj.quantize(dY, 0, B.ROUND_SR, seed=sr_seed, tensor_id=li * 16 + 3, outer=outer, rht_id=rid("dx")), o3, "Q3(dY)")
    same_bytes(tj.quantize(Wq, 1, B.ROUND_SR, seed=sr_seed, tensor_id=li * 16 + 4, outer=outer, rht_id=rid("dx")), o4, "Q4(W_hat)")
    o5, o6 = oracle.linear_bwd_dw_operands(dYb, oXq, sr_seed, li, outer=outer, rht=rht)
    same_bytes(tj.quantize(dY, 1, B.ROUND_SR, seed=sr_seed, tensor_id=li * 16 + 5, outer=outer, rht_id=rid("dw")), o5, "Q5(dY^T)")
    same_bytes(tj.quantize(Xq, 1, B.ROUND_SR, seed=sr_seed, tensor_id=li * 16 + 6, outer=outer, rht_id=rid("dw")), o6, "Q6(X_hat)")
    dX1 = tj.linear_bwd_dx(dY, Wq, sr_seed, li, B.OUT_BF16, rht=rht)
    dW1 = tj.linear_bwd_dw(dY, Xq, sr_seed, li, B.OUT_BF16, rht=rht)
    torch.cuda.synchronize()
    assert torch.equal(dX, dX1) and torch.equal(dW, dW1), "fused backward differs from the separate calls"

    outs = {"Y": Y, "dX": dX, "dW": dW}
    outs32 = {}
    if li == 0:
        # the same layer with FP32 outputs: the 1e-3 bound is stated on the value before any bf16 rounding
        say("[%s %s] FP32-output run" % (cfg, name))
        del dX1, dW1
        Y32, _, _ = tj.linear_fwd(X, W, B.OUT_F32, Xq=Xq, Wq=Wq, ws=ws, outer=outer)
        dX32, dW32 = tj.linear_bwd(dY, Xq, Wq, sr_seed, li, B.OUT_F32, ws=ws, rht=rht)
        torch.cuda.synchronize()
        outs32 = {"Y": Y32, "dX": dX32, "dW": dW32}
    rng = np.random.default_rng(seed)
    for pname, qa, qb in (("Y", oXq, oWq), ("dX", o3, o4), ("dW", o5, o6)):
        say("[%s %s] oracle product %s on %d sampled rows" % (cfg, name, pname, min(SAMPLE_ROWS, qa.rows)))
        rows = np.sort(rng.choice(qa.rows, min(SAMPLE_ROWS, qa.rows), replace=False))
        rows[0], rows[-1] = 0, qa.rows - 1                        # the corners are always in
        rows = np.unique(rows)
        ref, absref = oracle.gemm_nt(qa, qb, rows_a=rows)
        idx = torch.from_numpy(rows).cuda()
        product_ok(outs[pname][idx], ref, absref, "%s %s %s" % (cfg, name, pname))
        if pname in outs32:
            product_ok(outs32[pname][idx], ref, absref, "%s %s %s (FP32 output)" % (cfg, name, pname))


def _cases(cfg):
    return [pytest.param(cfg, li, id="%s-%s" % (cfg, lin[0])) for li, lin in enumerate(wl.config_linears(cfg))]


@pytest.mark.parametrize("cfg,li", _cases("cfg1_single") + _cases("cfg2_block768") + _cases("cfg3_block1024") + _cases("cfg5_square8192"))
def test_full_size_linear(cfg, li):
    name, N, D, C, seed, kind = wl.config_linears(cfg)[li]
    run_full_linear(cfg, name, N, D, C, seed, kind, li, sr_seed=0)


@pytest.mark.parametrize("cfg,li", _cases("cfg1_single") + _cases("cfg2_block768") + _cases("cfg3_block1024") + _cases("cfg5_square8192"))
def test_full_size_linear_block128(cfg, li):
    """the same workloads with the paper's 1 x 128 outer blocks on every operand (no maximum pass anywhere)"""
    name, N, D, C, seed, kind = wl.config_linears(cfg)[li]
    run_full_linear(cfg, name, N, D, C, seed, kind, li, sr_seed=0, outer=tj.binding.OUTER_BLOCK128)


@pytest.mark.parametrize("cfg,li", [pytest.param(c, 0, id=c) for c in ("cfg1_single", "cfg2_block768", "cfg3_block1024", "cfg5_square8192")])
def test_full_size_linear_block128_rht(cfg, li):
    """the first linear of every workload as TetraJet-v2-base runs it: 1 x 128 outer blocks and the random Hadamard
    transform on both operands of both backward products (Sec. 4.1)"""
    name, N, D, C, seed, kind = wl.config_linears(cfg)[li]
    run_full_linear(cfg, name, N, D, C, seed, kind, li, sr_seed=0, outer=tj.binding.OUTER_BLOCK128, rht=True)


def test_quantizer_stress_full():
    """8192 x 8192 Student-t(3) x 0.1: row-wise nearest and column-wise stochastic (seed 7), every byte."""
    B = tj.binding
    c = wl.CONFIGS["cfg4_quant_stress"]
    bits = wl.student_t_bf16((c["rows"], c["cols"]), c["nu"], c["scale"], c["seed"])
    x = dev_bf16(bits)
    say("[cfg4] row-wise nearest")
    same_bytes(tj.quantize(x, 0, B.ROUND_RTN), oracle.quantize_bf16(bits, 0, oracle.RTN), "row RTN", check_amax=True)
    say("[cfg4] column-wise stochastic")
    same_bytes(tj.quantize(x, 1, B.ROUND_SR, seed=7, tensor_id=5),
               oracle.quantize_bf16(bits, 1, oracle.SR, seed=7, tensor_id=5), "col SR")
    say("[cfg4] row-wise + column-wise stochastic from one read")
    row, col = tj.quantize_dual(x, B.ROUND_SR, seed=7, tensor_id_row=3, tensor_id_col=5)
    same_bytes(row, oracle.quantize_bf16(bits, 0, oracle.SR, seed=7, tensor_id=3), "dual row SR")
    same_bytes(col, oracle.quantize_bf16(bits, 1, oracle.SR, seed=7, tensor_id=5), "dual col SR")
    say("[cfg4] column-wise stochastic, 1 x 128 outer blocks")
    same_bytes(tj.quantize(x, 1, B.ROUND_SR, seed=7, tensor_id=5, outer=B.OUTER_BLOCK128),
               oracle.quantize_bf16(bits, 1, oracle.SR, seed=7, tensor_id=5, outer=oracle.OUTER_BLOCK128), "col SR block128")
    say("[cfg4] row-wise stochastic, 1 x 128 outer blocks")
    same_bytes(tj.quantize(x, 0, B.ROUND_SR, seed=7, tensor_id=3, outer=B.OUTER_BLOCK128),
               oracle.quantize_bf16(bits, 0, oracle.SR, seed=7, tensor_id=3, outer=oracle.OUTER_BLOCK128), "row SR block128")
