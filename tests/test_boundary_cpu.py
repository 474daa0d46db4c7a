"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

from paper_2510_27527_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000001000      # a 16-byte aligned, never dereferenced "device pointer"


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2510_27527_amd import build
        build.build(force=True)
    return B.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tjnvfp4.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nvfp4_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert {"nvfp4_quantize", "nvfp4_linear_fwd", "nvfp4_linear_bwd_dx", "nvfp4_linear_bwd_dw"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_version_and_strerror(lib):
    assert b"gfx950" in lib.nvfp4_version()
    for code in range(0, -9, -1):
        assert lib.nvfp4_strerror(code) not in (None, b"unknown error code")
    assert lib.nvfp4_strerror(-99) == b"unknown error code"


def _tensor(rows=0, K=0, outer=0, amax=FAKE):
    return B.CTensor(FAKE, FAKE + 0x1000, FAKE + 0x2000, amax, rows, K, outer, 0)


def _quant(lib, src=FAKE, kind=0, R=32, Cc=64, axis=0, cfg=None, out=None, ws=FAKE, ws_bytes=1 << 20):
    cfg = cfg or B.CQcfg(0, 0, 0, 0, 0, None)
    out = out or _tensor()
    return lib.nvfp4_quantize(src, kind, R, Cc, axis, C.byref(cfg), C.byref(out), ws, ws_bytes, None)


def test_quantize_rejects_bad_arguments(lib):
    assert _quant(lib, src=None) == -1
    assert lib.nvfp4_quantize(FAKE, 0, 32, 64, 0, None, C.byref(_tensor()), FAKE, 1 << 20, None) == -1
    assert _quant(lib, out=B.CTensor(None, FAKE, FAKE, None, 0, 0, 0, 0)) == -1
    assert _quant(lib, Cc=24) == -2                       # K % 16
    assert _quant(lib, R=24, Cc=64, axis=1) == -2         # K = R % 16
    assert _quant(lib, R=32, Cc=20, axis=1) == -2         # C % 8 for column-wise loads
    assert _quant(lib, R=-1) == -2
    assert _quant(lib, R=1 << 20, Cc=1 << 20) == -2       # > 2^33 elements
    assert _quant(lib, Cc=64, cfg=B.CQcfg(0, 0, 1, 0, 0, None)) == -2     # BLOCK128 needs K % 128
    assert _quant(lib, kind=5) == -3
    assert _quant(lib, axis=2) == -3
    assert _quant(lib, cfg=B.CQcfg(7, 0, 0, 0, 0, None)) == -3
    assert _quant(lib, cfg=B.CQcfg(0, 9, 0, 0, 0, None)) == -3
    assert _quant(lib, cfg=B.CQcfg(0, 0, 4, 0, 0, None)) == -3
    assert _quant(lib, Cc=128, cfg=B.CQcfg(1, 0, 0, 0, 0, None, 1, 7)) == -3      # transform without 1 x 128 outer blocks
    assert _quant(lib, Cc=128, cfg=B.CQcfg(1, 0, 1, 0, 0, None, 3, 7)) == -3
    assert _quant(lib, ws=None) == -4
    assert _quant(lib, ws_bytes=16) == -4
    assert _quant(lib, src=FAKE + 2) == -5
    assert _quant(lib, out=B.CTensor(FAKE + 1, FAKE, FAKE, None, 0, 0, 0, 0)) == -5
    # NVFP4 source: descriptor must match R, C and carry the maximum
    src = _tensor(32, 64, 0)
    cfg = B.CQcfg(1, 0, 0, 0, 0, None)
    call = lambda s, R, Cc, axis: lib.nvfp4_quantize(C.cast(C.pointer(s), C.c_void_p), 1, R, Cc, axis, C.byref(cfg),
                                                     C.byref(_tensor()), FAKE, 1 << 20, None)
    assert call(src, 32, 128, 1) == -6
    assert call(_tensor(32, 64, 0, amax=None), 32, 64, 1) == -1
    assert call(src, 32, 64, 0) == -3                     # same-axis re-quantization is not provided


def test_quantize_dual_rejects_bad_arguments(lib):
    cfg = B.CQcfg(1, 0, 0, 3, 0, None)

    def call(src=FAKE, R=32, Cc=64, cfg=cfg, orow=None, ocol=None, ws=FAKE, ws_bytes=1 << 20):
        orow = _tensor() if orow is None else orow
        ocol = _tensor() if ocol is None else ocol
        return lib.nvfp4_quantize_dual(src, R, Cc, C.byref(cfg) if cfg is not None else None, 5, C.byref(orow),
                                       C.byref(ocol), ws, ws_bytes, None)
    assert call(src=None) == -1
    assert call(cfg=None) == -1
    assert call(ocol=B.CTensor(None, FAKE, FAKE, None, 0, 0, 0, 0)) == -1
    assert call(R=24) == -2                               # groups of 16 down the columns
    assert call(Cc=24) == -2                              # groups of 16 along the rows
    assert call(cfg=B.CQcfg(1, 0, 1, 3, 0, None)) == -3   # tensor mode only
    assert call(cfg=B.CQcfg(5, 0, 0, 3, 0, None)) == -3
    assert call(ws=None) == -4
    assert call(ws_bytes=8) == -4
    assert call(src=FAKE + 2) == -5


def test_gemm_and_linear_reject_bad_arguments(lib):
    A, Bt = _tensor(128, 256), _tensor(64, 256)
    g = lambda a, b, out=FAKE, dt=0, ws=FAKE, wsb=1 << 30: lib.nvfp4_gemm_nt(C.byref(a), C.byref(b), out, dt, ws, wsb, None)
    assert g(A, _tensor(64, 128)) == -6
    assert g(_tensor(128, 80), _tensor(64, 80)) == -2      # K % 64
    assert g(_tensor(128, 256, outer=1), Bt) == -6         # operands in different outer modes
    assert g(_tensor(128, 256, outer=2), Bt) == -3
    assert g(_tensor(128, 320, outer=1), _tensor(64, 320, outer=1)) == -2   # K % 128 with 1 x 128 outer blocks
    assert g(A, Bt, out=None) == -1
    assert g(A, Bt, dt=3) == -3
    assert g(A, Bt, out=FAKE + 4) == -5
    big_a, big_b = _tensor(64, 16384), _tensor(64, 16384)   # split-K needs scratch
    assert lib.nvfp4_workspace_bytes(B.OP_GEMM, 64, 16384, 64, 0) > 0
    assert g(big_a, big_b, ws=None, wsb=0) == -4

    fwd = lambda N, D, Cc, ws=FAKE, wsb=1 << 40, outer=0: lib.nvfp4_linear_fwd(
        FAKE, FAKE, N, D, Cc, FAKE, 0, C.byref(_tensor()), C.byref(_tensor()), outer, ws, wsb, None)
    assert fwd(128, 100, 64) == -2
    assert fwd(128, 128, 64, outer=2) == -3
    assert fwd(128, 192, 64, outer=1) == -2                # D % 128 with 1 x 128 outer blocks
    assert fwd(128, 128, 64, wsb=8) == -4
    assert fwd(-1, 128, 64) == -2
    W = _tensor(64, 128)
    dx = lambda N, D, Cc, w=W, wsb=1 << 40, rht=0: lib.nvfp4_linear_bwd_dx(FAKE, C.byref(w), N, D, Cc, FAKE, 0, 0, 0, rht, FAKE, wsb, None)
    assert dx(128, 128, 32) == -2                          # C % 64
    assert dx(128, 256, 64) == -6
    assert dx(128, 128, 64, wsb=100) == -4
    X = _tensor(128, 128)
    dw = lambda N, D, Cc, x=X, wsb=1 << 40, rht=0: lib.nvfp4_linear_bwd_dw(FAKE, C.byref(x), N, D, Cc, FAKE, 0, 0, 0, rht, FAKE, wsb, None)
    assert dw(96, 128, 64) == -2                           # N % 64
    assert dw(128, 64, 64) == -6
    assert dw(128, 128, 64, wsb=100) == -4
    # the random Hadamard transform comes with 1 x 128 outer blocks: tensor-mode contexts refuse it
    assert dx(128, 128, 64, rht=1) == -3 and dw(128, 128, 64, rht=1) == -3
    assert dx(128, 128, 128, w=_tensor(128, 128, outer=1), rht=2) == -3


def test_fused_backward_rejects_bad_arguments(lib):
    X, W = _tensor(128, 128), _tensor(64, 128)
    f = lambda N, D, Cc, x=X, w=W, wsb=1 << 40, rht=0: lib.nvfp4_linear_bwd(FAKE, C.byref(x), C.byref(w), N, D, Cc, FAKE, FAKE,
                                                                         0, 0, 0, rht, FAKE, wsb, None)
    assert f(128, 128, 32) == -2
    assert f(96, 128, 64) == -2
    assert f(128, 64, 64) == -6
    assert f(128, 128, 64, wsb=64) == -4
    assert lib.nvfp4_linear_bwd(None, C.byref(X), C.byref(W), 128, 128, 64, FAKE, FAKE, 0, 0, 0, 0, FAKE, 1 << 40, None) == -1
    assert f(128, 128, 64, rht=1) == -3
    assert lib.nvfp4_workspace_bytes(B.OP_LINEAR_BWD, 128, 128, 64, 0) >= \
        lib.nvfp4_workspace_bytes(B.OP_LINEAR_BWD_DX, 128, 128, 64, 0)


def test_workspace_sizes(lib):
    assert lib.nvfp4_workspace_bytes(99, 1, 1, 1, 0) == 0
    q = lib.nvfp4_workspace_bytes(B.OP_QUANTIZE, 8192, 8192, 0, 0)
    assert 0 < q <= 4096
    dx = lib.nvfp4_workspace_bytes(B.OP_LINEAR_BWD_DX, 8192, 768, 3072, 0)
    assert dx >= (8192 * 3072 + 768 * 3072) * 9 // 16


def test_stream_key_is_a_function_of_seed_and_id(lib):
    ks = {lib.nvfp4_stream_key(s, t) for s in range(8) for t in range(8)}
    assert len(ks) == 64


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N with N > 1 exits with a message instead of measuring anything."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_planner_and_workspace_accept_empty_products(lib):
    """An empty output or an empty reduction has nothing to tile: plan and workspace size come back without arithmetic
    on a zero tile count (every linear-layer call sizes its workspace through this path)."""
    for M, N, K in [(0, 64, 128), (64, 0, 128), (64, 128, 0), (0, 0, 0)]:
        bm, bn, sp = C.c_int(), C.c_int(), C.c_int()
        assert lib.nvfp4_gemm_plan(M, N, K, 0, C.byref(bm), C.byref(bn), C.byref(sp)) == 0
        assert sp.value == 1
        assert lib.nvfp4_workspace_bytes(B.OP_GEMM, M, K, N, 0) == 0
    for op in (B.OP_LINEAR_FWD, B.OP_LINEAR_BWD_DX, B.OP_LINEAR_BWD_DW, B.OP_LINEAR_BWD):
        assert lib.nvfp4_workspace_bytes(op, 0, 128, 64, 0) > 0


def test_gemm_variant_table_reaches_every_kernel_instantiation():
    """Five workgroup tiles x {single, paired} scale fetch x {one pass, K split}; the 128 x 192 tile exists for the paired
    fetch only: 18 variants, and the planner picks each for its shape in the table the GPU parity test runs over."""
    from gemm_variants import VARIANT_SHAPES
    tiles = [(128, 128), (128, 256), (256, 128), (256, 256)]
    want = {(bm, bn, ps, sp) for bm, bn in tiles for ps in (False, True) for sp in (False, True)}
    want |= {(128, 192, True, False), (128, 192, True, True)}
    assert set(VARIANT_SHAPES) == want
    for (bm, bn, ps, sp), (M, N, K) in VARIANT_SHAPES.items():
        pm, pn, split = B.gemm_plan(M, N, K)
        assert (pm, pn, K % 256 == 0, split > 1) == (bm, bn, ps, sp), (M, N, K)
        assert M % 64 and N % 4
    # operands with 1 x 128 outer blocks: three tiles x fetch x split, and the 128 x 192 tile with the paired fetch
    from gemm_variants import VARIANT_SHAPES_BLOCK128
    want = {(bm, bn, ps, sp) for bm, bn in tiles[:3] for ps in (False, True) for sp in (False, True)}
    want |= {(128, 192, True, False), (128, 192, True, True)}
    assert set(VARIANT_SHAPES_BLOCK128) == want
    for (bm, bn, ps, sp), (M, N, K) in VARIANT_SHAPES_BLOCK128.items():
        pm, pn, split = B.gemm_plan(M, N, K, B.OUTER_BLOCK128)
        assert (pm, pn, K % 256 == 0, split > 1) == (bm, bn, ps, sp), (M, N, K)
        assert M % 64 and N % 4 and K % 128 == 0


def test_static_scratch_entry_rejects_bad_arguments_and_oversized_products(lib):
    """nvfp4_gemm_nt_static validates like nvfp4_gemm_nt and, before any HIP call, refuses a product whose split
    reduction needs more scratch than the library's static array."""
    ok = _tensor(256, 512)
    assert lib.nvfp4_gemm_nt_static(None, C.byref(ok), FAKE, 0, None) == -1
    assert lib.nvfp4_gemm_nt_static(C.byref(ok), C.byref(ok), None, 0, None) == -1
    assert lib.nvfp4_gemm_nt_static(C.byref(ok), C.byref(ok), FAKE, 5, None) == -3
    assert lib.nvfp4_gemm_nt_static(C.byref(ok), C.byref(ok), FAKE + 4, 0, None) == -5
    assert lib.nvfp4_gemm_nt_static(C.byref(ok), C.byref(_tensor(256, 576)), FAKE, 0, None) == -6
    assert lib.nvfp4_gemm_nt_static(C.byref(_tensor(256, 544)), C.byref(_tensor(256, 544)), FAKE, 0, None) == -2
    assert lib.nvfp4_gemm_nt_static(C.byref(_tensor(256, 512, outer=1)), C.byref(ok), FAKE, 0, None) == -6
    big = [(M, N, K) for (M, N, K) in ((3072, 3072, 65536), (2304, 4096, 65536), (1536, 8192, 32768), (4096, 3072, 262144))
           if B.workspace_bytes(B.OP_GEMM, M, K, N) > B.STATIC_SCRATCH_BYTES]
    assert big, "no candidate shape exceeds the static scratch array any more: extend the list"
    for M, N, K in big:
        assert lib.nvfp4_gemm_nt_static(C.byref(_tensor(M, K)), C.byref(_tensor(N, K)), FAKE, 0, None) == B.ERR_SCRATCH
    assert b"static" in lib.nvfp4_strerror(B.ERR_SCRATCH)
    header = open(os.path.join(ROOT, "include", "tjnvfp4.h")).read()
    assert "#define NVFP4_STATIC_SCRATCH_BYTES (64u << 20)" in header and B.STATIC_SCRATCH_BYTES == 64 << 20


def test_osci_calls_reject_bad_arguments(lib):
    up = lambda W=FAKE, Wp=FAKE, dm=FAKE, dq=FAKE, Cc=4, D=128, t0=1: lib.nvfp4_osci_update(W, Wp, dm, dq, Cc, D, t0, None)
    assert up(W=None) == -1 and up(dq=None) == -1
    assert up(D=192) == -2 and up(Cc=-1) == -2
    assert up(Wp=FAKE + 4) == -5
    assert up(t0=-1) == -3
    sp = lambda W=FAKE, dm=FAKE, dq=FAKE, tau=8.0, Cc=4, D=128, n=None: lib.nvfp4_osci_suppress(W, dm, dq, tau, Cc, D, n, None)
    assert sp(dm=None) == -1
    assert sp(D=64) == -2
    assert sp(tau=0.0) == -3 and sp(tau=float("nan")) == -3
    assert sp(n=FAKE + 4) == -5


def test_osci_subset_calls_reject_bad_arguments(lib):
    """Appendix Alg. 3 entry points: every validation path, and the calls that have nothing to do (k = 0, empty matrix)
    return before any launch"""
    big = 1 << 40
    sel = lambda W=FAKE, Cc=4, D=128, k=8, idx=FAKE, a=FAKE, b=FAKE, c=FAKE, d=FAKE, ws=FAKE, wsb=big: lib.nvfp4_osci_select(
        W, Cc, D, k, idx, a, b, c, d, ws, wsb, None)
    assert sel(W=None) == -1 and sel(idx=None) == -1 and sel(d=None) == -1
    assert sel(D=192) == -2 and sel(k=-1) == -2 and sel(k=4 * 128 + 1) == -2 and sel(Cc=1 << 30, D=128) == -2
    assert sel(wsb=16) == -4 and sel(ws=None) == -4
    assert sel(ws=FAKE + 4) == -5 and sel(W=FAKE + 4) == -5
    assert sel(k=0, idx=None, a=None, b=None, c=None, d=None, ws=None, wsb=0) == 0
    assert sel(Cc=0, k=0, ws=None, wsb=0) == 0
    need = lib.nvfp4_osci_select_workspace_bytes(8192, 8192)
    assert need == 256 + 8192 + (8192 * 8192 // 2048) * 8
    assert lib.nvfp4_osci_select_workspace_bytes(-1, 128) == 0 and lib.nvfp4_osci_select_workspace_bytes(1 << 30, 128) == 0
    up = lambda W=FAKE, Cc=4, D=128, idx=FAKE, k=8, a=FAKE, b=FAKE, c=FAKE, d=FAKE: lib.nvfp4_osci_update_sparse(
        W, Cc, D, idx, k, a, b, c, d, None)
    assert up(W=None) == -1 and up(b=None) == -1 and up(c=None) == -1
    assert up(D=64) == -2 and up(k=513) == -2
    assert up(k=0, idx=None) == 0
    sp = lambda W=FAKE, Cc=4, D=128, idx=FAKE, k=8, a=FAKE, b=FAKE, tau=8.0, n=None: lib.nvfp4_osci_suppress_sparse(
        W, Cc, D, idx, k, a, b, tau, n, None)
    assert sp(idx=None) == -1 and sp(a=None) == -1
    assert sp(tau=-1.0) == -3 and sp(tau=float("nan")) == -3
    assert sp(n=FAKE + 4) == -5
    assert sp(k=0, idx=None, a=None, b=None) == 0


def test_outctl_calls_reject_bad_arguments(lib):
    X, W = _tensor(128, 128), _tensor(64, 128)
    fwd = lambda Xh=FAKE, D_hp=32, outer=0, wsb=1 << 40, D_lo=128: lib.nvfp4_outctl_fwd(
        FAKE, FAKE, Xh, FAKE, 128, D_lo, D_hp, 64, FAKE, 0, C.byref(_tensor()), C.byref(_tensor()), outer, FAKE, wsb, None)
    assert fwd(Xh=None) == -1
    assert fwd(D_hp=48) == -2 and fwd(D_lo=100) == -2
    assert fwd(outer=3) == -3
    assert fwd(wsb=64) == -4
    bwd = lambda D_hp=32, x=X, w=W, wsb=1 << 40, rht=0, Cc=64: lib.nvfp4_outctl_bwd(
        FAKE, C.byref(x), C.byref(w), FAKE, FAKE, 128, 128, D_hp, Cc, FAKE, FAKE, FAKE, FAKE, 0, 0, 0, rht, FAKE, wsb, None)
    assert bwd(D_hp=40) == -2 and bwd(Cc=32) == -2
    assert bwd(w=_tensor(64, 256)) == -6
    assert bwd(wsb=1000) == -4
    assert bwd(rht=1) == -3                               # per-tensor contexts: the transform is not provided
    assert lib.nvfp4_outctl_workspace_bytes(1, 128, 128, 32, 64, 0, 0) > lib.nvfp4_workspace_bytes(B.OP_LINEAR_BWD, 128, 128, 64, 0)
    assert lib.nvfp4_outctl_workspace_bytes(0, 128, 128, 32, 64, 0, 1) == lib.nvfp4_workspace_bytes(B.OP_LINEAR_FWD, 128, 128, 64, 0)
