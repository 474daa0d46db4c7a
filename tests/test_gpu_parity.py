"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Bar: codes, E4M3 scale bytes, FP32 outer scales and stochastic-rounding outcomes are bit-exact;
matrix products satisfy |c - ref| <= 1e-3 |ref| + 1e-6 sum_k |a||b| on the FP32 output (the
second term covers cancellation) and 2^-8 |ref| + the same floor on the bf16 output (bf16
rounding alone is up to 2^-9 relative).
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

tj = None


@pytest.fixture(scope="module", autouse=True)
def _load():
    global tj
    import paper_2510_27527_amd as mod
    tj = mod
    mod.binding.lib()          # fails loudly if the HIP library is missing
    yield


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_dev(q: oracle.NVFP4):
    t = tj.alloc_nvfp4(q.rows, q.K, q.outer)
    t.codes.copy_(torch.from_numpy(q.codes))
    t.scales.copy_(torch.from_numpy(q.scales))
    t.gscale.copy_(torch.from_numpy(q.gscale))
    t.amax_deq.fill_(q.amax_deq)
    return t


def assert_same(q_gpu, q_ref: oracle.NVFP4, what="", check_amax=False):
    torch.cuda.synchronize()
    assert (q_gpu.rows, q_gpu.K) == (q_ref.rows, q_ref.K), what
    gs = q_gpu.gscale.cpu().numpy()
    assert np.array_equal(gs.view(np.uint32).ravel(), q_ref.gscale.view(np.uint32).ravel()), what + " gscale"
    sc = q_gpu.scales.cpu().numpy()
    bad = np.argwhere(sc != q_ref.scales)
    assert len(bad) == 0, "%s scales differ at %s (%d total)" % (what, bad[:5].tolist(), len(bad))
    cd = q_gpu.codes.cpu().numpy()
    bad = np.argwhere(cd != q_ref.codes)
    assert len(bad) == 0, "%s codes differ at %s (%d total): gpu %s ref %s" % (
        what, bad[:5].tolist(), len(bad), cd[tuple(bad[0])] if len(bad) else None,
        q_ref.codes[tuple(bad[0])] if len(bad) else None)
    if check_amax:
        a = float(q_gpu.amax_deq.cpu().numpy()[0])
        assert np.float32(a) == np.float32(q_ref.amax_deq), (what, a, q_ref.amax_deq)


def check_product(got: torch.Tensor, ref: np.ndarray, absref: np.ndarray, what=""):
    g = got.double().cpu().numpy()
    rel = 1e-3 if got.dtype == torch.float32 else 2.0 ** -8
    err = np.abs(g - ref)
    tol = rel * np.abs(ref) + 1e-6 * absref + 1e-30
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), "%s: err %.3e tol %.3e at %s (ref %.6e got %.6e)" % (
        what, err[worst], tol[worst], worst, ref[worst], g[worst])


ROW_SHAPES = [(256, 512), (1, 16), (3, 48), (100, 48), (37, 1040), (520, 2048)]
COL_SHAPES = [(256, 512), (16, 8), (144, 72), (1040, 136), (272, 1024)]


# ------------------------------------------------------------------ quantizers

def test_amax():
    for shape, seed in [((256, 512), 1), ((3, 16), 2), ((1000, 1000), 3), ((4096, 4096), 4)]:
        bits = wl.student_t_bf16(shape, 3.0, 0.1, seed)
        ws = tj.alloc_workspace(tj.workspace_bytes(tj.binding.OP_QUANTIZE, shape[0], shape[1], 0))
        got = float(tj.amax_bf16(dev_bf16(bits), ws).cpu()[0])
        assert got == float(np.abs(wl.bf16_to_f32(bits)).max())


@pytest.mark.parametrize("shape", ROW_SHAPES)
@pytest.mark.parametrize("rounding,scale_round", [(0, 0), (0, 2), (1, 0), (1, 1)])
def test_quant_row_tensor_mode(shape, rounding, scale_round):
    bits = wl.normal_bf16(shape, 1.0, 100 + shape[0], 1e-2, 50.0)
    ref = oracle.quantize_bf16(bits, 0, rounding, scale_round=scale_round, seed=5, tensor_id=9)
    got = tj.quantize(dev_bf16(bits), 0, rounding, scale_round=scale_round, seed=5, tensor_id=9)
    assert_same(got, ref, "row %s r%d s%d" % (shape, rounding, scale_round), check_amax=(rounding == 0))


@pytest.mark.parametrize("shape", [(8, 128), (5, 384), (130, 1152)])
@pytest.mark.parametrize("rounding", [0, 1])
def test_quant_row_block128_mode(shape, rounding):
    bits = wl.student_t_bf16(shape, 3.0, 0.1, 200 + shape[0])
    x = bits.copy()
    x[0, :128] = 0                     # an all-zero outer block
    ref = oracle.quantize_bf16(x, 0, rounding, outer=oracle.OUTER_BLOCK128, seed=6, tensor_id=1)
    got = tj.quantize(dev_bf16(x), 0, rounding, outer=tj.binding.OUTER_BLOCK128, seed=6, tensor_id=1)
    assert_same(got, ref, "row128 %s r%d" % (shape, rounding), check_amax=(rounding == 0))


def test_quant_row_amax_supplied_and_edge_values():
    bits = wl.student_t_bf16((64, 256), 3.0, 0.1, 300)
    bits[3, 16:32] = 0                 # zero group
    bits[4, :] = 0x8000                # a row of -0
    ref = oracle.quantize_bf16(bits, 0, 0)
    x = dev_bf16(bits)
    ws = tj.alloc_workspace(4096)
    amax = tj.amax_bf16(x, ws)
    got = tj.quantize(x, 0, 0, amax_in=amax)
    assert_same(got, ref, "amax_in")
    z = np.zeros((4, 64), dtype=np.uint16)
    assert_same(tj.quantize(dev_bf16(z), 0, 1, seed=1), oracle.quantize_bf16(z, 0, 1, seed=1), "zeros")
    # deterministic rounding also reports the largest dequantized magnitude (what a later re-quantization takes as its
    # tensor maximum): 0 for an all-zero tensor, and for a floored outer scale (maximum below 2688 * 2^-100) the
    # reduction over all groups instead of the closed form
    zq = tj.quantize(dev_bf16(z), 0, 0)
    zq.amax_deq.fill_(123.0)                       # stale value: the call must overwrite it
    assert_same(tj.quantize(dev_bf16(z), 0, 0, zq), oracle.quantize_bf16(z, 0, 0), "zeros nearest", check_amax=True)
    tiny = wl.f32_to_bf16(np.full((2, 32), 1e-38, dtype=np.float32))
    assert_same(tj.quantize(dev_bf16(tiny), 0, 0), oracle.quantize_bf16(tiny, 0, 0), "tiny", check_amax=True)
    rng = np.random.default_rng(301)
    tiny2 = wl.f32_to_bf16((rng.uniform(0.1, 1.0, (300, 128)) * 1e-28).astype(np.float32))     # several workgroups
    ref = oracle.quantize_bf16(tiny2, 0, 0)
    assert ref.gscale[0] == np.float32(2.0 ** -100) and ref.amax_deq > 0
    assert_same(tj.quantize(dev_bf16(tiny2), 0, 0), ref, "tiny, many groups", check_amax=True)
    huge = wl.f32_to_bf16(np.full((2, 32), 3e38, dtype=np.float32))
    assert_same(tj.quantize(dev_bf16(huge), 0, 0), oracle.quantize_bf16(huge, 0, 0), "huge")


def test_every_bf16_value_up_to_six_as_rounding_argument():
    """Tensor maximum 2688 and group maximum 6 make S_global = S_block = 1, so the rounding functions
    see every bf16 value in [-6, 6] exactly (all ties included)."""
    vals = np.arange(0, 0x40C1, dtype=np.uint16)               # 0 .. 6.0
    vals = np.concatenate([vals, vals | 0x8000])
    pad = (-len(vals)) % 15
    vals = np.concatenate([vals, np.zeros(pad, dtype=np.uint16)])
    blocks = vals.reshape(-1, 15)
    six = np.full((blocks.shape[0], 1), 0x40C0, dtype=np.uint16)
    body = np.concatenate([blocks, six], axis=1).reshape(-1)
    lead = np.zeros(16, dtype=np.uint16)
    lead[0] = wl.f32_to_bf16(np.array([2688.0], dtype=np.float32))[0]
    flat = np.concatenate([lead, body])
    pad = (-len(flat)) % 64
    flat = np.concatenate([flat, np.zeros(pad, dtype=np.uint16)])
    bits = flat.reshape(-1, 64)
    for rounding, sr in [(0, 1), (0, 2), (1, 2), (1, 1)]:
        for seed in (0, 1):
            ref = oracle.quantize_bf16(bits, 0, rounding, scale_round=sr, seed=seed, tensor_id=2)
            assert ref.gscale[0] == 1.0 and ref.scales[0, 1] == 0x38
            got = tj.quantize(dev_bf16(bits), 0, rounding, scale_round=sr, seed=seed, tensor_id=2)
            assert_same(got, ref, "all-bf16 r%d" % rounding)


def test_every_scale_code_is_reachable_and_exact():
    """Group maxima 6 * v for every E4M3 value v (tensor maximum 2688): the scale byte must be v's code."""
    L = oracle.lib()
    codes = np.arange(1, 0x7F)
    v = np.array([L.oracle_e4m3_value(int(c)) for c in codes], dtype=np.float32)
    x = np.zeros((len(codes), 16), dtype=np.float32)
    x[:, 3] = 6.0 * v
    x[:, 7] = -2.0 * v
    x[-1, 3] = 2688.0
    bits = wl.f32_to_bf16(x)
    assert np.array_equal(wl.bf16_to_f32(bits), x)
    for rounding in (0, 1):
        ref = oracle.quantize_bf16(bits, 0, rounding, seed=3)
        assert np.array_equal(ref.scales[:, 0], codes.astype(np.uint8))
        got = tj.quantize(dev_bf16(bits), 0, rounding, seed=3)
        assert_same(got, ref, "scale codes")


@pytest.mark.parametrize("shape", COL_SHAPES)
@pytest.mark.parametrize("rounding", [0, 1])
def test_quant_col(shape, rounding):
    bits = wl.normal_bf16(shape, 1e-3, 400 + shape[0], 1e-2, 30.0)
    ref = oracle.quantize_bf16(bits, 1, rounding, seed=8, tensor_id=5)
    got = tj.quantize(dev_bf16(bits), 1, rounding, seed=8, tensor_id=5)
    assert_same(got, ref, "col %s r%d" % (shape, rounding))


@pytest.mark.parametrize("shape", [(128, 8), (256, 512), (384, 136), (1152, 1040), (2048, 72)])
@pytest.mark.parametrize("rounding", [0, 1])
def test_quant_col_block128_mode(shape, rounding):
    """column-wise with the paper's 1 x 128 outer blocks (along the source's rows): single pass, no tensor maximum"""
    bits = wl.student_t_bf16(shape, 3.0, 0.1, 450 + shape[1])
    bits[:128, 0] = 0                  # an all-zero outer block
    bits[16:32, 2] = 0                 # an all-zero inner block
    ref = oracle.quantize_bf16(bits, 1, rounding, outer=oracle.OUTER_BLOCK128, seed=8, tensor_id=4)
    got = tj.quantize(dev_bf16(bits), 1, rounding, outer=tj.binding.OUTER_BLOCK128, seed=8, tensor_id=4)
    assert_same(got, ref, "col128 %s r%d" % (shape, rounding))


@pytest.mark.parametrize("shape", [(128, 128), (256, 512), (384, 1152), (1024, 256)])
@pytest.mark.parametrize("src_outer,out_outer", [(1, 1), (0, 1), (1, 0)])
@pytest.mark.parametrize("rounding", [0, 1])
def test_requant_col_outer_modes(shape, src_outer, out_outer, rounding):
    """re-quantization of a packed tensor along its other axis with 1 x 128 outer blocks on the source, the output,
    or both (the backward operands Q4 / Q6 of a layer whose operands carry the paper's outer scale)"""
    bits = wl.normal_bf16(shape, 1.0, 460 + shape[0], 1e-2, 50.0)
    bits[5, 128:256] = 0 if shape[1] >= 256 else bits[5, 128:256]
    src_ref = oracle.quantize_bf16(bits, 0, 0, outer=src_outer)
    ref = oracle.requantize(src_ref, 1, rounding, outer=out_outer, seed=17, tensor_id=6)
    src = tj.quantize(dev_bf16(bits), 0, 0, outer=src_outer)
    assert_same(src, src_ref, "source", check_amax=True)
    got = tj.quantize(src, 1, rounding, outer=out_outer, seed=17, tensor_id=6)
    assert_same(got, ref, "requant %s src%d out%d r%d" % (shape, src_outer, out_outer, rounding))


@pytest.mark.parametrize("shape", [(256, 512), (16, 16), (144, 80), (1040, 144), (272, 1024), (528, 2064)])
@pytest.mark.parametrize("rounding", [0, 1])
def test_quantize_dual_equals_both_quantizations(shape, rounding):
    """One read of the tensor, both backward operands: the bytes of the row-wise and of the column-wise call."""
    bits = wl.normal_bf16(shape, 1e-3, 31)
    x = dev_bf16(bits)
    row, col = tj.quantize_dual(x, rounding, seed=9, tensor_id_row=11, tensor_id_col=13)
    assert_same(row, oracle.quantize_bf16(bits, 0, rounding, scale_round=2 if rounding else 1, seed=9, tensor_id=11), "dual row")
    assert_same(col, oracle.quantize_bf16(bits, 1, rounding, scale_round=2 if rounding else 1, seed=9, tensor_id=13), "dual col")
    # with the maximum supplied by the caller
    amax = tj.amax_bf16(x, tj.alloc_workspace(1 << 14))
    row2, col2 = tj.quantize_dual(x, rounding, seed=9, tensor_id_row=11, tensor_id_col=13, amax_in=amax)
    torch.cuda.synchronize()
    assert torch.equal(row2.codes, row.codes) and torch.equal(col2.codes, col.codes)
    assert torch.equal(row2.scales, row.scales) and torch.equal(col2.scales, col.scales)


@pytest.mark.parametrize("shape", [(256, 512), (16, 16), (144, 80), (1040, 144), (272, 1024)])
@pytest.mark.parametrize("rounding", [0, 1])
def test_requant_col(shape, rounding):
    bits = wl.normal_bf16(shape, 0.02, 500 + shape[0], 1e-2, 30.0)
    src_ref = oracle.quantize_bf16(bits, 0, 0)
    ref = oracle.requantize(src_ref, 1, rounding, seed=4, tensor_id=6)
    src_gpu = tj.quantize(dev_bf16(bits), 0, 0)
    assert_same(src_gpu, src_ref, "requant source", check_amax=True)
    got = tj.quantize(src_gpu, 1, rounding, seed=4, tensor_id=6)
    assert_same(got, ref, "requant %s r%d" % (shape, rounding))


@pytest.mark.parametrize("rounding,scale_round", [(0, 2), (1, 1)])
def test_non_default_scale_rounding_in_every_quantizer(rounding, scale_round):
    """Nearest rounding with the scale rounded up, stochastic rounding with the scale rounded to nearest: the kernel
    instantiations the defaults never pick, for the column-wise, dual, re-quantizing and 1 x 128 row-wise quantizers."""
    kw = dict(scale_round=scale_round, seed=12)
    bits = wl.normal_bf16((272, 208), 1e-3, 41, 1e-2, 30.0)
    x = dev_bf16(bits)
    assert_same(tj.quantize(x, 1, rounding, tensor_id=5, **kw), oracle.quantize_bf16(bits, 1, rounding, tensor_id=5, **kw), "col")
    row, col = tj.quantize_dual(x, rounding, scale_round=scale_round, seed=12, tensor_id_row=3, tensor_id_col=5)
    assert_same(row, oracle.quantize_bf16(bits, 0, rounding, tensor_id=3, **kw), "dual row")
    assert_same(col, oracle.quantize_bf16(bits, 1, rounding, tensor_id=5, **kw), "dual col")
    src = oracle.quantize_bf16(bits, 0, 0)
    assert_same(tj.quantize(to_dev(src), 1, rounding, tensor_id=6, **kw), oracle.requantize(src, 1, rounding, tensor_id=6, **kw),
                "requant")
    wide = wl.student_t_bf16((37, 384), 3.0, 0.1, 42)
    assert_same(tj.quantize(dev_bf16(wide), 0, rounding, outer=tj.binding.OUTER_BLOCK128, tensor_id=1, **kw),
                oracle.quantize_bf16(wide, 0, rounding, outer=oracle.OUTER_BLOCK128, tensor_id=1, **kw), "row128",
                check_amax=(rounding == 0))


def test_requant_on_the_truncation_boundary():
    """Q6 of a 256 x 256 tensor with seed 1322: one argument below 1 sits exactly where dropping and rounding its bits
    under 2^-23 give different codes (tests/test_oracle_pins.py shows that on the CPU); the GPU must drop them too."""
    src = oracle.quantize_bf16(wl.normal_bf16((256, 256), 1.0, 77), 0, oracle.RTN)
    got = tj.quantize(to_dev(src), 1, 1, seed=1322, tensor_id=6)
    assert_same(got, oracle.requantize(src, 1, oracle.SR, seed=1322, tensor_id=6), "Q6 boundary case")


# ------------------------------------------------------------------------ GEMM

GEMM_SHAPES = [(128, 128, 64), (32, 32, 64), (200, 72, 192), (256, 384, 512), (130, 258, 1024), (64, 96, 4096),
               (16, 16, 8192)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("out_dtype", [1, 0])
def test_gemm_nt(M, N, K, out_dtype):
    A = oracle.quantize_bf16(wl.normal_bf16((M, K), 1.0, 600 + M, 1e-2, 50.0), 0, 0)
    B = oracle.quantize_bf16(wl.normal_bf16((N, K), 0.02, 601 + N), 0, 1, seed=2)
    ref, absref = oracle.gemm_nt(A, B)
    got = tj.gemm_nt(to_dev(A), to_dev(B), out_dtype)
    torch.cuda.synchronize()
    check_product(got, ref, absref, "gemm %dx%dx%d" % (M, N, K))


@pytest.mark.parametrize("M,N,K", [(8100, 700, 768), (8155, 745, 768), (3000, 770, 2304), (700, 760, 8192),
                                   (8192, 2000, 768), (1000, 520, 3072)])
@pytest.mark.parametrize("out_dtype", [0, 1])
def test_gemm_ragged_large_tiles_sampled_rows(M, N, K, out_dtype):
    """Shapes for which the planner takes its large workgroup tiles (128 x 192, 256 x 256, 256 x 128; with and without a
    K split), with ragged edges in both directions and N not a multiple of 4: sampled rows, all columns."""
    assert max(tj.binding.gemm_plan(M, N, K)[:2]) >= 192
    A = oracle.quantize_bf16(wl.normal_bf16((M, K), 1.0, 700 + N, 1e-2, 50.0), 0, 0)
    B = oracle.quantize_bf16(wl.normal_bf16((N, K), 0.02, 701 + M), 0, 1, seed=4)
    got = tj.gemm_nt(to_dev(A), to_dev(B), out_dtype)
    again = tj.gemm_nt(to_dev(A), to_dev(B), out_dtype)
    torch.cuda.synchronize()
    assert torch.equal(got, again)                            # fixed summation order, also when K is split
    rng = np.random.default_rng(M + N)
    rows = np.unique(np.concatenate([[0, M - 1, (M // 128) * 128 - 1, (M // 128) * 128 % M],
                                     rng.choice(M, 40, replace=False)]))
    ref, absref = oracle.gemm_nt(A, B, rows_a=rows)
    check_product(got[torch.from_numpy(rows).cuda()], ref, absref, "gemm %dx%dx%d" % (M, N, K))


def _variant_cases():
    from gemm_variants import VARIANT_SHAPES
    cases, nsplit = [], 0
    for key, shape in sorted(VARIANT_SHAPES.items()):
        # one pass: the kernel converts and stores itself, so both output types are kernels of their own;
        # K split: the kernel writes FP32 partials either way, the output type alternates over the table
        nsplit += key[3]
        for out_dtype in ((nsplit & 1,) if key[3] else (0, 1)):
            cases.append(pytest.param(key, shape, out_dtype, id="%dx%d-ps%d-split%d-out%d" % (*map(int, key), out_dtype)))
    return cases


@pytest.mark.parametrize("key,shape,out_dtype", _variant_cases())
def test_gemm_every_kernel_instantiation(key, shape, out_dtype):
    """Every workgroup tile x scale fetch x split x output variant of the product kernel, on a ragged shape for which
    the planner picks it (checked without a GPU in test_boundary_cpu.py): sampled rows, all columns."""
    M, N, K = shape
    pm, pn, split = tj.binding.gemm_plan(M, N, K)
    assert (pm, pn, K % 256 == 0, split > 1) == key
    A = oracle.quantize_bf16(wl.normal_bf16((M, K), 1.0, 900 + N, 1e-2, 50.0), 0, 0)
    B = oracle.quantize_bf16(wl.normal_bf16((N, K), 0.02, 901 + M), 0, 1, seed=6)
    got = tj.gemm_nt(to_dev(A), to_dev(B), out_dtype)
    torch.cuda.synchronize()
    rng = np.random.default_rng(M * 31 + N)
    edge = [0, M - 1, (M // pm) * pm - 1, (M // pm) * pm % M, min(M - 1, pm - 1), min(M - 1, pm)]
    rows = np.unique(np.concatenate([[r for r in edge if 0 <= r < M], rng.choice(M, min(M, 24), replace=False)]))
    ref, absref = oracle.gemm_nt(A, B, rows_a=rows)
    check_product(got[torch.from_numpy(rows).cuda()], ref, absref, "gemm %dx%dx%d" % (M, N, K))


# (outer mode, M, N, K, tile): whole tiles, K a multiple of 256, more workgroups than the chip holds of that tile at
# once and not a multiple of that number, so tiles start and end at different times on one compute unit.  K = 256 is the
# shortest reduction with paired scale fetch (two stages, one scale pair), 768 a typical short one.
WALK_SHAPES = [(0, 6016, 4096, 256, (128, 128)), (0, 4736, 3456, 256, (128, 192)), (0, 3200, 5120, 256, (128, 256)),
               (0, 5120, 3200, 256, (256, 128)), (0, 4352, 5888, 256, (256, 256)), (0, 4352, 5888, 768, None),
               (0, 4736, 3456, 512, None), (1, 6016, 4096, 256, (128, 128)), (1, 4736, 3456, 256, (128, 192)),
               (1, 3200, 5120, 256, (128, 256)), (1, 2816, 4480, 256, (256, 128)), (1, 2816, 4480, 768, None)]


@pytest.mark.parametrize("outer,M,N,K,tile", WALK_SHAPES)
@pytest.mark.parametrize("out_dtype", [0, 1])
def test_gemm_more_tiles_than_resident_workgroups(outer, M, N, K, tile, out_dtype):
    pm, pn, split = tj.binding.gemm_plan(M, N, K, outer)
    assert M % pm == 0 and N % pn == 0 and split == 1 and (tile is None or (pm, pn) == tile)
    resident = 256 * {(256, 256): 1, (256, 128): 1, (128, 256): 1, (128, 128): 3, (128, 192): 2}[(pm, pn)]
    assert (M // pm) * (N // pn) > resident
    if outer:
        A = oracle.quantize_bf16(_block_operand(M, K, 730 + N, 1.0), 0, 0, outer=oracle.OUTER_BLOCK128)
        B = oracle.quantize_bf16(_block_operand(N, K, 731 + M, 0.02), 0, 1, outer=oracle.OUTER_BLOCK128, seed=6)
    else:
        A = oracle.quantize_bf16(wl.normal_bf16((M, K), 1.0, 730 + N, 1e-2, 50.0), 0, 0)
        B = oracle.quantize_bf16(wl.normal_bf16((N, K), 0.02, 731 + M), 0, 1, seed=6)
    got = tj.gemm_nt(to_dev(A), to_dev(B), out_dtype)
    torch.cuda.synchronize()
    # rows from every tile row: first and last row of each, plus random ones
    rng = np.random.default_rng(M + 7 * N + K)
    tiles = np.arange(M // pm) * pm
    rows = np.unique(np.concatenate([tiles, tiles + pm - 1, rng.choice(M, 32, replace=False)]))
    ref, absref = oracle.gemm_nt(A, B, rows_a=rows)
    check_product(got[torch.from_numpy(rows).cuda()], ref, absref, "gemm many tiles %dx%dx%d" % (M, N, K))


def _block_operand(rows, K, seed, std):
    """an operand with 1 x 128 outer blocks whose outer scales differ widely from block to block (each 128-block of each
    row gets its own magnitude, 2^-6 .. 2^6 times the base law; a few blocks are all zero)"""
    rng = np.random.default_rng(seed)
    x = wl.bf16_to_f32(wl.normal_bf16((rows, K), std, seed, 1e-2, 30.0)).reshape(rows, K // 128, 128)
    mag = np.exp2(rng.integers(-6, 7, (rows, K // 128, 1))).astype(np.float32)
    mag[rng.random((rows, K // 128, 1)) < 0.02] = 0.0
    return wl.f32_to_bf16((x * mag).reshape(rows, K))


def _variant_cases_block128():
    from gemm_variants import VARIANT_SHAPES_BLOCK128
    cases, nsplit = [], 0
    for key, shape in sorted(VARIANT_SHAPES_BLOCK128.items()):
        nsplit += key[3]
        for out_dtype in ((nsplit & 1,) if key[3] else (0, 1)):
            cases.append(pytest.param(key, shape, out_dtype, id="b128-%dx%d-ps%d-split%d-out%d" % (*map(int, key), out_dtype)))
    return cases


@pytest.mark.parametrize("key,shape,out_dtype", _variant_cases_block128())
def test_gemm_block128_every_kernel_instantiation(key, shape, out_dtype):
    """The product on operands with the paper's 1 x 128 outer blocks (Sec. 2.2): every tile x scale fetch x split x output
    variant of that mode, on ragged shapes, against the float64 product of the same dequantized operands."""
    M, N, K = shape
    O = tj.binding.OUTER_BLOCK128
    pm, pn, split = tj.binding.gemm_plan(M, N, K, O)
    assert (pm, pn, K % 256 == 0, split > 1) == key
    A = oracle.quantize_bf16(_block_operand(M, K, 700 + N, 1.0), 0, 0, outer=oracle.OUTER_BLOCK128)
    B = oracle.quantize_bf16(_block_operand(N, K, 701 + M, 0.02), 0, 1, outer=oracle.OUTER_BLOCK128, seed=6)
    got = tj.gemm_nt(to_dev(A), to_dev(B), out_dtype)
    torch.cuda.synchronize()
    rng = np.random.default_rng(M * 31 + N)
    edge = [0, M - 1, (M // pm) * pm - 1, (M // pm) * pm % M, min(M - 1, pm - 1), min(M - 1, pm)]
    rows = np.unique(np.concatenate([[r for r in edge if 0 <= r < M], rng.choice(M, min(M, 24), replace=False)]))
    ref, absref = oracle.gemm_nt(A, B, rows_a=rows)
    check_product(got[torch.from_numpy(rows).cuda()], ref, absref, "gemm block128 %dx%dx%d" % (M, N, K))


def test_gemm_block128_small_shapes_in_full_and_mode_mismatch():
    O = oracle.OUTER_BLOCK128
    for (M, N, K) in [(33, 20, 128), (130, 257, 384), (256, 512, 1024), (64, 64, 4096)]:
        A = oracle.quantize_bf16(_block_operand(M, K, 720 + M, 1.0), 0, 0, outer=O)
        B = oracle.quantize_bf16(_block_operand(N, K, 721 + N, 0.5), 0, 0, outer=O)
        ref, absref = oracle.gemm_nt(A, B)
        for out_dtype in (1, 0):
            check_product(tj.gemm_nt(to_dev(A), to_dev(B), out_dtype), ref, absref, "block128 %dx%dx%d" % (M, N, K))
    At = oracle.quantize_bf16(_block_operand(64, 256, 1, 1.0), 0, 0)
    Bb = oracle.quantize_bf16(_block_operand(64, 256, 2, 1.0), 0, 0, outer=O)
    with pytest.raises(tj.NVFP4Error) as e:
        tj.gemm_nt(to_dev(At), to_dev(Bb), 1)
    assert e.value.code == -6


@pytest.mark.parametrize("N,D,C", [(256, 512, 384), (384, 128, 640), (1152, 256, 128)])
def test_linear_block128_mode(N, D, C):
    """The whole layer with the paper's 1 x 128 outer blocks on every operand: forward, the two separate backward calls
    and the fused one; operands bit for bit, products within tolerance, no maximum pass anywhere."""
    B = tj.binding
    O = oracle.OUTER_BLOCK128
    Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed=40 + N)
    X, W, dY = dev_bf16(Xb), dev_bf16(Wb), dev_bf16(dYb)
    Y, Xq, Wq = tj.linear_fwd(X, W, B.OUT_F32, outer=B.OUTER_BLOCK128)
    oXq, oWq = oracle.linear_fwd(Xb, Wb, outer=O)
    assert_same(Xq, oXq, "Q1 block128", check_amax=True)
    assert_same(Wq, oWq, "Q2 block128", check_amax=True)
    check_product(Y, *oracle.gemm_nt(oXq, oWq), "Y block128")
    o3, o4 = oracle.linear_bwd_dx_operands(dYb, oWq, 5, 2, outer=O)
    o5, o6 = oracle.linear_bwd_dw_operands(dYb, oXq, 5, 2, outer=O)
    assert_same(tj.quantize(dY, 0, B.ROUND_SR, seed=5, tensor_id=35, outer=B.OUTER_BLOCK128), o3, "Q3 block128")
    assert_same(tj.quantize(Wq, 1, B.ROUND_SR, seed=5, tensor_id=36, outer=B.OUTER_BLOCK128), o4, "Q4 block128")
    assert_same(tj.quantize(dY, 1, B.ROUND_SR, seed=5, tensor_id=37, outer=B.OUTER_BLOCK128), o5, "Q5 block128")
    assert_same(tj.quantize(Xq, 1, B.ROUND_SR, seed=5, tensor_id=38, outer=B.OUTER_BLOCK128), o6, "Q6 block128")
    dX = tj.linear_bwd_dx(dY, Wq, 5, 2, B.OUT_F32)
    dW = tj.linear_bwd_dw(dY, Xq, 5, 2, B.OUT_F32)
    check_product(dX, *oracle.gemm_nt(o3, o4), "dX block128")
    check_product(dW, *oracle.gemm_nt(o5, o6), "dW block128")
    dX2, dW2 = tj.linear_bwd(dY, Xq, Wq, 5, 2, B.OUT_F32)
    torch.cuda.synchronize()
    assert torch.equal(dX, dX2) and torch.equal(dW, dW2)


@pytest.mark.parametrize("rounding", [0, 1])
def test_quantizers_with_random_hadamard_transform(rounding):
    """Sec. 4.1: every quantizer that serves the backward pass, with x S H_16 along the grouped axis first (1 x 128
    outer blocks): row-wise and column-wise from bf16 (Q3, Q5), column-wise from packed tensors (Q4, Q6); bytes."""
    B = tj.binding
    O, OB = oracle.OUTER_BLOCK128, B.OUTER_BLOCK128
    for shape in [(128, 128), (260, 384), (1152, 1024), (40, 8320)]:
        bits = wl.normal_bf16(shape, 1e-3, 480 + shape[0], 1e-2, 50.0)
        bits[0, :128] = 0
        x = dev_bf16(bits)
        ref = oracle.quantize_bf16(bits, 0, rounding, outer=O, seed=3, tensor_id=11, rht_id=15)
        assert_same(tj.quantize(x, 0, rounding, outer=OB, seed=3, tensor_id=11, rht_id=15), ref, "row rht %s" % (shape,))
        # another sign stream gives other bytes
        other = tj.quantize(x, 0, rounding, outer=OB, seed=3, tensor_id=11, rht_id=16)
        torch.cuda.synchronize()
        assert not np.array_equal(other.codes.cpu().numpy(), ref.codes)
    for shape in [(128, 8), (256, 512), (1152, 136), (2048, 1040)]:
        bits = wl.student_t_bf16(shape, 3.0, 0.1, 490 + shape[1])
        ref = oracle.quantize_bf16(bits, 1, rounding, outer=O, seed=4, tensor_id=13, rht_id=8)
        assert_same(tj.quantize(dev_bf16(bits), 1, rounding, outer=OB, seed=4, tensor_id=13, rht_id=8), ref, "col rht %s" % (shape,))
    for shape in [(128, 128), (384, 1152), (1024, 256)]:
        for src_outer in (1, 0):
            bits = wl.normal_bf16(shape, 1.0, 500 + shape[0], 1e-2, 50.0)
            src_ref = oracle.quantize_bf16(bits, 0, 0, outer=src_outer)
            ref = oracle.requantize(src_ref, 1, rounding, outer=O, seed=17, tensor_id=6, rht_id=7)
            got = tj.quantize(to_dev(src_ref), 1, rounding, outer=OB, seed=17, tensor_id=6, rht_id=7)
            assert_same(got, ref, "requant rht %s src%d" % (shape, src_outer))


@pytest.mark.parametrize("N,D,C", [(256, 512, 384), (1152, 256, 128)])
def test_linear_backward_with_random_hadamard_transform(N, D, C):
    """The backward pass of TetraJet-v2-base: 1 x 128 outer blocks, stochastic rounding, and the random Hadamard
    transform on both operands of dX and of dW (Sec. 4.1); separate calls, the fused call, against the oracle."""
    B = tj.binding
    O = oracle.OUTER_BLOCK128
    Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed=60 + N)
    X, W, dY = dev_bf16(Xb), dev_bf16(Wb), dev_bf16(dYb)
    Y, Xq, Wq = tj.linear_fwd(X, W, B.OUT_F32, outer=B.OUTER_BLOCK128)
    oXq, oWq = oracle.linear_fwd(Xb, Wb, outer=O)
    o3, o4 = oracle.linear_bwd_dx_operands(dYb, oWq, 5, 2, outer=O, rht=True)
    o5, o6 = oracle.linear_bwd_dw_operands(dYb, oXq, 5, 2, outer=O, rht=True)
    dX = tj.linear_bwd_dx(dY, Wq, 5, 2, B.OUT_F32, rht=True)
    dW = tj.linear_bwd_dw(dY, Xq, 5, 2, B.OUT_F32, rht=True)
    check_product(dX, *oracle.gemm_nt(o3, o4), "dX rht")
    check_product(dW, *oracle.gemm_nt(o5, o6), "dW rht")
    dX2, dW2 = tj.linear_bwd(dY, Xq, Wq, 5, 2, B.OUT_F32, rht=True)
    torch.cuda.synchronize()
    assert torch.equal(dX, dX2) and torch.equal(dW, dW2)
    # and it is a different estimate from the one without the transform, of the same quantity
    dX0 = tj.linear_bwd_dx(dY, Wq, 5, 2, B.OUT_F32)
    torch.cuda.synchronize()
    assert not torch.equal(dX, dX0)
    exact = wl.bf16_to_f32(dYb).astype(np.float64) @ oracle.dequant_f64(oWq)
    for est in (dX, dX0):
        rel = np.abs(est.double().cpu().numpy() - exact).mean() / np.abs(exact).mean()
        assert rel < 0.25
    with pytest.raises(tj.NVFP4Error):
        Yt, Xqt, Wqt = tj.linear_fwd(X, W, B.OUT_F32)
        tj.linear_bwd_dx(dY, Wqt, 5, 2, B.OUT_F32, rht=True)       # per-tensor contexts: not provided


def test_gemm_exact_on_integer_operands():
    """Scales 1 and grid-valued operands: the product is a small-integer matrix product, exact in FP32."""
    rng = np.random.default_rng(7)
    grid = oracle.FP4_VALUES
    M, N, K = 96, 160, 256

    def operand(rows, big_col, zero_col):
        m = rng.integers(0, 8, (rows, K))
        m[:, ::16] = 7                                      # a 6 in every group -> S_block = 1
        sg = rng.integers(0, 2, (rows, K))
        x = np.where(sg == 1, -grid[m], grid[m]).astype(np.float32)
        x[:, zero_col] = 0.0                                # the other operand's 2688 meets only zeros
        x[0, big_col] = 2688.0                              # S_global = 1
        return wl.f32_to_bf16(x)

    A = oracle.quantize_bf16(operand(M, 1, 2), 0, 0)
    B = oracle.quantize_bf16(operand(N, 2, 1), 0, 0)
    assert A.gscale[0] == 1.0 and B.gscale[0] == 1.0
    ref, _ = oracle.gemm_nt(A, B)
    got = tj.gemm_nt(to_dev(A), to_dev(B), 1).double().cpu().numpy()
    assert np.array_equal(got, ref)


def test_gemm_all_scale_codes_and_all_element_codes():
    """Every E4M3 scale byte (subnormal ones included) times every E2M1 code expands exactly."""
    M, N, K = 128, 32, 64
    codes = np.zeros((M, K // 2), dtype=np.uint8)
    scales = np.zeros((M, K // 16), dtype=np.uint8)
    for r in range(M):
        scales[r, :] = [(r * 4 + j) % 0x7F for j in range(4)]
        nib = (np.arange(K) + r) % 16
        codes[r] = (nib[0::2] | (nib[1::2] << 4)).astype(np.uint8)
    A = oracle.NVFP4(codes, scales, np.array([1.0], np.float32), 0.0, M, K, 0)
    bc = np.zeros((N, K // 2), dtype=np.uint8)
    for r in range(N):
        bc[r, (r % 32)] = 0x02 if r % 2 == 0 else 0x20        # a single 1.0 per row: picks one column of A
    B = oracle.NVFP4(bc, np.full((N, K // 16), 0x38, np.uint8), np.array([1.0], np.float32), 0.0, N, K, 0)
    ref, _ = oracle.gemm_nt(A, B)
    got = tj.gemm_nt(to_dev(A), to_dev(B), 1).double().cpu().numpy()
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- linear layer

def run_linear_case(N, D, C, seed, kind="block", sr_seed=0, layer_id=1, out_dtype=1, sample=None):
    Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed, kind)
    X, W, dY = dev_bf16(Xb), dev_bf16(Wb), dev_bf16(dYb)
    Y, Xq, Wq = tj.linear_fwd(X, W, out_dtype)
    dX = tj.linear_bwd_dx(dY, Wq, sr_seed, layer_id, out_dtype)
    dW = tj.linear_bwd_dw(dY, Xq, sr_seed, layer_id, out_dtype)
    torch.cuda.synchronize()
    oXq, oWq = oracle.linear_fwd(Xb, Wb)
    assert_same(Xq, oXq, "Q1(X)", check_amax=True)
    assert_same(Wq, oWq, "Q2(W)", check_amax=True)
    o3, o4 = oracle.linear_bwd_dx_operands(dYb, oWq, sr_seed, layer_id)
    o5, o6 = oracle.linear_bwd_dw_operands(dYb, oXq, sr_seed, layer_id)
    rng = np.random.default_rng(seed)

    def rows_of(n):
        if sample is None or n <= sample:
            return None
        return np.sort(rng.choice(n, sample, replace=False))

    for name, got, qa, qb in (("Y", Y, oXq, oWq), ("dX", dX, o3, o4), ("dW", dW, o5, o6)):
        ra = rows_of(qa.rows)
        ref, absref = oracle.gemm_nt(qa, qb, rows_a=ra)
        g = got if ra is None else got[torch.from_numpy(ra).cuda()]
        check_product(g, ref, absref, "%s %dx%dx%d" % (name, N, D, C))
    return Xq, Wq


def test_linear_config1_full():
    """Single layer 256 x 512 -> 512, RTN forward, SR backward, seed 0: checked in full, both output types."""
    run_linear_case(256, 512, 512, seed=0, sr_seed=0, out_dtype=1)
    run_linear_case(256, 512, 512, seed=0, sr_seed=0, out_dtype=0)


def test_linear_ragged_shapes():
    run_linear_case(192, 320, 448, seed=5, sr_seed=3)
    run_linear_case(64, 64, 64, seed=6, sr_seed=4)
    run_linear_case(1088, 192, 576, seed=7, sr_seed=5, sample=128)


def test_backward_operands_match_oracle_bitwise():
    """The temporaries of the backward calls (Q3..Q6) are produced by the same kernels nvfp4_quantize exposes."""
    Xb, Wb, dYb = wl.linear_inputs(256, 384, 512, seed=9)
    oXq, oWq = oracle.linear_fwd(Xb, Wb)
    o3, o4 = oracle.linear_bwd_dx_operands(dYb, oWq, 13, 7)
    o5, o6 = oracle.linear_bwd_dw_operands(dYb, oXq, 13, 7)
    dY = dev_bf16(dYb)
    Xq = tj.quantize(dev_bf16(Xb), 0, 0)
    Wq = tj.quantize(dev_bf16(Wb), 0, 0)
    assert_same(tj.quantize(dY, 0, 1, seed=13, tensor_id=7 * 16 + 3), o3, "Q3")
    assert_same(tj.quantize(Wq, 1, 1, seed=13, tensor_id=7 * 16 + 4), o4, "Q4")
    assert_same(tj.quantize(dY, 1, 1, seed=13, tensor_id=7 * 16 + 5), o5, "Q5")
    assert_same(tj.quantize(Xq, 1, 1, seed=13, tensor_id=7 * 16 + 6), o6, "Q6")


def test_same_seed_same_bytes_other_seed_other_bytes():
    bits = wl.normal_bf16((512, 1024), 1e-3, 11)
    x = dev_bf16(bits)
    a = tj.quantize(x, 1, 1, seed=1, tensor_id=2)
    b = tj.quantize(x, 1, 1, seed=1, tensor_id=2)
    c = tj.quantize(x, 1, 1, seed=2, tensor_id=2)
    torch.cuda.synchronize()
    assert torch.equal(a.codes, b.codes) and torch.equal(a.scales, b.scales)
    assert (a.codes != c.codes).float().mean().item() > 0.2


@pytest.mark.parametrize("N,D,C", [(256, 512, 512), (192, 320, 448), (1088, 192, 576), (128, 64, 1088)])
def test_fused_backward_equals_separate_calls(N, D, C):
    """nvfp4_linear_bwd (one read of dY for both of its quantizations) gives the bytes of the two separate calls."""
    Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed=21)
    X, W, dY = dev_bf16(Xb), dev_bf16(Wb), dev_bf16(dYb)
    for out_dtype in (1, 0):
        _, Xq, Wq = tj.linear_fwd(X, W, out_dtype)
        dX1 = tj.linear_bwd_dx(dY, Wq, 17, 3, out_dtype)
        dW1 = tj.linear_bwd_dw(dY, Xq, 17, 3, out_dtype)
        dX2, dW2 = tj.linear_bwd(dY, Xq, Wq, 17, 3, out_dtype)
        torch.cuda.synchronize()
        assert torch.equal(dX1, dX2) and torch.equal(dW1, dW2)
    oXq, oWq = oracle.linear_fwd(Xb, Wb)
    ref, absref = oracle.gemm_nt(*oracle.linear_bwd_dw_operands(dYb, oXq, 17, 3))
    check_product(dW2, ref, absref, "fused dW")


# ------------------------------------------------------------------ degenerate sizes

def test_empty_inputs_are_accepted_and_write_nothing():
    """Zero rows / zero tokens: every entry point returns OK, launches nothing that could fault, leaves outputs alone."""
    B = tj.binding
    dev = torch.device("cuda")
    x0 = torch.empty((0, 128), dtype=torch.bfloat16, device=dev)
    q = tj.quantize(x0, 0, B.ROUND_RTN)
    assert (q.rows, q.K) == (0, 128)
    q = tj.quantize(x0, 1, B.ROUND_SR, seed=1)
    assert (q.rows, q.K) == (128, 0)
    r, c = tj.quantize_dual(x0, B.ROUND_SR, seed=1)
    assert (r.rows, r.K, c.rows, c.K) == (0, 128, 128, 0)
    # a layer with no tokens: Y and dX are empty, dW is all zeros
    W = dev_bf16(wl.normal_bf16((64, 128), 0.02, 3))
    Y, Xq, Wq = tj.linear_fwd(x0, W, B.OUT_F32)
    assert Y.shape == (0, 64)
    dY = torch.empty((0, 64), dtype=torch.bfloat16, device=dev)
    dX, dW = tj.linear_bwd(dY, Xq, Wq, 5, 0, B.OUT_F32)
    torch.cuda.synchronize()
    assert dX.shape == (0, 128) and dW.shape == (64, 128)
    assert torch.count_nonzero(dW).item() == 0


def test_gemm_longest_reduction():
    """K = 2^22, the longest reduction the product accepts (its tile offsets are 32-bit): 16 x 16 outputs, split along K."""
    M = N = 16
    K = 1 << 22
    A = oracle.quantize_bf16(wl.normal_bf16((M, K), 1.0, 901), 0, 0)
    Bq = oracle.quantize_bf16(wl.normal_bf16((N, K), 0.02, 902), 0, 1, seed=3)
    assert tj.binding.gemm_plan(M, N, K)[2] > 1
    ref, absref = oracle.gemm_nt(A, Bq)
    got = tj.gemm_nt(to_dev(A), to_dev(Bq), 1)
    torch.cuda.synchronize()
    check_product(got, ref, absref, "gemm 16x16x2^22")
    with pytest.raises(tj.NVFP4Error):                       # one step beyond is refused on the host
        bad = tj.alloc_nvfp4(16, 2 * K)
        tj.gemm_nt(bad, bad, 1)


# ------------------------------------------------- more than 2^32 elements (64-bit indexing, sampled)

def _rows_match(q_gpu, row, ref: oracle.NVFP4, what):
    assert np.array_equal(q_gpu.codes[row].cpu().numpy(), ref.codes[0]), "%s: codes of row %d" % (what, row)
    assert np.array_equal(q_gpu.scales[row].cpu().numpy(), ref.scales[0]), "%s: scales of row %d" % (what, row)
    assert np.float32(q_gpu.gscale.cpu().numpy()[0]) == ref.gscale[0], what


def test_quantizers_beyond_2_to_32_elements():
    """A 32800 x 131200 tensor (4.3e9 elements): every quantizer's rows / columns on both sides of element 2^32, the
    first and the last, against the oracle's slice entry.  The tensor is drawn on the GPU (standard normal, one planted
    maximum of 40 in the last element) and the sampled rows and columns are copied to the host for the oracle."""
    B = tj.binding
    R, C = 32800, 131200
    assert R * C > 2 ** 32
    gen = torch.Generator(device="cuda")
    gen.manual_seed(20)
    x = torch.empty((R, C), dtype=torch.bfloat16, device="cuda").normal_(generator=gen)
    x[R - 1, C - 1] = 40.0
    ws = tj.alloc_workspace(tj.workspace_bytes(B.OP_QUANTIZE, R, C, 0))
    amax = float(tj.amax_bf16(x, ws).cpu()[0])
    assert amax == 40.0
    rows = [0, 1, R // 2, 2 ** 32 // C, 2 ** 32 // C + 1, R - 1]
    cols = [0, 1, C // 2, 2 ** 32 // R, 2 ** 32 // R + 1, C - 1]
    x_rows = {r: x[r].float().cpu().numpy()[None, :] for r in rows}
    x_cols = {c: x[:, c].float().cpu().numpy()[None, :] for c in cols}

    print("[2^32] row-wise", flush=True)
    q_rtn = tj.quantize(x, 0, B.ROUND_RTN, ws=ws)
    for r in rows:
        _rows_match(q_rtn, r, oracle.quantize_f32_slice(x_rows[r], r, amax, oracle.RTN), "row RTN")
    last = oracle.quantize_f32_slice(x_rows[R - 1], R - 1, amax, oracle.RTN)
    amax_deq = float(np.abs(oracle.dequant_f32(last)).max())
    assert float(q_rtn.amax_deq.cpu()[0]) == amax_deq          # the planted maximum dominates every other value
    q = tj.quantize(x, 0, B.ROUND_SR, seed=21, tensor_id=3, ws=ws)
    for r in rows:
        _rows_match(q, r, oracle.quantize_f32_slice(x_rows[r], r, amax, oracle.SR, seed=21, tensor_id=3), "row SR")
    del q

    print("[2^32] column-wise", flush=True)
    q = tj.quantize(x, 1, B.ROUND_SR, seed=21, tensor_id=5, ws=ws)
    for c in cols:
        _rows_match(q, c, oracle.quantize_f32_slice(x_cols[c], c, amax, oracle.SR, seed=21, tensor_id=5), "col SR")
    del q

    print("[2^32] row-wise and column-wise from one read", flush=True)
    qr, qc = tj.quantize_dual(x, B.ROUND_SR, seed=21, tensor_id_row=3, tensor_id_col=5, ws=ws)
    for r in rows:
        _rows_match(qr, r, oracle.quantize_f32_slice(x_rows[r], r, amax, oracle.SR, seed=21, tensor_id=3), "dual row SR")
    for c in cols:
        _rows_match(qc, c, oracle.quantize_f32_slice(x_cols[c], c, amax, oracle.SR, seed=21, tensor_id=5), "dual col SR")
    del qr, qc, x

    print("[2^32] column-wise from the packed tensor", flush=True)
    q = tj.quantize(q_rtn, 1, B.ROUND_SR, seed=21, tensor_id=6, ws=ws)
    for c in cols:
        g = c // 16
        grp = oracle.NVFP4(q_rtn.codes[:, 8 * g:8 * g + 8].cpu().numpy().copy(), q_rtn.scales[:, g:g + 1].cpu().numpy().copy(),
                           q_rtn.gscale.cpu().numpy(), amax_deq, R, 16, oracle.OUTER_TENSOR)
        col = np.ascontiguousarray(oracle.dequant_f32(grp)[:, c % 16])[None, :]
        _rows_match(q, c, oracle.quantize_f32_slice(col, c, amax_deq, oracle.SR, seed=21, tensor_id=6), "requant SR")


@pytest.mark.parametrize("out_dtype", [0, 1])
def test_gemm_beyond_2_to_32_outputs(out_dtype):
    """65600 x 65600 outputs (4.3e9) of a K = 64 product: rows on both sides of output 2^31 and 2^32, first and last."""
    M = N = 65600
    K = 64
    A = oracle.quantize_bf16(wl.normal_bf16((M, K), 1.0, 31, 1e-2, 50.0), 0, 0)
    Bq = oracle.quantize_bf16(wl.normal_bf16((N, K), 0.02, 32), 0, 1, seed=4)
    got = tj.gemm_nt(to_dev(A), to_dev(Bq), out_dtype)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 2 ** 31 // N, 2 ** 31 // N + 1, 2 ** 32 // N, 2 ** 32 // N + 1, M - 2, M - 1])
    ref, absref = oracle.gemm_nt(A, Bq, rows_a=rows)
    check_product(got[torch.from_numpy(rows).cuda()], ref, absref, "gemm %dx%dx%d" % (M, N, K))
