"""Pins for the CPU oracle: what the paper and the mathematics fix, checked on the CPU.

The paper (TetraJet-v2, arXiv 2510.27527) prints no worked numeric example, so the
oracle is pinned by: the printed E2M1 value set and range limits (tests/golden/),
an independent library decoding of E4M3 (torch.float8_e4m3fn), the argmin definition
of deterministic rounding, the closed-form probability of stochastic rounding,
exact round trips of representable tensors, the scale / absmax invariants of the
double-block formulas, empirical unbiasedness, symmetries, and brute-force matrix
products (integer arithmetic and numpy) for the three products of the linear layer.
"""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _golden_grid():
    with open(os.path.join(GOLDEN, "e2m1_values.txt")) as f:
        return np.array([float(l) for l in f if l.strip() and not l.startswith("#")])


def _golden_limits():
    out = {}
    with open(os.path.join(GOLDEN, "format_limits.txt")) as f:
        for l in f:
            if l.strip() and not l.startswith("#"):
                k, v = l.split()
                out[k] = float(v)
    return out


GRID = _golden_grid()
LIM = _golden_limits()


def decode_codes(codes: np.ndarray) -> np.ndarray:
    """[rows, K/2] bytes -> [rows, K] signed E2M1 values, using the golden value list only."""
    lo, hi = codes & 0xF, codes >> 4
    nib = np.stack([lo, hi], axis=-1).reshape(codes.shape[0], -1)
    v = GRID[nib & 7]
    return np.where(nib & 8, -v, v)


def e4m3_torch(codes: np.ndarray) -> np.ndarray:
    return torch.from_numpy(codes.astype(np.uint8)).view(torch.float8_e4m3fn).to(torch.float64).numpy()


# ------------------------------------------------------------------ formats

def test_grid_is_the_papers():
    assert list(GRID) == [0, 0.5, 1, 1.5, 2, 3, 4, 6]
    assert np.array_equal(oracle.FP4_VALUES, GRID)


def test_e4m3_decode_matches_library():
    L = oracle.lib()
    codes = np.arange(0, 0x7F, dtype=np.uint8)
    mine = np.array([L.oracle_e4m3_value(int(c)) for c in codes], dtype=np.float64)
    assert np.array_equal(mine, e4m3_torch(codes))
    assert mine.max() == LIM["e4m3_max"]
    assert np.all(np.diff(mine) > 0)


def test_e4m3_round_nearest_matches_library():
    L = oracle.lib()
    rng = np.random.default_rng(1)
    s = np.concatenate([
        np.exp(rng.uniform(np.log(2.0 ** -12), np.log(448.0), 4000)),
        np.array([0.0, 2.0 ** -10, 2.0 ** -9, 1.5 * 2.0 ** -9, 2.5 * 2.0 ** -9, 2.0 ** -6, 448.0,
                  0.3, 1.0, 1.0625, 1.1875, 17.0, 19.0, 447.9]),
    ]).astype(np.float32)
    mine = np.array([L.oracle_e4m3_round(float(v), oracle.SCALE_NE) for v in s], dtype=np.uint8)
    lib_codes = torch.from_numpy(s).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(mine, lib_codes)
    # saturation instead of overflow
    assert L.oracle_e4m3_round(1e9, oracle.SCALE_NE) == 0x7E
    assert L.oracle_e4m3_round(1e9, oracle.SCALE_UP) == 0x7E


def test_e4m3_round_up_is_least_upper_bound():
    L = oracle.lib()
    rng = np.random.default_rng(2)
    s = np.exp(rng.uniform(np.log(2.0 ** -14), np.log(448.0), 3000)).astype(np.float32)
    vals = e4m3_torch(np.arange(0, 0x7F, dtype=np.uint8))
    for v in s:
        c = L.oracle_e4m3_round(float(v), oracle.SCALE_UP)
        assert vals[c] >= v
        assert c == 0 or vals[c - 1] < v
    for c in range(0x7F):                 # representable scales are fixed points of both modes
        assert L.oracle_e4m3_round(float(vals[c]), oracle.SCALE_UP) == c
        assert L.oracle_e4m3_round(float(vals[c]), oracle.SCALE_NE) == c


# --------------------------------------------------------- rounding functions

def test_rtn_is_argmin_with_even_ties():
    L = oracle.lib()
    rng = np.random.default_rng(3)
    a = np.concatenate([rng.uniform(0, 6, 20000), GRID, np.linspace(0, 6, 1201)]).astype(np.float32)
    for v in a:
        m = L.oracle_round_rtn(float(v))
        d = np.abs(GRID - float(v))
        assert d[m] == d.min()                       # Sec. 2.1: argmin_q |x - q|
    mids = (GRID[:-1] + GRID[1:]) / 2
    for i, mid in enumerate(mids):
        m = L.oracle_round_rtn(float(mid))
        assert m in (i, i + 1) and m % 2 == 0         # tie -> even code
        below = np.nextafter(np.float32(mid), np.float32(0))
        above = np.nextafter(np.float32(mid), np.float32(7))
        assert L.oracle_round_rtn(float(below)) == i
        assert L.oracle_round_rtn(float(above)) == i + 1


@pytest.mark.parametrize("a", [0.0, 0.1, 0.25, 0.49, 0.5, 0.77, 1.0, 1.3, 1.99, 2.0, 2.6, 3.999, 4.5, 5.9, 6.0,
                               0.3000001, 1.0000001, 5.9999995])
def test_sr_closed_form_probability(a):
    """P(q2) = (x - q1)/(q2 - q1) (Sec. 2.1), here on a 22-bit uniform: exhaustive over all 2^22 values of u."""
    import ctypes
    L = oracle.lib()
    a32 = float(np.float32(a))
    lower = ctypes.c_int(0)
    ups = L.oracle_round_sr_count_up(a32, ctypes.byref(lower))
    assert ups >= 0                                       # only the two neighbours, rounded-up set = upper interval of u
    if a32 >= 6.0:
        assert lower.value == 7 and ups == 0
        return
    a_img = float(np.floor(np.float64(a32) * 2.0 ** 23) / 2.0 ** 23) if a32 < 1.0 else a32  # R5: 2^-23 grid below 1
    i1 = int(np.searchsorted(GRID, a_img, side="right") - 1)
    assert lower.value == i1
    q1, q2 = GRID[i1], GRID[i1 + 1]
    assert ups == (a_img - q1) / (q2 - q1) * 2.0 ** 22       # exact: the closed form at 22-bit resolution
    assert abs(ups / 2.0 ** 22 - (a32 - q1) / (q2 - q1)) <= 2.0 ** -21
    if a32 == q1:
        assert ups == 0                                   # grid points never move


def test_sr_mean_equals_value_on_average_over_u():
    """E_u[round_S(a)] = a (unbiasedness, Sec. 2.1): mean over a stride of u values."""
    L = oracle.lib()
    rng = np.random.default_rng(4)
    us = np.arange(0, 1 << 22, 977)
    for a in rng.uniform(0, 6, 30).astype(np.float32):
        vals = np.array([GRID[L.oracle_round_sr(float(a), int(u))] for u in us])
        assert abs(vals.mean() - float(a)) < 2.0 * (977.0 / 2 ** 22 + 2.0 ** -21)


def test_rand22_uniform_and_keyed():
    L = oracle.lib()
    key = L.oracle_stream_key(7, 3)
    n = 1 << 16
    u = np.array([L.oracle_rand22(e, key) for e in range(n)])
    assert u.min() >= 0 and u.max() < (1 << 22)
    # chi-square on 256 buckets of the top byte, 255 dof: mean 255, sd ~22.6
    counts = np.bincount(u >> 14, minlength=256)
    chi2 = ((counts - n / 256) ** 2 / (n / 256)).sum()
    assert chi2 < 255 + 6 * 22.6
    # low bits are uniform too
    counts = np.bincount(u & 255, minlength=256)
    assert ((counts - n / 256) ** 2 / (n / 256)).sum() < 255 + 6 * 22.6
    # the four elements of a quad are different draws: every pair of positions is uncorrelated, also in the joint
    # distribution of their leading bits (16 x 16 contingency table, 225 dof); so are neighbouring quads
    for i in range(4):
        for j in range(i + 1, 4):
            assert abs(np.corrcoef(u[i::4], u[j::4])[0, 1]) < 0.03, (i, j)
            table = np.zeros((16, 16))
            np.add.at(table, (u[i::4] >> 18, u[j::4] >> 18), 1)
            exp = table.sum() / 256
            assert ((table - exp) ** 2 / exp).sum() < 225 + 6 * np.sqrt(2 * 225), (i, j)
    assert abs(np.corrcoef(u[:-4], u[4:])[0, 1]) < 0.02
    # the leading bytes of a quad's four draws are the four bytes of one hash word
    for q in range(0, 64):
        h = L.oracle_quad_bits(q, key)
        assert [int(u[4 * q + i]) >> 14 for i in range(4)] == [(h >> 24) & 255, h & 255, (h >> 8) & 255, (h >> 16) & 255]
    # another tensor id or seed gives another stream
    for other in (L.oracle_stream_key(7, 4), L.oracle_stream_key(8, 3)):
        v = np.array([L.oracle_rand22(e, other) for e in range(4096)])
        assert np.mean(v == u[:4096]) < 0.01
        assert abs(np.corrcoef(v, u[:4096])[0, 1]) < 0.06


def test_quad_bits_avalanche():
    """Flipping one counter bit flips about half of the output bits."""
    L = oracle.lib()
    key = L.oracle_stream_key(0, 0)
    rng = np.random.default_rng(5)
    ps = rng.integers(0, 1 << 32, 400, dtype=np.uint64)
    for bit in range(32):
        flips = [bin(L.oracle_quad_bits(int(p), key) ^ L.oracle_quad_bits(int(p) ^ (1 << bit), key)).count("1")
                 for p in ps]
        assert 13.0 < np.mean(flips) < 19.0, (bit, np.mean(flips))


# ------------------------------------------------------------------ quantizer

def _representable(rows, K, rng, j=-3, outer=oracle.OUTER_TENSOR, pow2_scales=False):
    """X = P * S_b * 2^j with a +-6 in every 16-block and S_b = 448 once per outer group."""
    nb = K // 16
    if pow2_scales:
        sc = (rng.integers(1, 15, (rows, nb)) << 3).astype(np.uint8)       # mantissa 0
    else:
        sc = rng.integers(1, 0x7F, (rows, nb)).astype(np.uint8)
    if outer == oracle.OUTER_TENSOR:
        sc[rng.integers(rows), rng.integers(nb)] = 0x7E
    else:
        for r in range(rows):
            for g in range(K // 128):
                sc[r, g * 8 + rng.integers(8)] = 0x7E
    m = rng.integers(0, 8, (rows, K))
    sg = rng.integers(0, 2, (rows, K))
    pos = rng.integers(0, 16, (rows, nb))
    for r in range(rows):
        for b in range(nb):
            m[r, b * 16 + pos[r, b]] = 7
    P = np.where(sg == 1, -GRID[m], GRID[m])
    Sb = np.repeat(e4m3_torch(sc), 16, axis=1)
    X = (P * Sb * 2.0 ** j).astype(np.float32)
    nib = (sg << 3 | m).astype(np.uint8)
    codes = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return X, codes, sc


@pytest.mark.parametrize("outer", [oracle.OUTER_TENSOR, oracle.OUTER_BLOCK128])
@pytest.mark.parametrize("scale_round", [oracle.SCALE_NE, oracle.SCALE_UP])
def test_exact_round_trip_rtn(outer, scale_round):
    rng = np.random.default_rng(10)
    X, codes, sc = _representable(24, 256, rng, j=-5, outer=outer)
    q = oracle.quantize_f32(X, oracle.RTN, scale_round=scale_round, outer=outer)
    assert np.array_equal(q.codes, codes)
    assert np.array_equal(q.scales, sc)
    assert np.all(q.gscale == 2.0 ** -5)
    assert np.array_equal(oracle.dequant_f64(q), X.astype(np.float64))
    assert q.amax_deq == np.abs(X).max()


@pytest.mark.parametrize("outer", [oracle.OUTER_TENSOR, oracle.OUTER_BLOCK128])
def test_exact_round_trip_sr_pow2_scales(outer):
    """With power-of-two block scales every step is exact, so SR must not move a grid point."""
    rng = np.random.default_rng(11)
    X, codes, sc = _representable(16, 256, rng, j=2, outer=outer, pow2_scales=True)
    for seed in range(5):
        q = oracle.quantize_f32(X, oracle.SR, outer=outer, seed=seed, tensor_id=seed)
        assert np.array_equal(q.codes, codes)
        assert np.array_equal(q.scales, sc)


def _check_invariants(x, q, scale_round):
    """Sec. 2.2 formulas as inequalities: S_g*2688 = amax_g; S_b vs amax_b/(6 S_g); |P| <= 6."""
    rows, K = x.shape
    xa = np.abs(x.astype(np.float64))
    if q.outer == oracle.OUTER_TENSOR:
        Sg = np.full((rows, K // 16), float(q.gscale[0]))
        amax_g = np.full((rows, 1), xa.max())
        Sg_groups = np.full((rows, 1), float(q.gscale[0]))
        sc_groups = q.scales.reshape(1, 1, -1)
    else:
        Sg = np.repeat(q.gscale.astype(np.float64), 8, axis=1)
        amax_g = xa.reshape(rows, K // 128, 128).max(axis=2)
        Sg_groups = q.gscale.astype(np.float64)
        sc_groups = q.scales.reshape(rows, K // 128, 8)
    nz = amax_g > 0
    assert np.allclose(Sg_groups[nz] * LIM["outer_range"], amax_g[nz], rtol=2.0 ** -22)
    assert np.all(Sg_groups[~nz] == 1.0)
    # the block holding the group maximum gets the largest scale, 448
    if q.outer == oracle.OUTER_TENSOR:
        assert (sc_groups.max() == 0x7E) == bool(nz.all())
    else:
        assert np.all((sc_groups.max(axis=2) == 0x7E) == nz)
    amax_b = xa.reshape(rows, K // 16, 16).max(axis=2)
    s = amax_b / (LIM["fp4_max"] * Sg)
    Sb = e4m3_torch(q.scales)
    vals = e4m3_torch(np.arange(0, 0x7F, dtype=np.uint8))
    if scale_round == oracle.SCALE_UP:
        ok_hi = Sb >= np.minimum(s, 448.0) * (1 - 2.0 ** -21)
        prev = np.where(q.scales > 0, vals[np.maximum(q.scales.astype(int) - 1, 0)], -1.0)
        ok_lo = prev < s * (1 + 2.0 ** -21)
        assert ok_hi.all() and ok_lo.all()
        assert np.all((q.scales == 0) == (amax_b == 0))
    else:
        ulp = np.where(Sb < 2.0 ** -6, 2.0 ** -9, 2.0 ** (np.floor(np.log2(np.maximum(Sb, 2.0 ** -9))) - 3))
        assert np.all(np.abs(Sb - np.minimum(s, 448.0)) <= 0.5 * ulp * (1 + 2.0 ** -20) + s * 2.0 ** -21)
    P = decode_codes(q.codes)
    assert np.all(np.isin(np.abs(P), GRID))
    assert np.abs(P).max() <= LIM["fp4_max"]
    # the sign bit of every code is the input's sign bit
    lo, hi = q.codes & 0xF, q.codes >> 4
    nib = np.stack([lo, hi], axis=-1).reshape(rows, K)
    assert np.array_equal((nib >> 3).astype(bool), np.signbit(x))
    return P, Sb, Sg


@pytest.mark.parametrize("outer", [oracle.OUTER_TENSOR, oracle.OUTER_BLOCK128])
@pytest.mark.parametrize("rounding,scale_round", [(oracle.RTN, oracle.SCALE_NE), (oracle.RTN, oracle.SCALE_UP),
                                                  (oracle.SR, oracle.SCALE_UP), (oracle.SR, oracle.SCALE_NE)])
def test_scale_invariants_and_error_bound(outer, rounding, scale_round):
    x = wl.bf16_to_f32(wl.student_t_bf16((48, 384), 3.0, 0.1, 21))
    x[5, 128:256] = 0.0                      # an all-zero outer block
    x[7, 16:32] = 0.0                        # an all-zero inner block
    q = oracle.quantize_f32(x, rounding, scale_round=scale_round, outer=outer, seed=9, tensor_id=2)
    P, Sb, Sg = _check_invariants(x, q, scale_round)
    deq = oracle.dequant_f64(q)
    Sb16, Sg16 = np.repeat(Sb, 16, axis=1), np.repeat(Sg, 16, axis=1)
    assert np.array_equal(deq, P * Sb16 * Sg16)
    y = np.divide(x.astype(np.float64), Sb16 * Sg16, out=np.zeros_like(deq), where=(Sb16 > 0))
    # local grid step at |y|: 0.5 below 2, 1 below 4, else 2
    step = np.where(np.abs(y) < 2, 0.5, np.where(np.abs(y) < 4, 1.0, 2.0))
    err = np.abs(P - np.clip(y, -6, 6))
    bound = step / 2 if rounding == oracle.RTN else step
    assert np.all(err <= bound * (1 + 1e-6) + 1e-6)
    if scale_round == oracle.SCALE_UP:
        assert np.abs(y).max() <= 6 * (1 + 2.0 ** -20)        # nothing is clipped
    assert np.all(P[Sb16 == 0] == 0)
    assert np.all(np.sign(P)[P != 0] == np.sign(x)[P != 0])


def test_zero_tensor_and_tiny_tensor():
    z = np.zeros((4, 128), dtype=np.float32)
    for outer in (oracle.OUTER_TENSOR, oracle.OUTER_BLOCK128):
        for rnd in (oracle.RTN, oracle.SR):
            q = oracle.quantize_f32(z, rnd, outer=outer)
            assert not q.codes.any() and not q.scales.any() and np.all(q.gscale == 1.0)
            assert q.amax_deq == 0.0
    t = np.full((4, 128), 1e-38, dtype=np.float32)
    q = oracle.quantize_f32(t, oracle.RTN)
    assert np.isfinite(oracle.dequant_f64(q)).all() and q.gscale[0] == 2.0 ** -100


def test_rtn_is_odd_and_sr_sign_follows_input():
    x = wl.bf16_to_f32(wl.normal_bf16((32, 256), 1.0, 33, 1e-2, 50.0))
    a = oracle.quantize_f32(x, oracle.RTN)
    b = oracle.quantize_f32(-x, oracle.RTN)
    assert np.array_equal(decode_codes(a.codes), -decode_codes(b.codes))
    assert np.array_equal(a.scales, b.scales) and a.gscale[0] == b.gscale[0]


@pytest.mark.parametrize("rounding", [oracle.RTN, oracle.SR])
def test_colwise_equals_rowwise_of_transpose(rounding):
    bits = wl.normal_bf16((64, 48), 1.0, 34, 1e-2, 50.0)
    col = oracle.quantize_bf16(bits, 1, rounding, seed=5, tensor_id=6)
    row = oracle.quantize_bf16(np.ascontiguousarray(bits.T), 0, rounding, seed=5, tensor_id=6)
    assert col.rows == 48 and col.K == 64
    assert np.array_equal(col.codes, row.codes) and np.array_equal(col.scales, row.scales)
    assert col.gscale[0] == row.gscale[0]


def test_block128_reduces_to_tensor_mode_for_one_outer_block():
    x = wl.bf16_to_f32(wl.normal_bf16((1, 128), 1.0, 35))
    a = oracle.quantize_f32(x, oracle.SR, outer=oracle.OUTER_TENSOR, seed=1, tensor_id=1)
    b = oracle.quantize_f32(x, oracle.SR, outer=oracle.OUTER_BLOCK128, seed=1, tensor_id=1)
    assert np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
    assert a.gscale[0] == b.gscale[0, 0]


def test_sr_is_unbiased_and_ne_scales_clip():
    """Mean over seeds of the dequantized value -> x (Sec. 2.1 / 2.3 unbiasedness), including the
    block maxima under upward-rounded scales; nearest-rounded scales clip block maxima."""
    x = wl.bf16_to_f32(wl.normal_bf16((8, 128), 1.0, 36, 2e-2, 20.0))
    n = 600
    acc = np.zeros(x.shape)
    acc_ne = np.zeros(x.shape)
    for seed in range(n):
        acc += oracle.dequant_f64(oracle.quantize_f32(x, oracle.SR, seed=seed, tensor_id=1))
        acc_ne += oracle.dequant_f64(oracle.quantize_f32(x, oracle.SR, scale_round=oracle.SCALE_NE,
                                                         seed=seed, tensor_id=1))
    q = oracle.quantize_f32(x, oracle.SR, seed=0, tensor_id=1)
    Sb = np.repeat(e4m3_torch(q.scales), 16, axis=1) * float(q.gscale[0])
    sigma = Sb * 1.0                         # sd of one draw <= step/2 <= 1 scaled unit
    dev = np.abs(acc / n - x)
    assert np.all(dev <= 5 * sigma / np.sqrt(n) + 1e-7)
    # with NE scales the largest element of some blocks is clipped below its value: biased
    blk_max = np.abs(x).reshape(8, 8, 16).argmax(axis=2)
    idx = (np.repeat(np.arange(8), 8), (np.arange(8)[None, :] * 16 + blk_max).ravel())
    bias_ne = (np.abs(x) - np.abs(acc_ne / n))[idx]
    assert bias_ne.max() > 10 * (5 * sigma[idx] / np.sqrt(n)).min() or bias_ne.max() > 0.01 * np.abs(x)[idx].max()


def test_different_streams_differ():
    x = wl.bf16_to_f32(wl.normal_bf16((16, 256), 1.0, 37))
    a = oracle.quantize_f32(x, oracle.SR, seed=1, tensor_id=3)
    b = oracle.quantize_f32(x, oracle.SR, seed=1, tensor_id=4)
    c = oracle.quantize_f32(x, oracle.SR, seed=1, tensor_id=3)
    assert np.array_equal(a.codes, c.codes)
    assert np.mean(a.codes != b.codes) > 0.2


def test_bad_shapes_rejected():
    with pytest.raises(ValueError):
        oracle.quantize_f32(np.zeros((2, 24), np.float32), oracle.RTN)
    with pytest.raises(ValueError):
        oracle.quantize_f32(np.zeros((2, 64), np.float32), oracle.RTN, outer=oracle.OUTER_BLOCK128)


# ----------------------------------------------------------------------- GEMM

def test_gemm_nt_against_numpy_and_integers():
    rng = np.random.default_rng(40)
    A = rng.standard_normal((7, 33))
    B = rng.standard_normal((5, 33))
    Cm, Ab = oracle.gemm_nt_f64(A, B)
    assert np.allclose(Cm, A @ B.T, rtol=1e-13, atol=1e-13)
    assert np.allclose(Ab, np.abs(A) @ np.abs(B).T, rtol=1e-13)
    # asymmetric shapes catch a transposed operand
    assert Cm.shape == (7, 5)
    Ai = rng.integers(-12, 13, (6, 64))
    Bi = rng.integers(-12, 13, (9, 64))
    Ci, _ = oracle.gemm_nt_f64(Ai / 2.0, Bi / 2.0)
    assert np.array_equal(Ci * 4, (Ai.astype(np.int64) @ Bi.astype(np.int64).T).astype(np.float64))


def _grid_tensor(rows, cols, rng, c=0.875):
    """Grid-valued tensor * c with a 6 in every 16-block of every row AND every column."""
    m = rng.integers(0, 8, (rows, cols))
    for i in range(rows):
        for j in range(0, cols, 16):
            m[i, j + i % 16] = 7
    sg = rng.integers(0, 2, (rows, cols))
    return (np.where(sg == 1, -GRID[m], GRID[m]) * c).astype(np.float32)


def test_linear_layer_products_on_representable_tensors():
    """With tensors every quantizer reproduces exactly, the three products of Sec. 2.3 must equal
    Y = X W^T, dX = dY W, dW = dY^T X computed by numpy (pins axes and transposes)."""
    rng = np.random.default_rng(41)
    N, D, Cc = 32, 48, 64
    X = _grid_tensor(N, D, rng, 0.875)          # 448 * 2^-9
    W = _grid_tensor(Cc, D, rng, 0.875 / 4)
    dY = _grid_tensor(N, Cc, rng, 0.875 / 64)
    Xb, Wb, dYb = wl.f32_to_bf16(X), wl.f32_to_bf16(W), wl.f32_to_bf16(dY)
    assert np.array_equal(wl.bf16_to_f32(Xb), X)
    Xq, Wq = oracle.linear_fwd(Xb, Wb)
    Y, _ = oracle.gemm_nt(Xq, Wq)
    assert np.array_equal(Y, X.astype(np.float64) @ W.astype(np.float64).T)
    dYq, Wq2 = oracle.linear_bwd_dx_operands(dYb, Wq, seed=3, layer_id=1)
    assert (Wq2.rows, Wq2.K) == (D, Cc)
    dX, _ = oracle.gemm_nt(dYq, Wq2)
    assert np.array_equal(dX, dY.astype(np.float64) @ W.astype(np.float64))
    dYq2, Xq2 = oracle.linear_bwd_dw_operands(dYb, Xq, seed=3, layer_id=1)
    assert (dYq2.rows, dYq2.K) == (Cc, N) and (Xq2.rows, Xq2.K) == (D, N)
    dW, _ = oracle.gemm_nt(dYq2, Xq2)
    assert np.array_equal(dW, dY.astype(np.float64).T @ X.astype(np.float64))


def test_linear_layer_close_to_unquantized_and_aligned():
    """Quantized products approximate the exact ones; the backward operands are estimates of the
    forward-quantized tensors (alignment, Sec. 2.3 item 1 and 3), not of the originals."""
    Xb, Wb, dYb = wl.linear_inputs(64, 128, 96, seed=42)
    X, W, dY = (wl.bf16_to_f32(t).astype(np.float64) for t in (Xb, Wb, dYb))
    Xq, Wq = oracle.linear_fwd(Xb, Wb)
    Y, _ = oracle.gemm_nt(Xq, Wq)
    rel = np.linalg.norm(Y - X @ W.T) / np.linalg.norm(X @ W.T)
    assert rel < 0.2
    Xhat, What = oracle.dequant_f64(Xq), oracle.dequant_f64(Wq)
    accW = np.zeros((128, 96))
    accX = np.zeros((128, 64))
    n = 200
    for seed in range(n):
        _, Wq2 = oracle.linear_bwd_dx_operands(dYb, Wq, seed=seed, layer_id=0)
        _, Xq2 = oracle.linear_bwd_dw_operands(dYb, Xq, seed=seed, layer_id=0)
        accW += oracle.dequant_f64(Wq2)
        accX += oracle.dequant_f64(Xq2)
    # mean of re-quantized operand -> forward-quantized tensor (transposed), closer than to the original
    eW_hat = np.abs(accW / n - What.T).mean()
    eW_org = np.abs(accW / n - W.T).mean()
    assert eW_hat < 0.5 * eW_org
    eX_hat = np.abs(accX / n - Xhat.T).mean()
    eX_org = np.abs(accX / n - X.T).mean()
    assert eX_hat < 0.5 * eX_org


def boundary_case():
    """A small re-quantization (Q6 of a 256 x 256 tensor, seed 1322) in which one element sits exactly on the boundary
    where dropping and rounding the bits below 2^-23 of an argument below 1 give different codes."""
    import workloads as wl
    Xb = wl.normal_bf16((256, 256), 1.0, 77)
    src = oracle.quantize_bf16(Xb, 0, oracle.RTN)
    return src, 1322, 6, 16083


def test_sr_boundary_case_is_on_the_truncation_boundary():
    """R5 below 1: the bits of the argument under 2^-23 are dropped.  In this case floor(a 2^23) + u = 2^22 - 1 (no carry:
    the lower neighbour) while the dropped fraction is >= 1/2, so rounding to nearest first would have carried."""
    L = oracle.lib()
    src, seed, tid, e = boundary_case()
    x = oracle.transpose_f32(oracle.dequant_f32(src))
    rows, K = x.shape
    codes = np.zeros((rows, K // 2), np.uint8)
    scales = np.zeros((rows, K // 16), np.uint8)
    gs = np.zeros(1, np.float32)
    y = np.zeros((rows, K), np.float32)
    rc = L.oracle_quantize_rows_y(oracle._ptr(x), rows, K, oracle.SR, 0, 0, seed, tid, oracle._ptr(codes), oracle._ptr(scales),
                                  oracle._ptr(gs), None, oracle._ptr(y))
    assert rc == 0
    a = float(abs(y.ravel()[e]))
    u = L.oracle_rand22(e, L.oracle_stream_key(seed, tid))
    F = a * 2.0 ** 23
    assert a < 1.0 and F - np.floor(F) >= 0.5
    assert (int(np.floor(F)) & 0x3FFFFF) + u == (1 << 22) - 1
    lower = L.oracle_round_sr(a, u)
    assert L.oracle_round_sr(a, u + 1) == lower + 1          # one more and it carries
    r, k = divmod(e, K)
    nib = (codes[r, k // 2] >> (4 * (k & 1))) & 7
    assert nib == lower
    # the same call through the ordinary entry point gives the same bytes
    ref = oracle.requantize(src, 1, oracle.SR, seed=seed, tensor_id=tid)
    assert np.array_equal(ref.codes, codes) and np.array_equal(ref.scales, scales)


def test_slice_helper_gives_the_rows_of_the_whole_quantization():
    """The slice entry (rows from row0 on, the tensor's maximum passed in) is the full quantizer restricted to those rows,
    for both roundings; it exists for sampled checks of tensors too large to quantize whole on the CPU."""
    x = oracle.bf16_to_f32(wl.student_t_bf16((96, 160), 3.0, 0.1, 71))
    amax = float(np.abs(x).max())
    for rounding in (oracle.RTN, oracle.SR):
        full = oracle.quantize_f32(x, rounding, seed=5, tensor_id=12)
        for row0, n in ((0, 96), (17, 1), (40, 23), (95, 1)):
            part = oracle.quantize_f32_slice(x[row0:row0 + n], row0, amax, rounding, seed=5, tensor_id=12)
            assert part.gscale[0] == full.gscale[0]
            assert np.array_equal(part.codes, full.codes[row0:row0 + n])
            assert np.array_equal(part.scales, full.scales[row0:row0 + n])
    # a different row offset moves the random stream (stochastic rounding only)
    a = oracle.quantize_f32_slice(x[:8], 0, amax, oracle.SR, seed=5, tensor_id=12)
    b = oracle.quantize_f32_slice(x[:8], 8, amax, oracle.SR, seed=5, tensor_id=12)
    assert not np.array_equal(a.codes, b.codes) and np.array_equal(a.scales, b.scales)
