"""Pins for the oracle's readings of the paper, checked against the paper's formulas evaluated independently.

The oracle fixes several points the paper (TetraJet-v2, arXiv 2510.27527) leaves open: the binary32 evaluation order
of the double-block formulas (R1), the discretisation of the stochastic-rounding noise (R5), the random bit
generator (R6) and the dequantized value a re-quantization starts from (R8).  The tests here do not repeat the
oracle's formulas: they evaluate Sec. 2.1 / Sec. 2.2 in exact rational or binary64 arithmetic and bound, count or
locate every place where the oracle's bytes differ from that.
"""
import ctypes
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

GRID = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]
GRID_F = np.array([float(g) for g in GRID])
E4M3 = torch.arange(0, 0x7F, dtype=torch.uint8).view(torch.float8_e4m3fn).to(torch.float64).numpy()   # 127 values
RTN_THRESHOLDS = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])


# ------------------------------------------------------------------------------------------ R5

def _neighbours(a: Fraction):
    i1 = max(i for i in range(7) if GRID[i] <= a)
    return i1, GRID[i1], GRID[i1 + 1]


def _values_with_low_bits(rng, n):
    """binary32 magnitudes in [0, 6): uniform ones, some with all 24 significand bits set, some tiny, some just under
    a grid point - below 1 most of them have bits under 2^-23."""
    a = rng.uniform(0, 6, n).astype(np.float32)
    b = (rng.uniform(0, 1, n).astype(np.float32).view(np.uint32) | np.uint32(0x7FF)).view(np.float32)
    c = np.array([1e-9, 3e-8, 2.0 ** -23, 2.0 ** -24, 0.24999999, 0.49999997, 0.99999994, 0.7500001], dtype=np.float32)
    d = np.nextafter(GRID_F[1:].astype(np.float32), np.float32(0))
    return np.concatenate([a, b, c, d])


def test_sr_is_the_papers_rule_on_a_22_bit_uniform():
    """Sec. 2.1: with xi uniform on (-D/2, D/2), D = q2 - q1, x goes to q2 iff x + xi > (q1 + q2)/2.  Writing
    v = xi/D + 1/2 (uniform on (0, 1)) and f = (x - q1)/D this is f + v > 1.  The oracle's only change is to draw v
    from the 22-bit grid u / 2^22; the rule itself is evaluated here in exact rational arithmetic on the unmodified
    binary32 argument, for sampled u and for the two u on either side of the decision."""
    L = oracle.lib()
    rng = np.random.default_rng(11)
    for a32 in _values_with_low_bits(rng, 300):
        a = Fraction(float(a32))
        i1, q1, q2 = _neighbours(a)
        f = (a - q1) / (q2 - q1)
        us = list(rng.integers(0, 1 << 22, 12)) + [0, (1 << 22) - 1]
        edge = (1 << 22) - int(f * (1 << 22))               # first u that rounds up, by the rule
        us += [u for u in (edge - 1, edge) if 0 <= u < (1 << 22)]
        for u in us:
            want = i1 + 1 if f + Fraction(int(u), 1 << 22) >= 1 else i1
            assert L.oracle_round_sr(float(a32), int(u)) == want, (float(a32), int(u))


def test_sr_probability_and_bias_from_the_unmodified_argument():
    """Counted over all 2^22 draws: P(q2) = floor(f 2^22) / 2^22 with f from the unmodified argument, so from 1 to 6
    (where f 2^22 is an integer for every binary32 value) the rounding is exactly unbiased, and below 1 its mean is
    short of the argument by less than 2^-23 (toward zero, never away): E[round_S(a)] - a in (-2^-23, 0]."""
    L = oracle.lib()
    rng = np.random.default_rng(12)
    vals = np.concatenate([_values_with_low_bits(rng, 8), np.array([0.3000001, 0.77, 0.1, 1.3, 2.6, 5.9], np.float32)])
    saw_dropped_bits = 0
    for a32 in vals:
        a = Fraction(float(a32))
        i1, q1, q2 = _neighbours(a)
        lower = ctypes.c_int(0)
        ups = L.oracle_round_sr_count_up(float(a32), ctypes.byref(lower))
        assert lower.value == i1 and ups >= 0
        F = (a - q1) / (q2 - q1) * (1 << 22)
        assert ups == F.numerator // F.denominator                     # floor
        bias = q1 + (q2 - q1) * Fraction(ups, 1 << 22) - a
        if a >= 1:
            assert bias == 0
        else:
            assert -Fraction(1, 1 << 23) < bias <= 0
            saw_dropped_bits += F.denominator != 1
    assert saw_dropped_bits >= 5                                       # the case the bound is about was exercised


# ------------------------------------------------------------------------------------------ R1

def _e4m3_literal(s: np.ndarray, up: bool) -> np.ndarray:
    """E4M3 code of a non-negative binary64 array: nearest value with ties to the even code, or the least value >= s;
    both saturate at 448.  Written on the library's decoding of the 127 codes."""
    s = np.minimum(s, 448.0)
    hi = np.searchsorted(E4M3, s, side="left")              # least code with value >= s
    if up:
        return hi.astype(np.uint8)
    lo = np.maximum(hi - 1, 0)
    dl, dh = s - E4M3[lo], E4M3[hi] - s
    pick_hi = (dh < dl) | ((dh == dl) & (hi % 2 == 0))
    return np.where(pick_hi, hi, lo).astype(np.uint8)


def _e4m3_boundary_distance(s: np.ndarray, up: bool) -> np.ndarray:
    """relative distance of s from the nearest point where the E4M3 rounding decision changes"""
    s = np.minimum(s, 448.0)
    if up:
        pts = E4M3
    else:
        pts = (E4M3[:-1] + E4M3[1:]) / 2
    i = np.clip(np.searchsorted(pts, s), 1, len(pts) - 1)
    d = np.minimum(np.abs(s - pts[i - 1]), np.abs(pts[i] - s))
    return d / np.maximum(s, 1e-300)


def _rtn_literal(a: np.ndarray) -> np.ndarray:
    a = np.minimum(a, 6.0)
    d = np.abs(a[..., None] - GRID_F)
    idx = np.argmin(d, axis=-1)                              # first minimum
    nxt = np.minimum(idx + 1, 7)
    tie = np.take_along_axis(d, nxt[..., None], -1)[..., 0] == np.take_along_axis(d, idx[..., None], -1)[..., 0]
    return np.where(tie & (idx % 2 == 1), nxt, idx)


def _nibbles(codes: np.ndarray) -> np.ndarray:
    return np.stack([codes & 0xF, codes >> 4], axis=-1).reshape(codes.shape[0], -1)


LAWS = {
    "activation (N(0,1), 0.1 % x50)": lambda: wl.normal_bf16((512, 768), 1.0, 600, 1e-3, 50.0),
    "weight (N(0,0.02))": lambda: wl.normal_bf16((768, 768), 0.02, 601),
    "gradient (N(0,1e-3))": lambda: wl.normal_bf16((512, 768), 1e-3, 602),
    "0.1 Student-t(3)": lambda: wl.student_t_bf16((512, 512), 3.0, 0.1, 7),
    "outlier channels (1 % x100)": lambda: wl.outlier_channel_bf16(256, 2048, 1500),
}
R1_REPORT = {}


@pytest.mark.parametrize("outer", [oracle.OUTER_TENSOR, oracle.OUTER_BLOCK128])
@pytest.mark.parametrize("law", list(LAWS))
def test_r1_against_the_formulas_of_sec_2_2_in_binary64(law, outer):
    """Sec. 2.2 evaluated literally in binary64 - S_block = max|X / S_global| / 6 rounded to E4M3,
    P = round_FP4(X / (S_global S_block)) - with S_global the stored binary32 value.  The oracle's binary32 chain (R1)
    must give the same argument to 4 roundings (4 * 2^-24 relative), and wherever one of its bytes differs from the
    literal evaluation, the literal value must sit within that distance of a point where the rounding decision
    changes (an E4M3 tie / grid point, an E2M1 midpoint).  The counts are the size of what the paper leaves open."""
    L = oracle.lib()
    x = wl.bf16_to_f32(LAWS[law]())
    rows, K = x.shape
    eps = 4 * 2.0 ** -24 * (1 + 1e-6)
    for rounding, up in ((oracle.RTN, False), (oracle.SR, True)):
        codes = np.zeros((rows, K // 2), np.uint8)
        scales = np.zeros((rows, K // 16), np.uint8)
        gs = np.zeros((1,) if outer == oracle.OUTER_TENSOR else (rows, K // 128), np.float32)
        y = np.zeros((rows, K), np.float32)
        rc = L.oracle_quantize_rows_y(oracle._ptr(x), rows, K, rounding, 0, outer, 3, 1, oracle._ptr(codes),
                                      oracle._ptr(scales), oracle._ptr(gs), None, oracle._ptr(y))
        assert rc == 0
        xa = np.abs(x.astype(np.float64))
        # the outer scale is a stored binary32 number: amax / (448 * 6) rounded once
        if outer == oracle.OUTER_TENSOR:
            assert gs[0] == np.float32(xa.max()) / np.float32(2688.0)
            Sg = np.full((rows, K // 16), np.float64(gs[0]))
        else:
            amax_g = xa.reshape(rows, K // 128, 128).max(axis=2).astype(np.float32)
            assert np.array_equal(gs, np.where(amax_g > 0, amax_g / np.float32(2688.0), np.float32(1.0)))
            Sg = np.repeat(gs.astype(np.float64), 8, axis=1)
        amax_b = xa.reshape(rows, K // 16, 16).max(axis=2)
        s_lit = amax_b / Sg / 6.0
        sc_lit = _e4m3_literal(s_lit, up)
        sdiff = sc_lit != scales
        assert np.all(np.abs(sc_lit.astype(int) - scales.astype(int)) <= 1)
        assert np.all(_e4m3_boundary_distance(s_lit[sdiff], up) <= eps), law
        # the argument of round_FP4, on the oracle's own scale bytes
        Sb = np.repeat(E4M3[scales], 16, axis=1)
        Sg16 = np.repeat(Sg, 16, axis=1)
        nz = Sb > 0
        y_lit = np.divide(x.astype(np.float64), Sg16 * Sb, out=np.zeros((rows, K)), where=nz)
        rel = np.abs(y.astype(np.float64) - y_lit)[nz] / np.maximum(np.abs(y_lit[nz]), 1e-300)
        rel = rel[np.abs(y_lit[nz]) > 2.0 ** -100]
        assert rel.max() <= eps, (law, rel.max())
        if rounding == oracle.RTN:
            m_lit = _rtn_literal(np.abs(y_lit))
            m = _nibbles(codes) & 7
            cdiff = (m_lit != m) & nz
            assert np.all(np.abs(m_lit - m)[cdiff] == 1)
            a = np.abs(y_lit[cdiff])
            dist = np.min(np.abs(a[:, None] - RTN_THRESHOLDS), axis=1)
            assert np.all(dist <= eps * a), law
            # the fully literal pipeline (literal scale bytes too): how many codes differ in total
            Sb_l = np.repeat(E4M3[sc_lit], 16, axis=1)
            y_l = np.divide(x.astype(np.float64), Sg16 * Sb_l, out=np.zeros((rows, K)), where=Sb_l > 0)
            total = int(np.sum(_rtn_literal(np.abs(y_l)) != m))
            R1_REPORT[(law, outer)] = dict(elements=x.size, scale_bytes=scales.size, scales_differ=int(sdiff.sum()),
                                           codes_differ_same_scale=int(cdiff.sum()), codes_differ_literal=total,
                                           max_rel_y=float(rel.max()))
            # the open part is small: under 4 % of scale bytes, under 1 % of codes, on every value law
            assert sdiff.mean() < 0.04 and total < 0.01 * x.size, R1_REPORT[(law, outer)]
        else:
            # upward scales: never below the literal S_block by more than the rounding noise (nothing is clipped)
            assert np.all(E4M3[scales] >= np.minimum(s_lit, 448.0) * (1 - eps))


def test_r1_report(capsys):
    """prints the counts gathered above (run with -s to read them; the design document quotes them)"""
    for (law, outer), r in sorted(R1_REPORT.items()):
        print("R1 vs literal binary64, %-32s outer=%d: %d / %d scale bytes, %d / %d codes (%d with equal scales), max rel y %.2e"
              % (law, outer, r["scales_differ"], r["scale_bytes"], r["codes_differ_literal"], r["elements"],
                 r["codes_differ_same_scale"], r["max_rel_y"]))


# ------------------------------------------------------------------------------------------ R8

def test_r8_dequantized_value_is_the_exact_product_rounded_once():
    """A re-quantization (Q4, Q6 of Sec. 2.3) starts from the binary32 image of P * S_block * S_global.  P * S_block
    is exact (6 significant bits), so the image is the exact product rounded ONCE.  With an outer scale that is not a
    power of two the other association, P * RN(S_block * S_global), rounds twice and differs on some codes; the pin is
    the exact product (binary64 holds all 30 bits) rounded to binary32."""
    rng = np.random.default_rng(21)
    rows, K = 64, 256
    codes = rng.integers(0, 256, (rows, K // 2), dtype=np.uint8)
    scales = rng.integers(1, 0x7F, (rows, K // 16), dtype=np.uint8)
    n_alt = 0
    for sg in (np.float32(0.1), np.float32(3.1415927), np.float32(2688.0 / 7.0), np.float32(1.0000001), np.float32(2.0 ** -40 * 1.7)):
        q = oracle.NVFP4(codes, scales, np.array([sg], np.float32), 0.0, rows, K, oracle.OUTER_TENSOR)
        got = oracle.dequant_f32(q)
        nib = _nibbles(codes)
        P = np.where(nib & 8, -GRID_F[nib & 7], GRID_F[nib & 7])
        Sb = np.repeat(E4M3[scales], 16, axis=1)
        exact = P * Sb * np.float64(sg)                     # <= 2 + 4 + 24 significant bits: exact in binary64
        assert np.array_equal(got.view(np.uint32), exact.astype(np.float32).view(np.uint32))
        assert np.array_equal(oracle.dequant_f64(q), exact)
        alt = (P.astype(np.float32) * (Sb.astype(np.float32) * sg)).astype(np.float32)
        n_alt += int(np.sum(alt != got))
    assert n_alt > 100        # the other association is a different function on these inputs: the pin can tell them apart
    # block mode: every outer block its own scale
    gs = rng.uniform(0.01, 5.0, (rows, K // 128)).astype(np.float32)
    q = oracle.NVFP4(codes, scales, gs, 0.0, rows, K, oracle.OUTER_BLOCK128)
    nib = _nibbles(codes)
    P = np.where(nib & 8, -GRID_F[nib & 7], GRID_F[nib & 7])
    exact = P * np.repeat(E4M3[scales], 16, axis=1) * np.repeat(gs.astype(np.float64), 128, axis=1)
    assert np.array_equal(oracle.dequant_f32(q).view(np.uint32), exact.astype(np.float32).view(np.uint32))


# ------------------------------------------------------------------------------------------ R6

def _rotr(h, r):
    return ((h >> np.uint32(r)) | (h << np.uint32(32 - r))) if r else h


def test_quad_draws_share_bits_only_below_their_leading_byte_and_the_joint_law_is_bounded():
    """The four draws of a quad are the top 22 bits of one 32-bit word h rotated by 0, 8, 16, 24.  Structure (checked
    here on the oracle's output): the leading byte of each draw is a byte of h of its own, and two draws overlap only in
    bits that are at least 8 places down in one of them.  For uniform h it follows exactly that for any two thresholds
    |P(u_i >= t_i, u_j >= t_j) - P(u_i >= t_i) P(u_j >= t_j)| <= 2^-8 / 4 = 2^-10: the shared bits decide one of the
    two events only when that draw's leading byte ties with its threshold's (probability 2^-8), and a covariance of
    two events is at most 1/4.  The second half checks the overlaps and the worst case on 2^22 quads of the oracle's stream."""
    L = oracle.lib()
    key = L.oracle_stream_key(2025, 5)
    n = 1 << 22
    u = np.zeros(4 * n, np.uint32)
    L.oracle_rand22_fill(key, 4 * n, oracle._ptr(u))
    u = u.reshape(n, 4)
    h = np.array([L.oracle_quad_bits(p, key) for p in range(4096)], dtype=np.uint32)
    for i in range(4):
        assert np.array_equal(u[:4096, i], _rotr(h, 8 * i) >> np.uint32(10))
    # which bits of h each draw sees, most significant first
    bits = [[(31 - 8 * i - b) % 32 for b in range(22)] for i in range(4)]
    for i in range(4):
        for j in range(4):
            if i != j:
                assert not set(bits[i][:8]) & set(bits[j][:8])           # leading bytes are disjoint bytes of h
                shared = set(bits[i]) & set(bits[j])
                # a shared bit is below the leading byte in at least one of the two draws
                assert all(bits[i].index(b) >= 8 or bits[j].index(b) >= 8 for b in shared)
    # the overlaps, exactly: draw 1's low 14 bits are draw 0's top 14, draw 2's low 6 bits are draw 0's top 6, and
    # draw 3's top 14 bits are draw 0's low 14 (the same relations hold between draws i and i + k by rotation)
    assert np.array_equal(u[:, 1] & np.uint32(0x3FFF), u[:, 0] >> np.uint32(8))
    assert np.array_equal(u[:, 2] & np.uint32(0x3F), u[:, 0] >> np.uint32(16))
    assert np.array_equal(u[:, 3] >> np.uint32(8), u[:, 0] & np.uint32(0x3FFF))
    # worst case by construction for the pair (0, 1).  Thresholds: t0 in the middle (P = 1/2), t1 with leading byte T
    # and low part 2^13.  Given a tie of draw 1's leading byte with T the two events coincide (covariance 1/4, the
    # most two events can have); given no tie they are independent.  So joint - product = 2^-8 / 4 exactly.
    T = 100
    t0, t1 = 1 << 21, (T << 14) + (1 << 13)
    e0, e1 = u[:, 0] >= t0, u[:, 1] >= t1
    tie = (u[:, 1] >> np.uint32(14)) == T
    assert abs(tie.mean() - 2.0 ** -8) < 5 * 2.0 ** -4 / np.sqrt(n)
    assert np.array_equal(e0[tie], e1[tie])                               # coincide on the tie
    above = (u[:, 1] >> np.uint32(14)) > T
    assert e1[above].all() and not e1[~above & ~tie].any()                # decided by the leading byte otherwise
    noise = 5 * 0.5 / np.sqrt(n)
    joint, prod = np.mean(e0 & e1), np.mean(e0) * np.mean(e1)
    assert abs(joint - prod) <= 2.0 ** -10 + noise
    # and for every pair, at thresholds where the leading bits decide: nothing beyond sampling noise
    for i in range(4):
        for j in range(i + 1, 4):
            a, b = u[:, i] >= (1 << 21), u[:, j] >= (3 << 20)
            assert abs(np.mean(a & b) - np.mean(a) * np.mean(b)) < noise, (i, j)


# ------------------------------------------------------------------------------------------ R12 (Sec. 4.1)

def _h16():
    H = np.array([[1.0]])
    for _ in range(4):
        H = np.block([[H, H], [H, -H]])                         # the paper's recursion, the four factors 1 / sqrt 2 ...
    return H / 4.0                                              # ... collected: (1 / sqrt 2)^4 = 1 / 4 exactly


def _signs(K, seed, rid):
    L = oracle.lib()
    key = L.oracle_stream_key(seed, rid)
    return np.array([-1.0 if L.oracle_rht_sign(k, key) else 1.0 for k in range(K)])


def test_rht_is_x_s_h_block_diagonal():
    """Sec. 4.1: A' = A S_n H_n with H_n = diag{H_16, ...} and S_n a random diagonal of +-1.  The oracle's binary32
    butterflies against that matrix product in binary64: equal on small integers (every sum exact), within a few
    roundings otherwise; the signs depend on the position along K only."""
    rng = np.random.default_rng(31)
    K, rows = 96, 20
    S = _signs(K, 5, 7)
    H = np.kron(np.eye(K // 16), _h16())
    assert np.allclose(H @ H.T, np.eye(K)) and np.allclose(H, H.T)
    xi = rng.integers(-8, 9, (rows, K)).astype(np.float32) * 4          # multiples of 4: the final 1/4 stays exact
    assert np.array_equal(oracle.rht16(xi, 5, 7).astype(np.float64), (xi.astype(np.float64) * S) @ H)
    x = wl.bf16_to_f32(wl.normal_bf16((rows, K), 1.0, 32, 1e-2, 50.0))
    got = oracle.rht16(x, 5, 7).astype(np.float64)
    want = (x.astype(np.float64) * S) @ H
    bound = 5 * 2.0 ** -24 * 0.25 * np.abs(x.astype(np.float64)).reshape(rows, K // 16, 16).sum(axis=2).repeat(16, axis=1)
    assert np.all(np.abs(got - want) <= bound + 1e-300)
    # a second row, another seed: same positions flip for every row of one stream, other positions for another stream
    assert np.array_equal(np.sign(oracle.rht16(np.ones((3, K), np.float32), 5, 7)), np.sign(np.tile((S @ H), (3, 1))))
    assert not np.array_equal(_signs(K, 5, 7), _signs(K, 6, 7)) and not np.array_equal(_signs(K, 5, 7), _signs(K, 5, 0))


def test_rht_on_both_operands_leaves_the_product_unchanged():
    """Sec. 4.1: A B^T = (A S H)(B S H)^T since S and H are orthogonal: on the unquantized operands, in binary64 of
    the oracle's binary32 output, to rounding."""
    A = wl.bf16_to_f32(wl.outlier_channel_bf16(24, 256, 41))
    B = wl.bf16_to_f32(wl.normal_bf16((40, 256), 0.02, 42))
    ref = A.astype(np.float64) @ B.astype(np.float64).T
    At, Bt = oracle.rht16(A, 9, 15).astype(np.float64), oracle.rht16(B, 9, 15).astype(np.float64)
    scale = np.abs(A.astype(np.float64)) @ np.abs(B.astype(np.float64)).T
    assert np.all(np.abs(At @ Bt.T - ref) <= 1e-5 * scale)
    # different signs on the two sides do change it
    Bo = oracle.rht16(B, 9, 16).astype(np.float64)
    assert np.abs(At @ Bo.T - ref).max() > 1e-2 * np.abs(ref).max()


def test_rht_sign_bits_use_every_bit_of_a_word_once_and_are_balanced():
    L = oracle.lib()
    key = L.oracle_stream_key(77, 7)
    for wi in (0, 1, 5):
        w = L.oracle_quad_bits(wi, key)
        bits = [L.oracle_rht_sign(32 * wi + k, key) for k in range(32)]
        pos = [(15 + (k >> 1) + 16 * (k & 1)) & 31 for k in range(32)]
        assert sorted(pos) == list(range(32))
        assert bits == [(w >> p) & 1 for p in pos]
    s = np.array([L.oracle_rht_sign(k, key) for k in range(1 << 14)])
    assert abs(s.mean() - 0.5) < 5 * 0.5 / np.sqrt(len(s))
    assert abs(np.corrcoef(s[:-1], s[1:])[0, 1]) < 0.05 and abs(np.corrcoef(s[:-16], s[16:])[0, 1]) < 0.05


def test_rht_spreads_an_outlier_and_the_quantized_backward_products_stay_unbiased():
    """What Sec. 4.1 is for: one huge entry in a group of 16 forces a scale under which the others vanish; after the
    transform the group is flat.  And the layer's backward products with the transform on both operands
    (1 x 128 outer blocks, stochastic rounding) are still unbiased estimates of the product of the aligned tensors."""
    x = np.full((1, 16), 0.01, np.float32)
    x[0, 3] = 100.0
    t = oracle.rht16(x, 1, 7)
    assert np.abs(t).max() / np.abs(t).min() < 1.01 and np.abs(x).max() / np.abs(x).min() > 1e3
    N, D, C = 128, 128, 128
    Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed=3)
    O = oracle.OUTER_BLOCK128
    Xq, Wq = oracle.linear_fwd(Xb, Wb, outer=O)
    dY = wl.bf16_to_f32(dYb).astype(np.float64)
    ref_dx = dY @ oracle.dequant_f64(Wq)
    acc = np.zeros_like(ref_dx)
    n = 24
    for seed in range(n):
        a, b = oracle.linear_bwd_dx_operands(dYb, Wq, seed, 1, outer=O, rht=True)
        acc += oracle.gemm_nt(a, b)[0]
    err_mean = np.abs(acc / n - ref_dx).mean()
    a, b = oracle.linear_bwd_dx_operands(dYb, Wq, 0, 1, outer=O, rht=True)
    err_one = np.abs(oracle.gemm_nt(a, b)[0] - ref_dx).mean()
    assert err_mean < 0.45 * err_one                          # averaging seeds shrinks the error (~ 1 / sqrt n): no bias floor
