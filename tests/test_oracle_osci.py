"""Pins for the oracle's OsciReset functions (Sec. 3.2-3.3, Alg. 1; Appendix Alg. 2) against hand-computed trajectories.

The weight matrix is built so that every scale is known in closed form: each 1 x 128 outer block holds one element
of magnitude 2688 (S_global = 2688 / (448 * 6) = 1; its group of 16 gets S_block = 448) and every other group of 16
holds an element of magnitude 6 (S_block = 6 / 6 = 1), so in those groups Q(w) is the nearest FP4 value to w itself.
"""
import numpy as np
import pytest

import oracle

TAU = 8.0       # the oscillation-risk threshold of the paper's hyper-parameter table


def base_matrix(rows=4, K=256):
    W = np.zeros((rows, K), np.float32)
    W[:, 0::128] = 2688.0            # group 0 of every outer block: S_block 448
    W[:, 16::16] = 6.0               # every group of 16 has a 6 -> S_block 1 (the 2688 groups aside)
    W[:, 0::128] = 2688.0
    return W


def test_quant_dequant_is_nearest_fp4_value_times_scale():
    W = base_matrix()
    vals = np.array([0.1, 0.24, 0.26, 0.74, 0.76, 1.2, 1.3, 1.74, 1.76, 2.4, 2.6, 3.4, 3.6, 4.9, 5.1, -0.26, -2.6], np.float32)
    want = np.array([0.0, 0.0, 0.5, 0.5, 1.0, 1.0, 1.5, 1.5, 2.0, 2.0, 3.0, 3.0, 4.0, 4.0, 6.0, -0.5, -3.0], np.float32)
    for g in range(len(vals)):
        W[1, 16 * (1 + g % 7) + 1 + g // 7] = vals[g]
    Q = oracle.quant_dequant_weight(W)
    for g in range(len(vals)):
        assert Q[1, 16 * (1 + g % 7) + 1 + g // 7] == want[g], (vals[g], want[g])
    assert np.all(Q[:, 0::128] == 2688.0) and Q[0, 16] == 6.0
    # in the group scaled by 448 the grid is 448 x FP4 values
    W2 = base_matrix()
    W2[0, 1] = 300.0                 # / 448 = 0.67 -> 0.5 -> 224
    assert oracle.quant_dequant_weight(W2)[0, 1] == 224.0


def test_update_and_suppress_on_hand_made_trajectories():
    """An element hopping 0.24 <-> 0.26 crosses the 0 / 0.5 decision threshold every step: dist_Q = 0.5 T against
    dist_M = 0.02 T, risk 25 >= 8 -> reset to its bin centre.  An element drifting 1.0 -> 2.0 in steps of 0.1 moves its
    quantized value as far as itself: risk 1 -> kept.  An element that never moves has 0 / 0 -> kept."""
    W = base_matrix()
    osc, drift, still = (2, 17), (2, 33), (2, 49)
    T = 10
    W[osc], W[drift], W[still] = 0.24, 1.0, 1.3
    Wp, dm, dq = np.empty_like(W), np.full_like(W, 7.0), np.full_like(W, 7.0)
    oracle.osci_update(W, Wp, dm, dq, 0)
    assert not dm.any() and not dq.any() and np.array_equal(Wp, W)          # t0 = 0: cleared, snapshot taken
    for t in range(1, T + 1):
        W[osc] = 0.26 if t % 2 else 0.24
        W[drift] = np.float32(1.0 + 0.1 * t)
        oracle.osci_update(W, Wp, dm, dq, t)
        assert np.array_equal(Wp, W)
    assert dq[osc] == 0.5 * T and abs(dm[osc] - 0.02 * T) < 1e-5
    assert abs(dm[drift] - 1.0) < 1e-5 and dq[drift] == 1.0                 # 1.0 -> 2.0 through 1.5: |dQ| sums to 1
    assert dm[still] == 0 and dq[still] == 0
    assert dq[osc] / dm[osc] > TAU > dq[drift] / dm[drift]
    untouched = (dm == 0) & (dq == 0)
    assert untouched.sum() == W.size - 2
    before = W.copy()
    n = oracle.osci_suppress(W, dm, dq, TAU)
    assert n == 1
    assert W[osc] == oracle.quant_dequant_weight(before)[osc] == 0.0        # T even: ends at 0.24 -> bin centre 0
    changed = W != before
    assert changed.sum() == 1 and changed[osc]
    # the reset leaves the quantized weights as they were (Sec. 3.3, first effect)
    assert np.array_equal(oracle.quant_dequant_weight(W), oracle.quant_dequant_weight(before))


def test_risk_threshold_is_inclusive_and_resets_are_counted():
    W = base_matrix()
    dm, dq = np.zeros_like(W), np.zeros_like(W)
    a, b, c = (0, 18), (0, 19), (0, 20)
    W[a], W[b], W[c] = 0.3, 0.3, 0.3
    dm[a], dq[a] = 1.0, 8.0          # risk exactly tau: reset (Alg. 1: risk >= tau)
    dm[b], dq[b] = 1.0, 7.999        # just below: kept
    dm[c], dq[c] = 0.0, 1.0          # never moved but quantized value did (scale change): risk = inf: reset
    n = oracle.osci_suppress(W, dm, dq, TAU)
    assert n == 2 and W[a] == 0.5 and W[b] == np.float32(0.3) and W[c] == 0.5


def test_random_walk_statistics_match_a_numpy_evaluation_of_the_definitions():
    """dist_M = sum_t |w_t - w_{t-1}| and dist_Q = sum_t |Q(w_t) - Q(w_{t-1})| (Sec. 3.2), evaluated independently with
    numpy on the sequence of oracle quant-dequant outputs."""
    rng = np.random.default_rng(3)
    W = (rng.standard_normal((8, 256)) * 0.02).astype(np.float32)
    Wp, dm, dq = np.empty_like(W), np.empty_like(W), np.empty_like(W)
    oracle.osci_update(W, Wp, dm, dq, 0)
    seq = [W.copy()]
    for t in range(1, 6):
        W = (W + rng.standard_normal(W.shape).astype(np.float32) * 2e-4).astype(np.float32)
        oracle.osci_update(W, Wp, dm, dq, t)
        seq.append(W.copy())
    M = sum(np.abs(seq[t].astype(np.float64) - seq[t - 1]) for t in range(1, 6))
    Q = [oracle.quant_dequant_weight(w).astype(np.float64) for w in seq]
    DQ = sum(np.abs(Q[t] - Q[t - 1]) for t in range(1, 6))
    assert np.allclose(dm, M, rtol=1e-5, atol=1e-9) and np.allclose(dq, DQ, rtol=1e-5, atol=1e-9)
    assert (dq > 0).mean() > 0.02                       # some quantized values did move


def test_bad_shapes():
    W = np.zeros((2, 64), np.float32)
    with pytest.raises(ValueError):
        oracle.quant_dequant_weight(W)                  # K % 128


# ---- memory-efficient statistics (Appendix Alg. 3) ----------------------------------------------------------------

def test_sensitivity_score_by_hand_in_every_bin():
    """In the groups of base_matrix the scale is 1 (or 448), so the score can be worked out by hand from the FP4 grid:
    |w - nearest value| over the length of the interval that rounds to that value (0.5 up to 1.5; 1.75..2.5 for 2;
    2.5..3.5 for 3; 3.5..5 for 4; 5..6 for 6)."""
    W = base_matrix()
    cases = [(0.1, 0.1 / 0.5), (0.3, 0.2 / 0.5), (1.1, 0.1 / 0.5), (1.6, 0.1 / 0.5), (2.2, 0.2 / 0.75), (1.8, 0.2 / 0.75),
             (3.4, 0.4 / 1.0), (2.6, 0.4 / 1.0), (4.9, 0.9 / 1.5), (3.6, 0.4 / 1.5), (5.2, 0.8 / 1.0), (-2.2, 0.2 / 0.75),
             (6.0, 0.0), (0.0, 0.0), (0.25, 0.5), (0.75, 0.5)]                 # the last two sit on a rounding threshold
    pos = [(1, 16 * (1 + g % 7) + 1 + g // 7) for g in range(len(cases))]
    for p, (w, _) in zip(pos, cases):
        W[p] = w
    W[3, 1] = 448 * 1.1                                                        # group scaled by 448: same score as 1.1
    q, s = oracle.osci_scores(W)
    assert np.array_equal(q, oracle.quant_dequant_weight(W))
    for p, (w, want) in zip(pos, cases):
        assert abs(float(s[p]) - want) < 2e-6, (w, float(s[p]), want)
    assert abs(float(s[3, 1]) - 0.2) < 2e-6
    assert s[0, 0] == 0 and np.all(s >= 0) and np.all(s <= 0.8 + 1e-6)
    # an all-zero outer block: scale 1 by convention, everything scores 0
    Z = np.zeros((1, 128), np.float32)
    assert not oracle.osci_scores(Z)[1].any()


def test_selection_takes_the_largest_scores_and_equal_scores_in_index_order():
    W = base_matrix(rows=2, K=256)
    # scores (scale 1): 0.4 at three places, 0.2 at two, 0.5 once
    W[0, 17], W[0, 40], W[1, 150] = 0.3, 1.3, 0.7           # |.|: 0.2 / 0.5 = 0.4 each
    W[0, 20], W[1, 21] = 1.1, 0.6                            # 0.2
    W[1, 100] = 0.25                                         # 0.5: on the threshold
    flat = lambda r, c: r * 256 + c
    idx, wm, wq, dm, dq = oracle.osci_select(W, 3)
    assert idx.dtype == np.uint32 and list(idx) == [flat(0, 17), flat(0, 40), flat(1, 100)]      # 0.5, then the two first 0.4
    assert list(wm) == [np.float32(0.3), np.float32(1.3), np.float32(0.25)] and list(wq) == [0.5, 1.5, 0.0]
    assert not dm.any() and not dq.any()
    idx4 = oracle.osci_select(W, 4)[0]
    assert list(idx4) == [flat(0, 17), flat(0, 40), flat(1, 100), flat(1, 150)]
    idx6 = oracle.osci_select(W, 6)[0]
    assert list(idx6) == sorted([flat(0, 17), flat(0, 40), flat(1, 100), flat(1, 150), flat(0, 20), flat(1, 21)])
    assert len(oracle.osci_select(W, 0)[0]) == 0
    # property on random weights: nothing outside the selection scores higher than anything inside
    rng = np.random.default_rng(3)
    R = (rng.standard_normal((8, 384)) * 0.02).astype(np.float32)
    s = oracle.osci_scores(R)[1].reshape(-1)
    k = 150
    sel = oracle.osci_select(R, k)[0]
    assert len(sel) == k and np.all(np.diff(sel.astype(np.int64)) > 0)
    mask = np.zeros(R.size, bool)
    mask[sel] = True
    assert s[mask].min() >= s[~mask].max()


def test_tracking_every_element_is_the_dense_algorithm():
    """With every element selected, Alg. 3 is Alg. 2, and the reset on the subset is Alg. 1: same states bit for bit
    over a period of random walks (the pin of the dense functions therefore carries over)."""
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((6, 256)) * 0.02).astype(np.float32)
    Wd = W.copy()
    Wp, dm, dq = np.empty_like(W), np.empty_like(W), np.empty_like(W)
    oracle.osci_update(Wd, Wp, dm, dq, 0)
    idx, wm, wq, sm, sq = oracle.osci_select(W, W.size)
    assert np.array_equal(idx, np.arange(W.size))
    for t in range(1, 7):
        step = (rng.standard_normal(W.shape) * 2e-3).astype(np.float32) * (rng.random(W.shape) < 0.5)
        W += step
        Wd += step
        oracle.osci_update(Wd, Wp, dm, dq, t)
        oracle.osci_update_sparse(W, idx, wm, wq, sm, sq)
        assert np.array_equal(sm, dm.reshape(-1)) and np.array_equal(sq, dq.reshape(-1))
        assert np.array_equal(wm, Wp.reshape(-1)) and np.array_equal(wq, oracle.quant_dequant_weight(Wp).reshape(-1))
    n_dense = oracle.osci_suppress(Wd, dm, dq, TAU)
    n_sparse = oracle.osci_suppress_sparse(W, idx, sm, sq, TAU)
    assert n_dense == n_sparse > 0 and np.array_equal(W, Wd)


def test_subset_tracks_the_oscillating_element_of_the_hand_made_trajectory():
    """The element hopping 0.24 <-> 0.26 sits next to a threshold (score 0.48): it is in a 5 % selection, is reset after
    the period, and nothing outside the selection is touched."""
    W = base_matrix()
    rng = np.random.default_rng(5)
    free = np.ones(W.shape, bool)
    free[:, 0::16] = False
    W[free] = (np.round(rng.uniform(0, 6, free.sum()) * 2) / 2).astype(np.float32)       # bin centres and thresholds mixed
    W[free] = np.where(np.isin(W[free], [0, .5, 1, 1.5, 2, 3, 4, 6]), W[free], 3.0)      # keep bin centres only: score 0
    osc = (2, 17)
    W[osc] = 0.24
    k = max(1, W.size // 20)
    idx, wm, wq, sm, sq = oracle.osci_select(W, k)
    j = int(np.searchsorted(idx, osc[0] * W.shape[1] + osc[1]))
    assert idx[j] == osc[0] * W.shape[1] + osc[1]
    before = W.copy()
    for t in range(1, 11):
        W[osc] = 0.26 if t % 2 else 0.24
        oracle.osci_update_sparse(W, idx, wm, wq, sm, sq)
    assert sq[j] == 5.0 and abs(sm[j] - 0.2) < 1e-5
    assert oracle.osci_suppress_sparse(W, idx, sm, sq, TAU) == 1
    assert W[osc] == 0.0                                    # 0.24 rounds to the value 0: the centre of its bin
    W[osc] = before[osc]
    assert np.array_equal(W, before)
