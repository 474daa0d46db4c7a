"""GPU parity of the OsciReset kernels (Sec. 3.2-3.3: Alg. 1; Appendix Alg. 2) with the CPU oracle: every float bit for bit.

Weights follow the paper's setting at the end of training: N(0, 0.02) master weights that move by small steps, a
fraction of them hopping across a quantization threshold (the oscillators of Sec. 3.1)."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu

TAU = 8.0


def bits(a):
    return np.ascontiguousarray(a).view(np.uint32)


def trajectory(shape, seed, steps):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal(shape) * 0.02).astype(np.float32)
    W[0, :128] = 0.0                                   # an all-zero outer block
    seq = [W.copy()]
    Q = oracle.quant_dequant_weight(W)
    osc = rng.random(shape) < 0.05                     # elements that hop around their own value
    amp = np.abs(W - Q) * 0.0 + np.abs(W) * 0.08
    for t in range(1, steps + 1):
        step = rng.standard_normal(shape).astype(np.float32) * 1e-5
        W = (W + step + np.where(osc, amp * (1 if t % 2 else -1), 0)).astype(np.float32)
        seq.append(W.copy())
    return seq


@pytest.mark.parametrize("shape", [(16, 128), (300, 1152), (2048, 1024)])
def test_update_and_suppress_match_the_oracle(shape):
    import paper_2510_27527_amd as tj
    tj.binding.lib()
    steps = 6
    seq = trajectory(shape, 11 + shape[0], steps)
    oWp, odm, odq = np.empty(shape, np.float32), np.full(shape, 3.0, np.float32), np.full(shape, 3.0, np.float32)
    gWp = torch.full(shape, 5.0, device="cuda")
    gdm = torch.full(shape, 3.0, device="cuda")
    gdq = torch.full(shape, 3.0, device="cuda")
    for t, W in enumerate(seq):
        oracle.osci_update(W, oWp, odm, odq, t)
        tj.osci_update(torch.from_numpy(W).cuda(), gWp, gdm, gdq, t)
        torch.cuda.synchronize()
        assert np.array_equal(bits(gWp.cpu().numpy()), bits(oWp)), t
        assert np.array_equal(bits(gdm.cpu().numpy()), bits(odm)), t
        assert np.array_equal(bits(gdq.cpu().numpy()), bits(odq)), t
    assert (odq > 0).mean() > 0.01
    oW = seq[-1].copy()
    gW = torch.from_numpy(seq[-1]).cuda()
    n = torch.zeros(1, dtype=torch.int64, device="cuda")
    want = oracle.osci_suppress(oW, odm, odq, TAU)
    tj.osci_suppress(gW, gdm, gdq, TAU, n)
    tj.osci_suppress(gW.clone(), gdm, gdq, TAU)        # without a counter
    torch.cuda.synchronize()
    assert int(n.item()) == want and 0 < want < oW.size
    assert np.array_equal(bits(gW.cpu().numpy()), bits(oW))
    # a reset weight sits on its bin centre: quantizing again returns it unchanged
    changed = oW != seq[-1]
    assert changed.sum() <= want
    assert np.array_equal(oracle.quant_dequant_weight(oW)[changed], oW[changed])


def test_empty_and_bad_arguments():
    import paper_2510_27527_amd as tj
    B = tj.binding
    z = torch.zeros((0, 128), device="cuda")
    tj.osci_update(z, z.clone(), z.clone(), z.clone(), 0)
    tj.osci_suppress(z, z.clone(), z.clone(), TAU)
    w = torch.zeros((4, 192), device="cuda")
    with pytest.raises(B.NVFP4Error) as e:
        tj.osci_update(w, w.clone(), w.clone(), w.clone(), 1)
    assert e.value.code == -2
    w = torch.zeros((4, 128), device="cuda")
    with pytest.raises(B.NVFP4Error) as e:
        tj.osci_suppress(w, w.clone(), w.clone(), 0.0)
    assert e.value.code == -3
    torch.cuda.synchronize()


# ---- memory-efficient statistics (Appendix Alg. 3) ----------------------------------------------------------------

def u32(t):
    return t.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("shape,frac", [((16, 128), 0.05), ((300, 1152), 0.05), ((2048, 1024), 0.05), ((300, 1152), 1.0),
                                        ((17, 128), 0.5), ((64, 256), 1.0 / 16384)])
def test_tracked_subset_matches_the_oracle(shape, frac):
    """selection (indices and snapshots), every later step and the reset, bit for bit; 2048 x 1024 spans 1024 tiles of
    the compaction, 17 x 128 ends in a partial tile, the last case tracks a single element"""
    import paper_2510_27527_amd as tj
    steps = 5
    seq = trajectory(shape, 23 + shape[0], steps)
    k = max(1, int(np.ceil(frac * seq[0].size)))
    o = list(oracle.osci_select(seq[0], k))
    g = list(tj.osci_select(torch.from_numpy(seq[0]).cuda(), k))
    torch.cuda.synchronize()
    assert np.array_equal(u32(g[0]), o[0])
    for a, b in zip(g[1:], o[1:]):
        assert np.array_equal(bits(a.cpu().numpy()), bits(b))
    for t in range(1, steps + 1):
        oracle.osci_update_sparse(seq[t], *o)
        tj.osci_update_sparse(torch.from_numpy(seq[t]).cuda(), *g)
        torch.cuda.synchronize()
        for a, b in zip(g[1:], o[1:]):
            assert np.array_equal(bits(a.cpu().numpy()), bits(b)), t
    oW, gW = seq[-1].copy(), torch.from_numpy(seq[-1]).cuda()
    n = torch.zeros(1, dtype=torch.int64, device="cuda")
    want = oracle.osci_suppress_sparse(oW, o[0], o[3], o[4], TAU)
    tj.osci_suppress_sparse(gW, g[0], g[3], g[4], TAU, n)
    torch.cuda.synchronize()
    assert int(n.item()) == want
    assert np.array_equal(bits(gW.cpu().numpy()), bits(oW))
    if frac == 0.05 and shape[0] >= 300:
        assert want > 0                                 # the hopping elements sit next to thresholds: they are tracked


def test_selection_with_many_equal_scores():
    """weights on a coarse grid give scores with long runs of exact ties, also at the selection threshold: the first
    ones in index order belong to the subset"""
    import paper_2510_27527_amd as tj
    rng = np.random.default_rng(2)
    W = np.zeros((64, 512), np.float32)
    W[:, 0::128] = 2688.0
    W[:, 16::16] = 6.0
    W[:, 0::128] = 2688.0
    free = np.ones(W.shape, bool)
    free[:, 0::16] = False
    W[free] = rng.choice(np.array([0.0, 0.1, 0.2, 0.6, 1.1, 1.9, 2.2, 3.4, 5.5], np.float32), free.sum())
    for k in (1, 100, 5000, 20000, W.size):
        o = oracle.osci_select(W, k)
        g = tj.osci_select(torch.from_numpy(W).cuda(), k)
        torch.cuda.synchronize()
        assert np.array_equal(u32(g[0]), o[0]), k
        assert np.array_equal(bits(g[2].cpu().numpy()), bits(o[2])), k


def test_subset_calls_empty_and_bad_arguments():
    import paper_2510_27527_amd as tj
    B = tj.binding
    w = torch.zeros((4, 128), device="cuda")
    st = tj.osci_select(w, 0)
    assert all(t.numel() == 0 for t in st)
    tj.osci_update_sparse(w, *st)
    tj.osci_suppress_sparse(w, st[0], st[3], st[4], TAU)
    z = torch.zeros((0, 128), device="cuda")
    tj.osci_select(z, 0)
    with pytest.raises(B.NVFP4Error) as e:
        tj.osci_select(w, w.numel() + 1)
    assert e.value.code == -2
    with pytest.raises(B.NVFP4Error) as e:
        tj.osci_select(torch.zeros((4, 192), device="cuda"), 1)
    assert e.value.code == -2
    st = tj.osci_select(w, 3)
    with pytest.raises(B.NVFP4Error) as e:
        tj.osci_suppress_sparse(w, st[0], st[3], st[4], 0.0)
    assert e.value.code == -3
