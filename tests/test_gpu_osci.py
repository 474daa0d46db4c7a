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
