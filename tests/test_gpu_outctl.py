"""GPU parity of the OutControl split linear (Sec. 4.2) with the oracle: the NVFP4 parts are the layer's own quantizers
and products (byte parity is covered elsewhere; here the contexts are checked again), the outlier channels run on the
bf16 matrix path; every output within 1e-3 |ref| + 1e-6 sum |a||b| (FP32 output) of the float64 reference."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu


def dev_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def check(got, ref, absref, what):
    g = got.double().cpu().numpy()
    rel = 1e-3 if got.dtype == torch.float32 else 2.0 ** -8
    err, tol = np.abs(g - ref), rel * np.abs(ref) + 1e-6 * absref + 1e-30
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert np.all(err <= tol), "%s: err %.3e tol %.3e at %s" % (what, err[worst], tol[worst], worst)


def inputs(N, D_lo, D_hp, C, seed):
    """activations with the last D_hp channels (the static outlier set, already split off) 30 x larger"""
    rng = np.random.default_rng(seed)
    Xl = wl.normal_bf16((N, D_lo), 1.0, seed, 1e-3, 50.0)
    Xh = wl.f32_to_bf16(rng.standard_normal((N, D_hp)).astype(np.float32) * 30.0)
    Wl, Wh = wl.normal_bf16((C, D_lo), 0.02, seed + 1), wl.normal_bf16((C, D_hp), 0.02, seed + 2)
    dY = wl.normal_bf16((N, C), 1e-3, seed + 3)
    return Xl, Wl, Xh, Wh, dY


@pytest.mark.parametrize("N,D_lo,D_hp,C,outer,rht", [(256, 384, 64, 320, 0, False), (384, 256, 32, 128, 1, False),
                                                     (1152, 896, 128, 640, 1, True), (192, 128, 0, 64, 0, False)])
@pytest.mark.parametrize("out_dtype", [1, 0])
def test_split_linear_forward_and_backward(N, D_lo, D_hp, C, outer, rht, out_dtype):
    import paper_2510_27527_amd as tj
    B = tj.binding
    Xl, Wl, Xh, Wh, dYb = inputs(N, D_lo, D_hp, C, 70 + N)
    dXl, dWl, dXh, dWh, dY = (dev_bf16(a) for a in (Xl, Wl, Xh, Wh, dYb))
    Y, Xq, Wq = tj.outctl_fwd(dXl, dWl, dXh, dWh, out_dtype, outer=outer)
    oXq, oWq, Yref, Yabs = oracle.outctl_fwd(Xl, Wl, Xh, Wh, outer=outer)
    torch.cuda.synchronize()
    assert np.array_equal(Xq.codes.cpu().numpy(), oXq.codes) and np.array_equal(Wq.scales.cpu().numpy(), oWq.scales)
    check(Y, Yref, Yabs, "Y")
    got = tj.outctl_bwd(dY, Xq, Wq, dXh, dWh, 9, 3, out_dtype, rht=rht)
    ref = oracle.outctl_bwd(dYb, oXq, oWq, Xh, Wh, 9, 3, rht=rht)
    torch.cuda.synchronize()
    for name, g in zip(("dX_lo", "dX_hp", "dW_lo", "dW_hp"), got):
        if name in ref:
            check(g, *ref[name], name)
        else:
            assert g.numel() == 0
    # the ordinary channels' gradients are those of the plain layer on them
    dX0, dW0 = tj.linear_bwd(dY, Xq, Wq, 9, 3, out_dtype, rht=rht)
    torch.cuda.synchronize()
    assert torch.equal(got[0], dX0) and torch.equal(got[2], dW0)


def test_high_precision_product_and_transpose_on_ragged_shapes():
    """the bf16 products on shapes that are no multiples of their 128 x 128 tile (token counts 64, 192, 320; 96 and 160
    outlier channels; 192 and 320 outputs)"""
    import paper_2510_27527_amd as tj
    B = tj.binding
    for (N, D_hp, C) in [(0, 32, 64), (130, 96, 192), (260, 160, 320)]:
        Xl, Wl, Xh, Wh, dYb = inputs(N - N % 64 + 64, 128, D_hp, C, 5 + C)
        Nn = Xl.shape[0]
        args = [dev_bf16(a) for a in (Xl, Wl, Xh, Wh)]
        Y, Xq, Wq = tj.outctl_fwd(*args, B.OUT_F32)
        _, _, Yref, Yabs = oracle.outctl_fwd(Xl, Wl, Xh, Wh)
        check(Y, Yref, Yabs, "Y ragged")
        got = tj.outctl_bwd(dev_bf16(dYb), Xq, Wq, args[2], args[3], 1, 0, B.OUT_F32)
        ref = oracle.outctl_bwd(dYb, *oracle.linear_fwd(Xl, Wl), Xh, Wh, 1, 0)
        check(got[3], *ref["dW_hp"], "dW_hp ragged")
        check(got[1], *ref["dX_hp"], "dX_hp ragged")


def test_bad_arguments():
    import paper_2510_27527_amd as tj
    B = tj.binding
    Xl, Wl, Xh, Wh, dYb = inputs(64, 128, 32, 64, 1)
    a = [dev_bf16(x) for x in (Xl, Wl, Xh, Wh)]
    bad = torch.zeros((64, 48), dtype=torch.bfloat16, device="cuda")          # D_hp % 32
    badw = torch.zeros((64, 48), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.NVFP4Error) as e:
        tj.outctl_fwd(a[0], a[1], bad, badw)
    assert e.value.code == -2
    torch.cuda.synchronize()


@pytest.mark.parametrize("N,D_lo,D_hp,C", [(3648, 64, 96, 3520), (64, 64, 3520, 3648)])
@pytest.mark.parametrize("out_dtype", [1, 0])
def test_high_precision_product_with_256x256_tiles(N, D_lo, D_hp, C, out_dtype):
    """outputs of more than 192 tiles of 256 x 256 take the large-tile instantiation of the bf16 product: the forward term
    (with the FP4 product as addend) in the first case, the weight gradient of the outlier channels (no addend) in the
    second; both ragged in both directions"""
    import paper_2510_27527_amd as tj
    Xl, Wl, Xh, Wh, dYb = inputs(N, D_lo, D_hp, C, 11 + N)
    args = [dev_bf16(a) for a in (Xl, Wl, Xh, Wh)]
    Y, Xq, Wq = tj.outctl_fwd(*args, out_dtype)
    oXq, oWq, Yref, Yabs = oracle.outctl_fwd(Xl, Wl, Xh, Wh)
    torch.cuda.synchronize()
    check(Y, Yref, Yabs, "Y")
    got = tj.outctl_bwd(dev_bf16(dYb), Xq, Wq, args[2], args[3], 4, 1, out_dtype)
    ref = oracle.outctl_bwd(dYb, oXq, oWq, Xh, Wh, 4, 1)
    torch.cuda.synchronize()
    for name, g in zip(("dX_lo", "dX_hp", "dW_lo", "dW_hp"), got):
        check(g, *ref[name], name)
