"""Pins for the oracle's OutControl split linear (Sec. 4.2): it is a composition of pinned pieces (the quantizers, the
float64 product), so what is checked here is the composition: the limits D_hp = 0 and D_lo -> all-hp, the shapes, and
the effect the section describes (keeping the structural outlier channels in high precision lowers the forward error)."""
import numpy as np

import oracle
import workloads as wl


def split(bits, hp_cols):
    lo = np.setdiff1d(np.arange(bits.shape[1]), hp_cols)
    return np.ascontiguousarray(bits[:, lo]), np.ascontiguousarray(bits[:, hp_cols])


def test_no_outlier_channels_is_the_plain_layer_and_all_high_precision_is_the_exact_product():
    N, D, C = 64, 256, 48
    Xb, Wb, dYb = wl.linear_inputs(N, D, C, seed=8)
    none = np.zeros((N, 0), np.uint16), np.zeros((C, 0), np.uint16)
    Xq, Wq, Y, Ab = oracle.outctl_fwd(Xb, Wb, none[0], none[1])
    Y0, Ab0 = oracle.gemm_nt(*oracle.linear_fwd(Xb, Wb))
    assert np.array_equal(Y, Y0) and np.array_equal(Ab, Ab0)
    res = oracle.outctl_bwd(dYb, Xq, Wq, none[0], none[1], 3, 1)
    assert set(res) == {"dX_lo", "dW_lo"}
    assert np.array_equal(res["dX_lo"][0], oracle.gemm_nt(*oracle.linear_bwd_dx_operands(dYb, Wq, 3, 1))[0])
    # the high-precision term alone is the exact product of the bf16 values
    Xl, Xh = split(Xb, np.arange(128, 256))
    Wl, Wh = split(Wb, np.arange(128, 256))
    _, _, Ys, _ = oracle.outctl_fwd(Xl, Wl, Xh, Wh)
    _, _, Yl, _ = oracle.outctl_fwd(Xl, Wl, none[0], none[1])
    exact_h = wl.bf16_to_f32(Xh).astype(np.float64) @ wl.bf16_to_f32(Wh).astype(np.float64).T
    assert np.allclose(Ys - Yl, exact_h, rtol=1e-12, atol=1e-12)
    r = oracle.outctl_bwd(dYb, *oracle.linear_fwd(Xl, Wl), Xh, Wh, 3, 1)
    assert r["dX_lo"][0].shape == (N, 128) and r["dX_hp"][0].shape == (N, 128)
    assert r["dW_lo"][0].shape == (C, 128) and r["dW_hp"][0].shape == (C, 128)
    assert np.allclose(r["dW_hp"][0], wl.bf16_to_f32(dYb).astype(np.float64).T @ wl.bf16_to_f32(Xh).astype(np.float64))
    # dX of the outlier channels is an unbiased FP4 estimate of dY x W_hp: close to it
    exact = wl.bf16_to_f32(dYb).astype(np.float64) @ wl.bf16_to_f32(Wh).astype(np.float64)
    assert np.abs(r["dX_hp"][0] - exact).mean() < 0.35 * np.abs(exact).mean()      # 48-term sums of stochastically rounded values


def test_keeping_the_outlier_channels_in_high_precision_lowers_the_forward_error():
    """Sec. 4.2: a few channels with consistently large magnitude force large scales on their groups; taking exactly
    those channels out of the FP4 path removes most of the forward error."""
    N, D, C = 128, 1024, 64
    rng = np.random.default_rng(5)
    x = rng.standard_normal((N, D)).astype(np.float32)
    hot = np.sort(rng.choice(D, 32, replace=False))
    x[:, hot] *= 100.0
    Xb = wl.f32_to_bf16(x)
    Wb = wl.normal_bf16((C, D), 0.02, 6)
    exact = wl.bf16_to_f32(Xb).astype(np.float64) @ wl.bf16_to_f32(Wb).astype(np.float64).T
    none = np.zeros((N, 0), np.uint16), np.zeros((C, 0), np.uint16)
    for outer in (oracle.OUTER_TENSOR, oracle.OUTER_BLOCK128):
        _, _, Y_plain, _ = oracle.outctl_fwd(Xb, Wb, none[0], none[1], outer=outer)
        cold = np.sort(rng.choice(np.setdiff1d(np.arange(D), hot), 32, replace=False))
        errs = {}
        for name, cols in (("hot", hot), ("cold", cold)):
            Xl, Xh = split(Xb, cols)
            Wl, Wh = split(Wb, cols)
            if outer == oracle.OUTER_BLOCK128:      # keep D_lo a multiple of 128: move 96 more (cold) channels out
                extra = np.setdiff1d(np.arange(D), cols)[:96]
                Xl, Xh = split(Xb, np.sort(np.concatenate([cols, extra])))
                Wl, Wh = split(Wb, np.sort(np.concatenate([cols, extra])))
            _, _, Y, _ = oracle.outctl_fwd(Xl, Wl, Xh, Wh, outer=outer)
            errs[name] = np.abs(Y - exact).mean()
        plain = np.abs(Y_plain - exact).mean()
        assert errs["hot"] < 0.5 * plain and errs["hot"] < 0.5 * errs["cold"], (outer, errs, plain)
