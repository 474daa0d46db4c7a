"""Seeded synthetic inputs for the NVFP4 quantized-linear hot path.

This module holds input recipes only: random draws, planted outliers and the
float32 -> bfloat16 storage cast.  None of the quantization method's arithmetic
lives here, so both the CPU oracle's tests and the GPU path's tests / bench can
feed from it without sharing any method code.

Every tensor is returned as a C-contiguous ``numpy.uint16`` array of bfloat16
bit patterns (numpy has no bfloat16 dtype).  ``bf16_to_f32`` widens them again.

The value laws follow the workload list this build is measured on:
  * activations  X  ~ N(0, 1) with a fraction of entries multiplied by 50
  * weights      W  ~ N(0, 0.02)          (second parameter = standard deviation)
  * gradients    dY ~ N(0, 1e-3)
  * bandwidth stress: 0.1 * Student-t(nu=3)
  * large GEMM: N(0,1) with 1 % of the K-channels of the activation scaled by 100
Shapes are the linears of one transformer block of the paper's model table
(hidden 768 / MLP 3072 and hidden 1024 / MLP 8192, Appendix "model
configurations") and the square M=N=K sweep of the paper's single-linear
throughput figure.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "f32_to_bf16", "bf16_to_f32", "normal_bf16", "student_t_bf16",
    "outlier_channel_bf16", "linear_inputs", "outlier_channel_split", "CONFIGS", "config_linears",
]


def f32_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round-to-nearest-even (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(b: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(shape, std: float, seed: int, outlier_frac: float = 0.0,
                outlier_mult: float = 1.0) -> np.ndarray:
    """N(0, std) entries; a Bernoulli(outlier_frac) mask multiplies entries by outlier_mult."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
    if outlier_frac > 0.0:
        mask = rng.random(shape, dtype=np.float32) < np.float32(outlier_frac)
        x = np.where(mask, x * np.float32(outlier_mult), x)
    return f32_to_bf16(x)


def student_t_bf16(shape, nu: float, scale: float, seed: int) -> np.ndarray:
    """scale * Student-t(nu) entries (heavy tails: a stress case for the block scales)."""
    rng = np.random.default_rng(seed)
    x = rng.standard_t(nu, size=shape).astype(np.float32) * np.float32(scale)
    return f32_to_bf16(x)


def outlier_channel_bf16(rows: int, K: int, seed: int, channel_frac: float = 0.01,
                         channel_mult: float = 100.0) -> np.ndarray:
    """N(0,1) [rows x K] with round(channel_frac*K) random K-columns scaled by channel_mult."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, K), dtype=np.float32)
    n_out = int(round(channel_frac * K))
    if n_out > 0:
        cols = rng.choice(K, size=n_out, replace=False)
        x[:, cols] *= np.float32(channel_mult)
    return f32_to_bf16(x)


def linear_inputs(N: int, D: int, C: int, seed: int, kind: str = "block"):
    """One linear layer's (X[N,D], W[C,D], dY[N,C]) as bf16 bit patterns.

    kind="block": transformer-block law (X with 0.1 % x50 outliers, W std 0.02, dY std 1e-3).
    kind="square": large-GEMM law (X with 1 % outlier channels x100, W ~ N(0,1), dY ~ N(0,1)).
    """
    if kind == "block":
        X = normal_bf16((N, D), 1.0, seed * 3 + 0, outlier_frac=1e-3, outlier_mult=50.0)
        W = normal_bf16((C, D), 0.02, seed * 3 + 1)
        dY = normal_bf16((N, C), 1e-3, seed * 3 + 2)
    elif kind == "square":
        X = outlier_channel_bf16(N, D, seed * 3 + 0)
        W = normal_bf16((C, D), 1.0, seed * 3 + 1)
        dY = normal_bf16((N, C), 1.0, seed * 3 + 2)
    else:
        raise ValueError(kind)
    return X, W, dY


def outlier_channel_split(X: np.ndarray, W: np.ndarray, n_hp: int):
    """The static channel split of the outlier-control layer: the n_hp input channels with the largest activation
    l2-norm go to the high-precision set, the rest stay; both tensors are split the same way, column order kept.
    Returns (X_lo, W_lo, X_hp, W_hp, hp_columns) as C-contiguous bf16 bit arrays."""
    norms = (bf16_to_f32(X).astype(np.float64) ** 2).sum(axis=0)
    hp = np.sort(np.argsort(-norms, kind="stable")[:n_hp])
    lo = np.setdiff1d(np.arange(X.shape[1]), hp)
    c = np.ascontiguousarray
    return c(X[:, lo]), c(W[:, lo]), c(X[:, hp]), c(W[:, hp]), hp


# name -> dict(tokens, linears=[(name, D_in, C_out)], kind, seed)
CONFIGS = {
    "cfg1_single": dict(tokens=256, linears=[("lin", 512, 512)], kind="block", seed=0),
    "cfg2_block768": dict(tokens=8192, kind="block", seed=200,
                          linears=[("qkv", 768, 2304), ("o", 768, 768),
                                   ("up", 768, 3072), ("down", 3072, 768)]),
    "cfg3_block1024": dict(tokens=16384, kind="block", seed=300,
                           linears=[("qkv", 1024, 3072), ("o", 1024, 1024),
                                    ("gate_up", 1024, 8192), ("down", 4096, 1024)]),
    "cfg4_quant_stress": dict(rows=8192, cols=8192, nu=3.0, scale=0.1, seed=7),
    "cfg5_square8192": dict(tokens=8192, kind="square", seed=500,
                            linears=[("sq", 8192, 8192)]),
}


def config_linears(name: str):
    """[(layer_name, N, D, C, seed, kind)] for a linear-layer config."""
    cfg = CONFIGS[name]
    out = []
    for i, (lname, D, C) in enumerate(cfg["linears"]):
        out.append((lname, cfg["tokens"], D, C, cfg["seed"] + i, cfg["kind"]))
    return out


def config_flops(name: str) -> float:
    """Algorithmic flops of fwd + dX + dW over all linears of a config: 3 * sum 2*N*D*C."""
    return float(sum(3 * 2 * N * D * C for (_, N, D, C, _, _) in config_linears(name)))
