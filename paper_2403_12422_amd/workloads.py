"""Seeded synthetic inputs shaped like the paper's workloads (Sec. 7; transformer linear layers, GELU, LayerNorm).

This module only draws random numbers: it contains none of the method's
arithmetic, and it is the one module that both the GPU tests and the CPU oracle
tests import.  Channel-wise outliers (Sec. 4, Fig. 2a) are modelled by scaling a
fixed fraction of columns by a constant factor.
"""
import numpy as np

BASE_SEED = 240312422


def rng(seed_offset=0):
    return np.random.Generator(np.random.PCG64(BASE_SEED + int(seed_offset)))


def gaussian(g, rows, cols, std=1.0, mean=0.0):
    return (g.standard_normal((rows, cols), dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(np.float32)


def with_outlier_columns(g, x, fraction, factor):
    """Scale max(1, round(fraction * cols)) distinct random columns of x by `factor` (in place); returns the columns."""
    cols = x.shape[1]
    n_out = max(1, int(round(fraction * cols)))
    idx = np.sort(g.choice(cols, size=n_out, replace=False))
    x[:, idx] *= np.float32(factor)
    return idx


def linear_layer(seed_offset, N, C, D, act_std=1.0, w_std=0.02, grad_std=1e-3, outlier_fraction=0.01,
                 outlier_factor=20.0):
    """FP32 activation X (N,C) with outlier channels, weight W (D,C), upstream gradient dY (N,D)."""
    g = rng(seed_offset)
    X = gaussian(g, N, C, act_std)
    with_outlier_columns(g, X, outlier_fraction, outlier_factor)
    W = gaussian(g, D, C, w_std)
    dY = gaussian(g, N, D, grad_std)
    return X, W, dY


def gelu_case(seed_offset, N, C, std=2.0, grad_std=1e-3):
    g = rng(seed_offset)
    return gaussian(g, N, C, std), gaussian(g, N, C, grad_std)


def layernorm_case(seed_offset, N, C, outlier_fraction=0.01, outlier_factor=20.0, grad_std=1e-3):
    g = rng(seed_offset)
    X = gaussian(g, N, C, 1.0)
    with_outlier_columns(g, X, outlier_fraction, outlier_factor)
    gamma = (1.0 + 0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)
    beta = (0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)
    dY = gaussian(g, N, C, grad_std)
    return X, gamma, beta, dY


def dropout_mask_bits(g, N, C, p):
    """Keep-mask of a dropout layer with drop probability p, packed 8 columns per byte (column c of a row is bit
    c % 8 of byte c // 8).  Returns (bits (N, C/8) uint8, mask (N, C) bool)."""
    keep = g.random((N, C), dtype=np.float32) >= np.float32(p)
    return np.packbits(keep, axis=1, bitorder="little"), keep


# The five benchmark configurations (shapes only; see the design notes for the value recipe).
CONFIGS = {
    "cfg1_single_fwd": dict(N=256, C=256, D=256, block=32, act_std=1.0, w_std=1.0),
    "cfg2_gpt2s_mlp": dict(N=4096, C=768, D=3072, block=32, act_std=1.0, w_std=0.02, grad_std=1e-3),
    "cfg3_gelu": dict(N=4096, C=3072, block=32),
    "cfg3_layernorm": dict(N=4096, C=768, block=32),
    "cfg4_gpt2l_block": dict(N=8192, hidden=1280, heads=20, ffn=5120, block=32),
}
