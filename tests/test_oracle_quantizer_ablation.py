"""Quantization error of the scale shapes of Sec. 4 on synthetic tensors with the outlier structure the paper
describes (Sec. 4: channel-wise outliers in activations, token-wise outliers in gradients), the synthetic stand-in
for the ablation of Sec. 7.3 ("Quantization Error").  CPU only; the real activations of the paper's GPT-2 runs
are not available here."""
import numpy as np

import oracle
from oracle import variants
from paper_2403_12422_amd import workloads


def _mse(x, xq):
    return float(np.mean((np.asarray(x, np.float64) - xq) ** 2))


def _errors(x, block=32):
    q, s = oracle.quantize_block(x, block)
    return {"per-tensor": _mse(x, variants.per_tensor(x)), "per-token": _mse(x, variants.per_token(x)),
            "per-channel": _mse(x, variants.per_channel(x)), "per-block": _mse(x, oracle.dequantize(q, s, block))}


def test_variants_reduce_to_each_other_on_special_shapes():
    g = workloads.rng(900)
    x = workloads.gaussian(g, 64, 96, 1.0)
    # one row: per-token == per-tensor; one column: per-channel == per-tensor; block = whole matrix: per-block == per-tensor
    np.testing.assert_array_equal(variants.per_token(x[:1]), variants.per_tensor(x[:1]))
    np.testing.assert_array_equal(variants.per_channel(x[:, :1]), variants.per_tensor(x[:, :1]))
    sq = x[:64, :64]
    q, s = oracle.quantize_block(sq, 64)
    np.testing.assert_array_equal(oracle.dequantize(q, s, 64), variants.per_tensor(sq))
    # every variant obeys the half-step bound of its own scale
    for f, ax in ((variants.per_token, 1), (variants.per_channel, 0)):
        step = np.abs(x).max(axis=ax, keepdims=True).astype(np.float64) / 127
        assert np.all(np.abs(x - f(x)) <= 0.5 * step * (1 + 1e-6))


def test_channel_outliers_activation():
    """Activations with 1 % outlier channels x20: per-token shares each row's scale with the outliers and is far
    worse than per-channel; per-block confines an outlier channel to its block column (Sec. 4, Sec. 7.3)."""
    g = workloads.rng(901)
    x = workloads.gaussian(g, 1024, 768, 1.0)
    workloads.with_outlier_columns(g, x, 0.01, 20.0)
    e = _errors(x)
    print("channel outliers:", {k: f"{v:.3e}" for k, v in e.items()})
    assert e["per-channel"] < e["per-token"] / 10
    # "lower quantization error than per-token": 8 outlier channels contaminate 8 of the 24 block columns, so the
    # error drops to about a third of per-token's plus the clean blocks' share
    assert e["per-block"] < 0.6 * e["per-token"]
    assert e["per-token"] <= e["per-tensor"] * 1.05


def test_token_outliers_gradient():
    """Gradients with 1 % outlier tokens x20 (Sec. 4): the mirror image -- per-channel is the bad shape, per-block
    again stays close to the good one."""
    g = workloads.rng(902)
    x = workloads.gaussian(g, 1024, 768, 1e-3)
    rows = g.choice(1024, size=10, replace=False)
    x[rows, :] *= np.float32(20.0)
    e = _errors(x)
    print("token outliers:", {k: f"{v:.3e}" for k, v in e.items()})
    assert e["per-token"] < e["per-channel"] / 10
    assert e["per-block"] < 0.6 * e["per-channel"]


def test_block_size_trades_error_for_scale_storage():
    g = workloads.rng(903)
    x = workloads.gaussian(g, 512, 512, 1.0)
    workloads.with_outlier_columns(g, x, 0.01, 20.0)
    errs = []
    for block in (32, 64, 128):
        q, s = oracle.quantize_block(x, block)
        errs.append(_mse(x, oracle.dequantize(q, s, block)))
    assert errs[0] < errs[1] < errs[2]
