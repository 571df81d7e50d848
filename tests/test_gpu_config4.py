"""GPU parity on the GPT-2-large-shaped transformer block (hidden 1280, 20 heads, FFN 5120, 8 x 1024 tokens, block 32):
forward and backward with the INT8 data flow between the layers.

The oracle walks the whole chain; at every operator the GPU entry point is run on the ORACLE's inputs and its
output is compared with the oracle's, so errors do not compound.  Multi-head attention stays in floating point
(Sec. 7.1): it is evaluated once, on the CPU with stock torch ops in float32 from the FP16 hand-over tensor, and
its result feeds both sides; the INT8 <-> FP16 hand-over on either side of it is part of the checked path.
No bias, no dropout.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_12422_amd as jf
from paper_2403_12422_amd import workloads
from parity import assert_layernorm_param_grads_close
from test_gpu_parity import _check_eltwise, _check_linear, dev, host, say

pytestmark = pytest.mark.gpu
B = 32


def _attention(qkv16, batch, seq, heads, grad16=None):
    """Causal multi-head attention on the CPU (float32 arithmetic on FP16 inputs); returns the FP16 output and,
    if the upstream gradient is given, the FP16 gradient with respect to qkv."""
    N, H3 = qkv16.shape
    H = H3 // 3
    t = torch.from_numpy(qkv16.astype(np.float32)).requires_grad_(grad16 is not None)
    q, k, v = (t[:, i * H:(i + 1) * H].reshape(batch, seq, heads, H // heads).transpose(1, 2) for i in range(3))
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    o = o.transpose(1, 2).reshape(N, H)
    if grad16 is None:
        return o.detach().numpy().astype(np.float16), None
    o.backward(torch.from_numpy(grad16.astype(np.float32)))
    return o.detach().numpy().astype(np.float16), t.grad.numpy().astype(np.float16)


def _check_quantize(name, x16, want):
    q, s = jf.jf_quantize_block(dev(x16), B)
    oq, os_ = want
    np.testing.assert_array_equal(host(s), os_, err_msg=name)
    np.testing.assert_array_equal(host(q), oq, err_msg=name)   # same values and scale in, exact rounding: same codes


def _check_dequantize(name, q, s):
    got = host(jf.jf_dequantize_block(dev(q), dev(s), B, torch.float16))
    want = oracle.dequantize(q, s, B).astype(np.float16)
    bad = got != want
    # the kernel rounds the FP32 product, the oracle the exact one: they can differ by one FP16 step at a tie
    assert np.count_nonzero(bad) <= 1e-3 * bad.size, name
    assert np.all(np.abs(got[bad].astype(np.float64) - want[bad].astype(np.float64)) <= np.spacing(np.abs(want[bad])).astype(np.float64)), name
    got32 = host(jf.jf_dequantize_block(dev(q), dev(s), B, torch.float32))
    np.testing.assert_array_equal(got32, oracle.dequantize(q, s, B).astype(np.float32), err_msg=name)
    return want


def test_config4_transformer_block_forward_backward():
    batch, seq, H, heads, F = 8, 1024, 1280, 20, 5120
    N = batch * seq
    g = workloads.rng(4004)
    x = workloads.gaussian(g, N, H, 1.0)
    workloads.with_outlier_columns(g, x, 13.0 / H, 20.0)
    Wqkv, Wo, W1, W2 = (workloads.gaussian(g, r, c, 0.02) for r, c in ((3 * H, H), (H, H), (F, H), (H, F)))
    vec = lambda m, sd: (m + sd * g.standard_normal(H, dtype=np.float32)).astype(np.float32)
    g1, b1, g2, b2 = vec(1.0, 0.1), vec(0.0, 0.1), vec(1.0, 0.1), vec(0.0, 0.1)
    dout = workloads.gaussian(g, N, H, 1e-3)
    eps = 1e-5
    Q = lambda a: oracle.quantize_block(a, B)
    (X, SX), (Wq, SWq), (Wo_, SWo), (W1_, SW1), (W2_, SW2), (dY, SdY) = (Q(a) for a in (x, Wqkv, Wo, W1, W2, dout))
    d = lambda *a: [dev(t) for t in a]

    def linear(name, which, a, sa, w, sw):
        fn_g = (jf.jf_linear_fwd, jf.jf_linear_dgrad, jf.jf_linear_wgrad)[which]
        fn_o = (oracle.linear_fwd, oracle.linear_dgrad, oracle.linear_wgrad)[which]
        want = fn_o(a, sa, w, sw, B)
        _check_linear(name, fn_g(*d(a, sa, w, sw), B, want_f32=True), want, B)
        return want[0], want[1]

    def eltwise(name, got, want):
        _check_eltwise(name, got[0], got[1], want[0], want[1], want[-1], B)

    def param_grads(name, got, dgamma, dbeta, gq, sg, xq, sx, mean, rstd):
        xh = (oracle.dequantize(xq, sx, B) - mean[:, None].astype(np.float64)) * rstd[:, None].astype(np.float64)
        assert_layernorm_param_grads_close(host(got[2]), host(got[3]), dgamma, dbeta, oracle.dequantize(gq, sg, B), xh, name)

    # ---------------------------------------------------------------- forward
    say("config 4 forward")
    A1, SA1, mean1, rstd1, f = oracle.layernorm_q(X, SX, g1, b1, eps, B)
    eltwise("ln1", jf.jf_layernorm_q(*d(X, SX, g1, b1), eps, B), (A1, SA1, f))
    QKV, SQKV = linear("qkv", 0, A1, SA1, Wq, SWq)
    qkv16 = _check_dequantize("qkv -> fp16", QKV, SQKV)
    say("  attention (CPU, float32 on FP16 inputs)")
    att16, _ = _attention(qkv16, batch, seq, heads)
    AT, SAT = Q(att16.astype(np.float32))
    _check_quantize("attention -> int8", att16, (AT, SAT))
    P, SP = linear("out-proj", 0, AT, SAT, Wo_, SWo)
    R1, SR1, rm, rq, f = oracle.add_q(X, SX, P, SP, B)
    got = jf.jf_add_q(*d(X, SX, P, SP), B, want_partials=True)
    eltwise("residual add 1", got, (R1, SR1, f))
    np.testing.assert_allclose(host(got[2]).T, rm, rtol=0, atol=1e-5 * np.abs(f).max())     # stored (C / block, N)
    np.testing.assert_allclose(host(got[3]).T, rq, rtol=1e-5)
    mean2, rstd2 = oracle.row_stats_from_partials(rm, rq, H, eps, B)
    A2, SA2, f = oracle.layernorm_q_stats(R1, SR1, g2, b2, mean2, rstd2, B)
    got = jf.jf_layernorm_q_partials(*d(R1, SR1, rm.T, rq.T, g2, b2), eps, B)
    eltwise("ln2 from partials", got, (A2, SA2, f))
    np.testing.assert_allclose(host(got[3]), rstd2, rtol=1e-5)
    H1, SH1 = linear("fc1", 0, A2, SA2, W1_, SW1)
    GE, SGE, f = oracle.gelu_q(H1, SH1, B)
    eltwise("gelu", jf.jf_gelu_q(*d(H1, SH1), B), (GE, SGE, f))
    H2, SH2 = linear("fc2", 0, GE, SGE, W2_, SW2)
    OUT, SOUT, _, _, f = oracle.add_q(R1, SR1, H2, SH2, B)
    eltwise("residual add 2", jf.jf_add_q(*d(R1, SR1, H2, SH2), B), (OUT, SOUT, f))

    # ---------------------------------------------------------------- backward
    say("config 4 backward")
    dGE, SdGE = linear("fc2 dgrad", 1, dY, SdY, W2_, SW2)
    linear("fc2 wgrad", 2, dY, SdY, GE, SGE)
    dH1, SdH1, f = oracle.gelu_q_bwd(dGE, SdGE, H1, SH1, B)
    eltwise("gelu bwd", jf.jf_gelu_q_bwd(*d(dGE, SdGE, H1, SH1), B), (dH1, SdH1, f))
    dA2, SdA2 = linear("fc1 dgrad", 1, dH1, SdH1, W1_, SW1)
    linear("fc1 wgrad", 2, dH1, SdH1, A2, SA2)
    dR1a, SdR1a, dg2, db2, f = oracle.layernorm_q_bwd(dA2, SdA2, R1, SR1, g2, mean2, rstd2, B)
    got = jf.jf_layernorm_q_bwd(*d(dA2, SdA2, R1, SR1, g2, mean2, rstd2), B)
    eltwise("ln2 bwd", got, (dR1a, SdR1a, f))
    param_grads("ln2 bwd", got, dg2, db2, dA2, SdA2, R1, SR1, mean2, rstd2)
    dR1, SdR1, _, _, f = oracle.add_q(dY, SdY, dR1a, SdR1a, B)
    eltwise("residual add 2 bwd", jf.jf_add_q(*d(dY, SdY, dR1a, SdR1a), B), (dR1, SdR1, f))
    dAT, SdAT = linear("out-proj dgrad", 1, dR1, SdR1, Wo_, SWo)
    linear("out-proj wgrad", 2, dR1, SdR1, AT, SAT)
    dat16 = _check_dequantize("d(attention) -> fp16", dAT, SdAT)
    say("  attention backward (CPU)")
    _, dqkv16 = _attention(qkv16, batch, seq, heads, dat16)
    dQKV, SdQKV = Q(dqkv16.astype(np.float32))
    _check_quantize("d(qkv) -> int8", dqkv16, (dQKV, SdQKV))
    dA1, SdA1 = linear("qkv dgrad", 1, dQKV, SdQKV, Wq, SWq)
    linear("qkv wgrad", 2, dQKV, SdQKV, A1, SA1)
    dXa, SdXa, dg1, db1, f = oracle.layernorm_q_bwd(dA1, SdA1, X, SX, g1, mean1, rstd1, B)
    got = jf.jf_layernorm_q_bwd(*d(dA1, SdA1, X, SX, g1, mean1, rstd1), B)
    eltwise("ln1 bwd", got, (dXa, SdXa, f))
    param_grads("ln1 bwd", got, dg1, db1, dA1, SdA1, X, SX, mean1, rstd1)
    dX, SdX, _, _, f = oracle.add_q(dR1, SdR1, dXa, SdXa, B)
    eltwise("residual add 1 bwd", jf.jf_add_q(*d(dR1, SdR1, dXa, SdXa), B), (dX, SdX, f))
