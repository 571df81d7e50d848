"""GPU parity on seeded random shapes (every entry point, every block size), and replay of the whole hot path from
a captured HIP graph."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_12422_amd as jf
from paper_2403_12422_amd import workloads
from parity import assert_layernorm_param_grads_close
from test_gpu_parity import _check_eltwise, _check_linear, dev, host, say

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", range(12))
def test_random_shapes_every_operator(case):
    g = workloads.rng(9000 + case)
    block = (32, 64, 128)[case % 3]
    N, C, D = (int(block * g.integers(1, 1 + 640 // block)) for _ in range(3))
    if C % 8:
        C += block                                              # the dropout mask packs 8 columns per byte
    say(f"random shape case {case}: block={block} N={N} C={C} D={D}")
    X, W, dY = workloads.linear_layer(9100 + case, N, C, D, w_std=0.5, grad_std=1e-2, outlier_fraction=0.02)
    (X, SX), (W, SW), (dY, SdY) = (oracle.quantize_block(a, block) for a in (X, W, dY))
    Xd, SXd, Wd, SWd, dYd, SdYd = map(dev, (X, SX, W, SW, dY, SdY))
    _check_linear("fwd", jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True), oracle.linear_fwd(X, SX, W, SW, block), block)
    _check_linear("dgrad", jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block, want_f32=True), oracle.linear_dgrad(dY, SdY, W, SW, block), block)
    _check_linear("wgrad", jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_f32=True), oracle.linear_wgrad(dY, SdY, X, SX, block), block)
    # element-wise operators on the (N, C) tensor and a second tensor of the same shape
    x2 = workloads.gaussian(g, N, C, 0.7)
    X2, SX2 = oracle.quantize_block(x2, block)
    gamma = (1.0 + 0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)
    beta = (0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)
    X2d, SX2d, gd, bd = map(dev, (X2, SX2, gamma, beta))
    o = oracle.gelu_q(X, SX, block)
    _check_eltwise("gelu", *jf.jf_gelu_q(Xd, SXd, block), o[0], o[1], o[2], block)
    o = oracle.gelu_q_bwd(X2, SX2, X, SX, block)
    _check_eltwise("gelu bwd", *jf.jf_gelu_q_bwd(X2d, SX2d, Xd, SXd, block), o[0], o[1], o[2], block)
    o = oracle.add_q(X, SX, X2, SX2, block)
    _check_eltwise("add", *jf.jf_add_q(Xd, SXd, X2d, SX2d, block), o[0], o[1], o[4], block)
    bits, _ = workloads.dropout_mask_bits(g, N, C, 0.2)
    o = oracle.dropout_q(X, SX, bits, 0.2, block)
    _check_eltwise("dropout", *jf.jf_dropout_q(Xd, SXd, dev(bits), 0.2, block), o[0], o[1], o[2], block)
    oY, oSY, omean, orstd, of = oracle.layernorm_q(X, SX, gamma, beta, 1e-5, block)
    Y, SY, mean, rstd = jf.jf_layernorm_q(Xd, SXd, gd, bd, 1e-5, block)
    _check_eltwise("layernorm", Y, SY, oY, oSY, of, block)
    np.testing.assert_allclose(host(rstd), orstd, rtol=1e-5)
    o = oracle.layernorm_q_bwd(X2, SX2, X, SX, gamma, omean, orstd, block)
    got = jf.jf_layernorm_q_bwd(X2d, SX2d, Xd, SXd, gd, dev(omean), dev(orstd), block)
    _check_eltwise("layernorm bwd", got[0], got[1], o[0], o[1], o[4], block)
    xh = (oracle.dequantize(X, SX, block) - omean[:, None].astype(np.float64)) * orstd[:, None].astype(np.float64)
    assert_layernorm_param_grads_close(host(got[2]), host(got[3]), o[2], o[3], oracle.dequantize(X2, SX2, block), xh, "layernorm bwd")
    np.testing.assert_array_equal(host(jf.jf_dequantize_block(Xd, SXd, block)), oracle.dequantize(X, SX, block).astype(np.float32))


def _bands(rows, block, unit):
    """Row ranges at the top, around row group 65535 (where a grid's y dimension would end) and at the bottom;
    unit = rows per workgroup of the kernel under test."""
    edge = 65535 * unit
    return [(0, 2 * block), (edge - 2 * block, edge + 2 * block), (rows - 2 * block, rows)]


@pytest.mark.parametrize("block", [32, 128])
def test_more_row_groups_than_a_grid_dimension_holds(block):
    """Tall tensors: more row groups than the 65535 a grid's y or z dimension can hold (the kernels number their
    workgroups along x).  The tensors are drawn on the GPU; bands of whole block rows -- the operators work block
    by block -- are checked against the oracle."""
    say(f"tall tensors, block {block}")
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(240312422 + block)
    rnd = lambda shape, sd: torch.randn(shape, generator=gen, device="cuda:0", dtype=torch.float32) * sd

    # quantizer: workgroups of 128 rows
    rows, cols = 128 * 65536 + 256, block
    x = rnd((rows, cols), 1.0)
    q, s = jf.jf_quantize_block(x, block)
    for r0, r1 in _bands(rows, block, 128):
        oq, os_ = oracle.quantize_block(host(x[r0:r1]), block)
        np.testing.assert_array_equal(host(q[r0:r1]), oq)
        np.testing.assert_array_equal(host(s[r0 // block:r1 // block]), os_)
    np.testing.assert_array_equal(host(jf.jf_dequantize_block(q, s, block)[rows - block:]),
                                  oracle.dequantize(host(q[rows - block:]), host(s[-1:]), block).astype(np.float32))
    del x, q, s

    # element-wise operators: workgroups of `block` rows
    rows, cols = block * 65536 + 2 * block, 2 * block
    codes = lambda: torch.randint(-127, 128, (rows, cols), generator=gen, device="cuda:0", dtype=torch.int8)
    scales = lambda sd: (torch.rand((rows // block, cols // block), generator=gen, device="cuda:0") + 0.5) * sd
    X, SX, G, SG = codes(), scales(0.02), codes(), scales(1e-5)
    bits = torch.randint(0, 256, (rows, cols // 8), generator=gen, device="cuda:0", dtype=torch.uint8)
    gamma, beta = 1.0 + rnd((cols,), 0.1), rnd((cols,), 0.1)
    got = {"gelu": jf.jf_gelu_q(X, SX, block), "gelu bwd": jf.jf_gelu_q_bwd(G, SG, X, SX, block),
           "add": jf.jf_add_q(X, SX, G, SG, block)[:2], "dropout": jf.jf_dropout_q(X, SX, bits, 0.25, block)}
    ln = jf.jf_layernorm_q(X, SX, gamma, beta, 1e-5, block)
    for r0, r1 in _bands(rows, block, block):
        b0, b1 = r0 // block, r1 // block
        Xh, SXh, Gh, SGh = host(X[r0:r1]), host(SX[b0:b1]), host(G[r0:r1]), host(SG[b0:b1])
        want = {"gelu": oracle.gelu_q(Xh, SXh, block), "gelu bwd": oracle.gelu_q_bwd(Gh, SGh, Xh, SXh, block),
                "dropout": oracle.dropout_q(Xh, SXh, host(bits[r0:r1]), 0.25, block)}
        o = oracle.add_q(Xh, SXh, Gh, SGh, block)
        want["add"] = (o[0], o[1], o[4])
        for name, (oq, os_, of) in want.items():
            _check_eltwise(f"{name} rows {r0}..{r1}", got[name][0][r0:r1], got[name][1][b0:b1], oq, os_, of, block)
        oY, oSY, omean, orstd, of = oracle.layernorm_q(Xh, SXh, host(gamma), host(beta), 1e-5, block)
        _check_eltwise(f"layernorm rows {r0}..{r1}", ln[0][r0:r1], ln[1][b0:b1], oY, oSY, of, block)
        np.testing.assert_allclose(host(ln[3][r0:r1]), orstd, rtol=1e-5)


def test_hot_path_replayed_from_a_hip_graph():
    """The whole step (quantize, LayerNorm, the three products, GELU forward / backward, LayerNorm backward) captured
    once and replayed: every replay must reproduce the eager results bit for bit, with eager work and
    synchronisations between the replays (the library records no memset nodes and allocates nothing)."""
    block, N, C, D = 32, 512, 256, 384
    Xh, Wh, dHh = workloads.linear_layer(77, N, C, D)
    g = workloads.rng(78)
    gamma = dev((1.0 + 0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32))
    beta = dev((0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32))
    X, W, dH = map(dev, (Xh, Wh, dHh))
    i8 = lambda r, c: torch.empty((r, c), dtype=torch.int8, device=X.device)
    sc = lambda r, c: torch.empty((r // block, c // block), dtype=torch.float32, device=X.device)
    f32 = lambda n: torch.empty((n,), dtype=torch.float32, device=X.device)
    bufs = dict(Xq=i8(N, C), SX=sc(N, C), Wq=i8(D, C), SW=sc(D, C), Gq=i8(N, D), SG=sc(N, D), Xn=i8(N, C), SXn=sc(N, C),
                mean=f32(N), rstd=f32(N), Y=i8(N, D), SY=sc(N, D), H=i8(N, D), SH=sc(N, D), dY=i8(N, D), SdY=sc(N, D),
                dXn=i8(N, C), SdXn=sc(N, C), dW=i8(D, C), SdW=sc(D, C), dX=i8(N, C), SdX=sc(N, C), dg=f32(C), db=f32(C))
    ws = torch.empty((max(16, jf.jf_workspace_bytes(7, N, C, 0, block)),), dtype=torch.uint8, device=X.device)
    b = bufs

    def step():
        jf.jf_quantize_block(X, block, out=(b["Xq"], b["SX"]))
        jf.jf_quantize_block(W, block, out=(b["Wq"], b["SW"]))
        jf.jf_quantize_block(dH, block, out=(b["Gq"], b["SG"]))
        jf.jf_layernorm_q(b["Xq"], b["SX"], gamma, beta, 1e-5, block, out=(b["Xn"], b["SXn"], b["mean"], b["rstd"]))
        jf.jf_linear_fwd(b["Xn"], b["SXn"], b["Wq"], b["SW"], block, out=(b["Y"], b["SY"], None))
        jf.jf_gelu_q(b["Y"], b["SY"], block, out=(b["H"], b["SH"]))
        jf.jf_gelu_q_bwd(b["Gq"], b["SG"], b["Y"], b["SY"], block, out=(b["dY"], b["SdY"]))
        jf.jf_linear_dgrad(b["dY"], b["SdY"], b["Wq"], b["SW"], block, out=(b["dXn"], b["SdXn"], None))
        jf.jf_linear_wgrad(b["dY"], b["SdY"], b["Xn"], b["SXn"], block, out=(b["dW"], b["SdW"], None))
        jf.jf_layernorm_q_bwd(b["dXn"], b["SdXn"], b["Xq"], b["SX"], gamma, b["mean"], b["rstd"], block, workspace=ws,
                              out=(b["dX"], b["SdX"], b["dg"], b["db"]))

    step()
    torch.cuda.synchronize()
    eager = {k: v.clone() for k, v in bufs.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(4):
        for v in bufs.values():
            v.zero_()                                           # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, v in bufs.items():
            assert torch.equal(v, eager[k]), f"replay {replay}: {k} differs from the eager result"
