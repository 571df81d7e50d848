"""GPU parity where rounding ties are the rule, not the exception (run with -m gpu).

Eq. 1 (Sec. 4) rounds x / s; the reading used here is round-half-to-even of the EXACT quotient.  On ordinary data
a quotient lands near k + 1/2 for about one element in 1e5, but whenever a block keeps its scale through an
operator -- an operator that halves values, a GELU derivative saturated to exactly 0, 1/2 or 1, a residual Add of
two tensors with the same scale grid -- half of the elements sit exactly on a tie or within 1e-7 of one, and a
quantizer that only knows the quotient to FP32 accuracy decides those at random.  Every quantizing kernel is run
in such a regime here and held to the same bound as everywhere else (codes within one on at most 0.1 % of the
elements); where both sides start from bit-identical FP32 values the codes must be identical.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_12422_amd as jf
from paper_2403_12422_amd import workloads
from parity import assert_codes_close, assert_scales_close

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.cpu().numpy()


def say(msg):
    print(msg, flush=True)


def _tie_field(g, rows, cols, block, scale_of_block):
    """FP32 matrix whose every block has max-abs 127 * s (s = scale_of_block(i, j), so that Eq. 1's scale is s when
    127 * s is exact) and whose elements are k * s / 2 for random integers k: half of them exact ties."""
    x = np.empty((rows, cols), np.float32)
    for i in range(rows // block):
        for j in range(cols // block):
            s = np.float32(scale_of_block(i, j))
            k = g.integers(-253, 254, size=(block, block))
            k[g.integers(block), g.integers(block)] = 254 * (1 if g.random() < 0.5 else -1)
            x[i * block:(i + 1) * block, j * block:(j + 1) * block] = (k.astype(np.float32) * np.float32(0.5)) * s
    return x


@pytest.mark.parametrize("block", [32, 64, 128])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_quantizer_exact_ties_and_neighbours(block, dtype):
    """Half-integers of the scale, and their FP32 neighbours on either side: codes must equal the oracle's."""
    say(f"quantizer ties block={block} {dtype}")
    g = workloads.rng(9000 + block)
    rows, cols = 2 * block, 3 * block
    scales = [1.0, 0.125, 1.25, 3.0, 2.0 ** -20, 1.0 + 2.0 ** -23]
    x = _tie_field(g, rows, cols, block, lambda i, j: scales[(3 * i + j) % len(scales)])
    if dtype == "f16":
        x = _tie_field(g, rows, cols, block, lambda i, j: [1.0, 0.125, 0.25][(i + j) % 3])   # k/2 * s exact in FP16
        xd = dev(x.astype(np.float16))
        assert np.array_equal(x.astype(np.float16).astype(np.float32), x)
    else:
        # nudge a third of the elements one FP32 step off the tie, up or down (never the block maximum)
        nudge = g.integers(0, 3, size=x.shape)
        amax = np.abs(x).reshape(rows // block, block, cols // block, block).max(axis=(1, 3))
        not_max = np.abs(x) < np.kron(amax, np.ones((block, block), np.float32))
        up = np.nextafter(x, np.float32(np.inf)).astype(np.float32)
        dn = np.nextafter(x, np.float32(-np.inf)).astype(np.float32)
        x = np.where((nudge == 1) & not_max, up, np.where((nudge == 2) & not_max, dn, x)).astype(np.float32)
        xd = dev(x)
    q, s = jf.jf_quantize_block(xd, block)
    oq, os_ = oracle.quantize_block(x, block)
    np.testing.assert_array_equal(host(s), os_)
    np.testing.assert_array_equal(host(q), oq)
    ties = np.mod(np.abs(x.astype(np.float64)) / np.kron(os_, np.ones((block, block))).astype(np.float64), 1.0) == 0.5
    assert ties.mean() > 0.1, "the case is meant to consist of ties and their neighbours"
    assert np.all(oq[ties] % 2 == 0), "exact ties go to the even code"


@pytest.mark.parametrize("amax", [3e-37, 1e-38, 2e-39, 1e-41, 3e-44])
def test_quantizer_tiny_blocks(amax):
    """Blocks whose scale is subnormal in FP32 or whose FP32 reciprocal would overflow."""
    block, rows, cols = 32, 64, 64
    g = workloads.rng(9100)
    x = (g.uniform(-1.0, 1.0, size=(rows, cols)) * amax).astype(np.float32)
    x[::32, ::32] = np.float32(amax)
    x[32:, 32:] = g.standard_normal((32, 32)).astype(np.float32)     # an ordinary block beside them
    say(f"quantizer tiny block amax={amax:g}")
    q, s = jf.jf_quantize_block(dev(x), block)
    oq, os_ = oracle.quantize_block(x, block)
    np.testing.assert_array_equal(host(s), os_)
    if float(np.float32(amax)) / 127.0 >= 2.0 ** -149:                # below that the scale itself rounds to zero
        np.testing.assert_array_equal(host(q), oq)
        assert np.abs(oq[:32, :32]).max() == 127


def _rank_one_operands(g, rows_a, rows_b, block):
    """Two integer vectors a (|a| <= 127, one entry of 127 per block of rows) and b (entries +-1, +-2, one entry of
    2 per block): the outer product a b^T has max-abs 254 in every block x block tile and is odd wherever b = +-1
    and a is odd."""
    a = g.integers(-127, 128, size=rows_a).astype(np.int8)
    b = g.choice(np.array([-2, -1, 1, 2], np.int8), size=rows_b)
    a[np.arange(0, rows_a, block) + g.integers(block, size=rows_a // block)] = 127
    b[np.arange(0, rows_b, block) + g.integers(block, size=rows_b // block)] = 2
    return a, b


def _assert_tie_product(name, got, want, block):
    q, s, f = (host(t) for t in got)
    oq, os_, o32, _ = want
    np.testing.assert_array_equal(f, o32, err_msg=name)
    np.testing.assert_array_equal(s, os_, err_msg=name)
    np.testing.assert_array_equal(q, oq, err_msg=name)
    quot = np.abs(o32.astype(np.float64)) / np.kron(os_, np.ones((block, block)))
    half = np.mod(quot, 1.0) == 0.5
    assert half.mean() > 0.15, name + ": the case is meant to consist of ties"
    assert np.all(oq[half] % 2 == 0), name
    say(f"  {name}: {int(half.sum())} of {half.size} accumulators are exact ties, all codes equal the oracle's")


@pytest.mark.parametrize("block", [32, 64, 128])
def test_linear_epilogue_exact_ties(block):
    """Accumulators that are exact odd multiples of half the output scale, for all three products: the operands
    are rank-one inside the first K-block (and zero in the second), the scales powers of two, so that
    acc = t a_i b_j exactly, every output block has max-abs 254 t and scale 2 t, and acc / scale = a_i b_j / 2."""
    N, C, D = 2 * block, 2 * block, 3 * block
    g = workloads.rng(9200 + block)
    say(f"linear epilogue ties block={block}")
    grid = lambda r, c, v: np.full((r // block, c // block), v, np.float32)
    k = int(g.integers(block))                                  # the one contributing position of K-block 0
    # forward  Y[n, d] = sum_c X[n, c] W[d, c]
    a, b = _rank_one_operands(g, N, D, block)
    X, W = np.zeros((N, C), np.int8), np.zeros((D, C), np.int8)
    X[:, k], W[:, k] = a, b
    SX, SW = grid(N, C, 0.25), grid(D, C, 2.0)
    _assert_tie_product("fwd", jf.jf_linear_fwd(dev(X), dev(SX), dev(W), dev(SW), block, want_f32=True),
                        oracle.linear_fwd(X, SX, W, SW, block), block)
    # dgrad  dX[n, c] = sum_d dY[n, d] W[d, c]
    N, C, D = 2 * block, 3 * block, 2 * block
    a, b = _rank_one_operands(g, N, C, block)
    dY, W = np.zeros((N, D), np.int8), np.zeros((D, C), np.int8)
    dY[:, k], W[k, :] = a, b
    SdY, SW = grid(N, D, 2.0 ** -10), grid(D, C, 0.5)
    _assert_tie_product("dgrad", jf.jf_linear_dgrad(dev(dY), dev(SdY), dev(W), dev(SW), block, want_f32=True),
                        oracle.linear_dgrad(dY, SdY, W, SW, block), block)
    # wgrad  dW[d, c] = sum_n dY[n, d] X[n, c]
    N, C, D = 2 * block, 3 * block, 2 * block
    a, b = _rank_one_operands(g, D, C, block)
    dY, X = np.zeros((N, D), np.int8), np.zeros((N, C), np.int8)
    dY[k, :], X[k, :] = a, b
    SdY, SX = grid(N, D, 2.0 ** -10), grid(N, C, 4.0)
    _assert_tie_product("wgrad", jf.jf_linear_wgrad(dev(dY), dev(SdY), dev(X), dev(SX), block, want_f32=True),
                        oracle.linear_wgrad(dY, SdY, X, SX, block), block)


def _check(name, q, s, oq, os_, of64, block, exact=False):
    assert_scales_close(host(s), os_, name + " scales")
    nbad = assert_codes_close(host(q), oq, name + " codes", prequant=of64, scales=os_, block=block)
    say(f"  {name}: {nbad} / {oq.size} codes differ by one")
    if exact:
        assert nbad == 0, name
    return nbad


@pytest.mark.parametrize("block,N,C", [(32, 128, 352), (64, 128, 192), (128, 256, 384), (32, 2048, 1536)])
def test_gelu_saturated(block, N, C):
    """Pre-activations far from zero or exactly zero: GELU'(x) is exactly 0, 1/2 or 1 and GELU(x) is 0 or x, so every
    block of the outputs keeps its input's scale and half of the gradient codes are halved."""
    say(f"gelu saturated block={block} {N}x{C}")
    g = workloads.rng(9300 + block + N)
    X = (g.choice([-127, -100, -90, 0, 0, 0, 90, 100, 127], size=(N, C))).astype(np.int8)
    X[::block, ::block] = 127
    SX = g.uniform(0.15, 0.6, size=(N // block, C // block)).astype(np.float32)      # |x| >= 13.5 or 0
    G, SG = oracle.quantize_block(workloads.gaussian(g, N, C, 1e-3), block)
    # the largest gradient of every block meets GELU' = 1, so that the block keeps its scale
    for i in range(N // block):
        for j in range(C // block):
            blk = G[i * block:(i + 1) * block, j * block:(j + 1) * block]
            r, c = np.unravel_index(np.argmax(np.abs(blk.astype(np.int16))), blk.shape)
            X[i * block + r, j * block + c] = 127
    Xd, SXd, Gd, SGd = map(dev, (X, SX, G, SG))
    Y, SY = jf.jf_gelu_q(Xd, SXd, block)
    oY, oSY, oy = oracle.gelu_q(X, SX, block)
    _check("gelu fwd (saturated)", Y, SY, oY, oSY, oy, block)
    dX, SdX = jf.jf_gelu_q_bwd(Gd, SGd, Xd, SXd, block)
    odX, oSdX, odx = oracle.gelu_q_bwd(G, SG, X, SX, block)
    np.testing.assert_array_equal(oSdX, SG)                       # the regime this test is about
    halves = (X == 0) & (G % 2 != 0)
    assert halves.mean() > 0.1
    _check("gelu bwd (saturated)", dX, SdX, odX, oSdX, odx, block)


@pytest.mark.parametrize("block,N,C", [(32, 128, 352), (64, 128, 192), (128, 256, 384), (32, 2048, 1536)])
def test_add_scale_preserving(block, N, C):
    """x + x (every code reproduces itself), and x1 + x2 on one power-of-two scale grid with block sums of 254
    (odd code sums are exact ties)."""
    say(f"add scale-preserving block={block} {N}x{C}")
    g = workloads.rng(9400 + block + N)
    x = workloads.gaussian(g, N, C, 1.0)
    workloads.with_outlier_columns(g, x, 0.01, 20.0)
    X, S = oracle.quantize_block(x, block)
    Xd, Sd = dev(X), dev(S)
    Y, SY = jf.jf_add_q(Xd, Sd, Xd, Sd, block)
    oY, oSY, _, _, of = oracle.add_q(X, S, X, S, block)
    np.testing.assert_array_equal(oY, X)
    _check("x + x", Y, SY, oY, oSY, of, block, exact=True)
    # equal power-of-two scales: sums are exact in FP32 on both sides
    X1 = g.integers(-127, 128, size=(N, C)).astype(np.int8)
    X2 = g.integers(-127, 128, size=(N, C)).astype(np.int8)
    X1[::block, ::block] = 127
    X2[::block, ::block] = 127
    S2 = np.exp2(g.integers(-12, 4, size=(N // block, C // block))).astype(np.float32)
    Y, SY, rm, rq = jf.jf_add_q(dev(X1), dev(S2), dev(X2), dev(S2), block, want_partials=True)
    oY, oSY, orm, orq, of = oracle.add_q(X1, S2, X2, S2, block)
    np.testing.assert_array_equal(oSY, 2 * S2)
    odd = (X1.astype(np.int16) + X2) % 2 != 0
    assert odd.mean() > 0.4 and np.all(oY[odd] % 2 == 0)
    _check("x1 + x2 (odd sums tie)", Y, SY, oY, oSY, of, block, exact=True)


@pytest.mark.parametrize("block,N,C,p", [(32, 128, 352, 0.5), (64, 128, 192, 0.5), (128, 256, 384, 0.75), (32, 2048, 1536, 0.5)])
def test_dropout_scale_preserving(block, N, C, p):
    """p = 1/2 (3/4): kept values double (quadruple); a block whose maximum is kept reproduces its codes."""
    say(f"dropout scale-preserving block={block} {N}x{C} p={p}")
    g = workloads.rng(9500 + block + N)
    x, _ = workloads.gelu_case(9500 + block, N, C)
    X, S = oracle.quantize_block(x, block)
    bits, keep = workloads.dropout_mask_bits(g, N, C, p)
    keep |= np.abs(X.astype(np.int16)) == 127                     # keep every block maximum
    bits = np.packbits(keep, axis=1, bitorder="little")
    Y, SY = jf.jf_dropout_q(dev(X), dev(S), dev(bits), p, block)
    oY, oSY, of = oracle.dropout_q(X, S, bits, p, block)
    np.testing.assert_array_equal(oY, np.where(keep, X, 0))
    _check("dropout", Y, SY, oY, oSY, of, block, exact=True)


def test_layer_chain_with_unit_variance_weights():
    """The chain LayerNorm -> linear -> GELU fwd/bwd -> dgrad / wgrad -> LayerNorm bwd with weights of standard
    deviation one: pre-activations of standard deviation sqrt(C), GELU' saturated almost everywhere, so the
    gradient that GELU backward hands to the two backward products keeps its scale block by block."""
    block, N, C, D = 32, 256, 256, 256
    X, W, dY = workloads.linear_layer(1, N, C, D, w_std=1.0)
    Xq, SX = oracle.quantize_block(X, block)
    Wq, SW = oracle.quantize_block(W, block)
    Gq, SG = oracle.quantize_block(dY, block)
    gamma, beta = np.ones(C, np.float32), np.zeros(C, np.float32)
    oY, oSY, omean, orstd, oy = oracle.layernorm_q(Xq, SX, gamma, beta, 1e-5, block)
    Y, SY, _, _ = jf.jf_layernorm_q(dev(Xq), dev(SX), dev(gamma), dev(beta), 1e-5, block)
    _check("layernorm fwd", Y, SY, oY, oSY, oy, block)
    oH, oSH, oH32, _ = oracle.linear_fwd(oY, oSY, Wq, SW, block)
    H, SH, Hf = jf.jf_linear_fwd(dev(oY), dev(oSY), dev(Wq), dev(SW), block, want_f32=True)
    np.testing.assert_array_equal(host(Hf), oH32)
    _check("linear fwd", H, SH, oH, oSH, oH32, block, exact=True)
    oA, oSA, oa = oracle.gelu_q(oH, oSH, block)
    A, SA = jf.jf_gelu_q(dev(oH), dev(oSH), block)
    _check("gelu fwd", A, SA, oA, oSA, oa, block)
    odH, oSdH, odh = oracle.gelu_q_bwd(Gq, SG, oH, oSH, block)
    dH, SdH = jf.jf_gelu_q_bwd(dev(Gq), dev(SG), dev(oH), dev(oSH), block)
    _check("gelu bwd", dH, SdH, odH, oSdH, odh, block)
    odX, oSdX, odX32, _ = oracle.linear_dgrad(odH, oSdH, Wq, SW, block)
    dX, SdX, dXf = jf.jf_linear_dgrad(dev(odH), dev(oSdH), dev(Wq), dev(SW), block, want_f32=True)
    np.testing.assert_array_equal(host(dXf), odX32)
    _check("linear dgrad", dX, SdX, odX, oSdX, odX32, block, exact=True)
    odW, oSdW, odW32, _ = oracle.linear_wgrad(odH, oSdH, oY, oSY, block)
    dW, SdW, dWf = jf.jf_linear_wgrad(dev(odH), dev(oSdH), dev(oY), dev(oSY), block, want_f32=True)
    np.testing.assert_array_equal(host(dWf), odW32)
    _check("linear wgrad", dW, SdW, odW, oSdW, odW32, block, exact=True)
    odXl, oSdXl, _, _, odxl = oracle.layernorm_q_bwd(odX, oSdX, Xq, SX, gamma, omean, orstd, block)
    dXl, SdXl, _, _ = jf.jf_layernorm_q_bwd(dev(odX), dev(oSdX), dev(Xq), dev(SX), dev(gamma), dev(omean), dev(orstd), block)
    _check("layernorm bwd", dXl, SdXl, odXl, oSdXl, odxl, block)
