"""GPU parity: every C-ABI entry point against the CPU oracle on the same seeded inputs (run with -m gpu).

The GEMM / element-wise parity runs feed the ORACLE's INT8 operands to both sides so that errors do not compound;
the quantizer's own parity is checked first.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_12422_amd as jf
from paper_2403_12422_amd import workloads
from parity import (assert_codes_close, assert_f32_close, assert_layernorm_param_grads_close, assert_scales_close, block_amax,
                    expand)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host(t):
    return t.cpu().numpy()


def say(msg):
    print(msg, flush=True)


# --------------------------------------------------------------------------- quantizer
@pytest.mark.parametrize("block,rows,cols", [(32, 160, 352), (32, 256, 256), (64, 192, 320), (128, 256, 384), (32, 32, 32)])
@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_quantize_block(block, rows, cols, dtype):
    say(f"quantize block={block} {rows}x{cols} {dtype}")
    g = workloads.rng(1000 + block + rows)
    x = workloads.gaussian(g, rows, cols, 1.0)
    workloads.with_outlier_columns(g, x, 0.01, 20.0)
    x[:block, :block] = 0.0                                   # an all-zero block
    x[block // 2, cols - 3] = 5000.0                          # a single outlier
    if dtype == "f16":
        x = x.astype(np.float16).astype(np.float32)           # the oracle sees exactly what the kernel reads
        xd = dev(x.astype(np.float16))
    else:
        xd = dev(x)
    q, s, qT, sT = jf.jf_quantize_block(xd, block, transposed_copy=True)
    torch.cuda.synchronize()
    oq, os_ = oracle.quantize_block(x, block)
    np.testing.assert_array_equal(host(s), os_)               # amax and its FP32 division are exact on both sides
    np.testing.assert_array_equal(host(q), oq)                # same FP32 values and scale in, exact rounding: same codes
    np.testing.assert_array_equal(host(qT), host(q).T)
    np.testing.assert_array_equal(host(sT), os_.T)
    q2, s2 = jf.jf_quantize_block(xd, block)
    np.testing.assert_array_equal(host(q2), host(q))
    np.testing.assert_array_equal(host(s2), os_)


# --------------------------------------------------------------------------- INT32 partial sums
def _rand_codes(g, rows, cols):
    return g.integers(-127, 128, size=(rows, cols)).astype(np.int8)


@pytest.mark.parametrize("block,N,C,D", [(32, 256, 256, 256), (32, 160, 96, 224), (64, 192, 128, 320), (128, 256, 128, 384)])
def test_int32_partials_bit_exact(block, N, C, D):
    say(f"partials block={block} N={N} C={C} D={D}")
    g = workloads.rng(2000 + block + N)
    X, W, dY = _rand_codes(g, N, C), _rand_codes(g, D, C), _rand_codes(g, N, D)
    X[:32, :32] = 127                                          # extreme sums +-B*127^2
    W[:32, :32] = -127
    Xd, Wd, dYd = dev(X), dev(W), dev(dY)
    for kb in range(C // block):
        got = host(jf.jf_debug_linear_partials(0, Xd, Wd, N, C, D, block, kb))
        np.testing.assert_array_equal(got, oracle.block_partials(X, W, block, kb))
    WT, XT, dYT = np.ascontiguousarray(W.T), np.ascontiguousarray(X.T), np.ascontiguousarray(dY.T)
    for kb in range(D // block):
        got = host(jf.jf_debug_linear_partials(1, dYd, Wd, N, C, D, block, kb))
        np.testing.assert_array_equal(got, oracle.block_partials(dY, WT, block, kb))
    for kb in range(N // block):
        got = host(jf.jf_debug_linear_partials(2, dYd, Xd, N, C, D, block, kb))
        np.testing.assert_array_equal(got, oracle.block_partials(dYT, XT, block, kb))


# --------------------------------------------------------------------------- linear layer
def _quantized_layer(seed, N, C, D, block, **kw):
    X, W, dY = workloads.linear_layer(seed, N, C, D, **kw)
    return oracle.quantize_block(X, block), oracle.quantize_block(W, block), oracle.quantize_block(dY, block)


def _check_linear(name, got, want, block):
    q, s, f = got
    oq, os_, o32, o64 = want
    f = host(f)
    assert_f32_close(f, o64, block, name + " f32 vs float64 oracle")
    exact = float(np.mean(f == o32))
    say(f"  {name}: FP32 accumulator bit-identical to the oracle's FP32 accumulator on {100 * exact:.4f}% of elements")
    assert exact == 1.0, name                                   # same fma order => same bits
    assert_scales_close(host(s), os_, name + " scales")
    # the FP32 accumulators are bit-identical and Eq. 1 rounds the exact quotient on both sides: identical codes
    np.testing.assert_array_equal(host(q), oq, err_msg=name + " codes")


@pytest.mark.parametrize("block,N,C,D,kw", [
    (32, 256, 256, 256, dict(w_std=1.0)),                       # config 1
    (32, 160, 96, 224, {}),                                     # ragged against the 64/128 tiles, odd K steps
    (32, 384, 160, 128, {}),
    (64, 192, 128, 320, {}),
    (128, 256, 128, 384, {}),
    (128, 128, 384, 128, {}),
])
def test_linear_three_products(block, N, C, D, kw):
    say(f"linear block={block} N={N} C={C} D={D}")
    (X, SX), (W, SW), (dY, SdY) = _quantized_layer(3000 + block + N, N, C, D, block, **kw)
    Xd, SXd, Wd, SWd, dYd, SdYd = map(dev, (X, SX, W, SW, dY, SdY))
    _check_linear("fwd", jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True), oracle.linear_fwd(X, SX, W, SW, block), block)
    _check_linear("dgrad", jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block, want_f32=True), oracle.linear_dgrad(dY, SdY, W, SW, block), block)
    _check_linear("wgrad", jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_f32=True), oracle.linear_wgrad(dY, SdY, X, SX, block), block)
    # wgrad output variants: FP32 only, INT8 only
    q0, s0, f0 = jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_q=False, want_f32=True)
    assert q0 is None and s0 is None
    q1, s1, f1 = jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_q=True, want_f32=False)
    assert f1 is None
    q2, s2, f2 = jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_f32=True)
    np.testing.assert_array_equal(host(f0), host(f2))
    np.testing.assert_array_equal(host(q1), host(q2))
    np.testing.assert_array_equal(host(s1), host(s2))


@pytest.mark.parametrize("shape", [1, 4, 6, 7, 8])
@pytest.mark.parametrize("block,N,C,D", [(32, 384, 160, 288), (32, 416, 96, 224), (64, 256, 192, 320), (128, 384, 256, 640)])
def test_linear_every_tile_shape(shape, block, N, C, D):
    """Each GEMM tile shape, forced through the test hook, on sizes that leave ragged tiles in both directions."""
    say(f"tile shape {shape} block={block} N={N} C={C} D={D}")
    (X, SX), (W, SW), (dY, SdY) = _quantized_layer(3500 + shape + N, N, C, D, block)
    Xd, SXd, Wd, SWd, dYd, SdYd = map(dev, (X, SX, W, SW, dY, SdY))
    jf.jf_debug_set_gemm_shape(shape)
    try:
        _check_linear("fwd", jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True), oracle.linear_fwd(X, SX, W, SW, block), block)
        _check_linear("dgrad", jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block, want_f32=True), oracle.linear_dgrad(dY, SdY, W, SW, block), block)
        _check_linear("wgrad", jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_f32=True), oracle.linear_wgrad(dY, SdY, X, SX, block), block)
        for which, (A, Bm, ref_a, ref_b, K) in enumerate(((Xd, Wd, X, W, C), (dYd, Wd, dY, np.ascontiguousarray(W.T), D),
                                                          (dYd, Xd, np.ascontiguousarray(dY.T), np.ascontiguousarray(X.T), N))):
            kb = K // block - 1
            got = host(jf.jf_debug_linear_partials(which, A, Bm, N, C, D, block, kb))
            np.testing.assert_array_equal(got, oracle.block_partials(ref_a, ref_b, block, kb))
    finally:
        jf.jf_debug_set_gemm_shape(0)


_K_SWEEP_CACHE = {}


def _k_sweep_case(nsteps):
    """Oracle results of a layer whose three contraction lengths are all 32 * nsteps (computed once per length)."""
    if nsteps not in _K_SWEEP_CACHE:
        n = 32 * nsteps
        (X, SX), (W, SW), (dY, SdY) = _quantized_layer(3900 + nsteps, n, n, n, 32)
        _K_SWEEP_CACHE[nsteps] = ((X, SX, W, SW, dY, SdY),
                                  oracle.linear_fwd(X, SX, W, SW, 32)[2], oracle.linear_dgrad(dY, SdY, W, SW, 32)[2],
                                  oracle.linear_wgrad(dY, SdY, X, SX, 32)[2])
    return _K_SWEEP_CACHE[nsteps]


@pytest.mark.parametrize("shape", [1, 4, 6, 7, 8])
def test_linear_k_loop_every_stage_count(shape):
    """The K loop of the block-32 kernels is a software pipeline whose prologue, main passes and last stages are
    separate code for every count of remaining stages, with the odd K steps of a stage-unaligned K run first.
    Sweep the number of 32-wide K steps so that every one of those paths runs, for every tile shape and for all
    three operand layouts; the FP32 accumulators must match the oracle's FP32 accumulators bit for bit."""
    jf.jf_debug_set_gemm_shape(shape)
    try:
        for nsteps in list(range(1, 19)) + [23, 24, 31, 32, 33, 35, 36, 41, 47]:
            say(f"tile shape {shape}: {nsteps} K steps")
            (X, SX, W, SW, dY, SdY), f_fwd, f_dgrad, f_wgrad = _k_sweep_case(nsteps)
            Xd, SXd, Wd, SWd, dYd, SdYd = map(dev, (X, SX, W, SW, dY, SdY))
            np.testing.assert_array_equal(host(jf.jf_linear_fwd(Xd, SXd, Wd, SWd, 32, want_f32=True)[2]), f_fwd)
            np.testing.assert_array_equal(host(jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, 32, want_f32=True)[2]), f_dgrad)
            np.testing.assert_array_equal(host(jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, 32, want_f32=True)[2]), f_wgrad)
    finally:
        jf.jf_debug_set_gemm_shape(0)


@pytest.mark.parametrize("block,shape", [(64, 1), (64, 4), (128, 1), (128, 6)])
def test_linear_k_loop_large_blocks(block, shape):
    """Blocks 64 and 128 run a chain of MFMAs per quantization block and, for waves of 2x2 sub-blocks, refill
    the fragment registers from the next stage while the current one is still being folded.  Sweep the number
    of K blocks so that the prologue, the main passes and every tail length run, for all three operand layouts;
    FP32 accumulators must match the oracle's bit for bit."""
    jf.jf_debug_set_gemm_shape(shape)
    try:
        for nkb in list(range(1, 11)) + [13, 16, 17]:
            n = block * nkb
            say(f"block {block} tile shape {shape}: {nkb} K blocks")
            (X, SX), (W, SW), (dY, SdY) = _quantized_layer(4200 + block + nkb, 256, n, 256, block)
            Xd, SXd, Wd, SWd = map(dev, (X, SX, W, SW))
            np.testing.assert_array_equal(host(jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True)[2]),
                                          oracle.linear_fwd(X, SX, W, SW, block)[2])
            # dgrad contracts over D, wgrad over N: build layers whose D resp. N is the swept length
            (X2, SX2), (W2, SW2), (dY2, SdY2) = _quantized_layer(4300 + block + nkb, 256, 256, n, block)
            np.testing.assert_array_equal(host(jf.jf_linear_dgrad(*map(dev, (dY2, SdY2, W2, SW2)), block, want_f32=True)[2]),
                                          oracle.linear_dgrad(dY2, SdY2, W2, SW2, block)[2])
            (X3, SX3), (W3, SW3), (dY3, SdY3) = _quantized_layer(4400 + block + nkb, n, 256, 256, block)
            np.testing.assert_array_equal(host(jf.jf_linear_wgrad(*map(dev, (dY3, SdY3, X3, SX3)), block, want_f32=True)[2]),
                                          oracle.linear_wgrad(dY3, SdY3, X3, SX3, block)[2])
    finally:
        jf.jf_debug_set_gemm_shape(0)


def test_linear_zero_blocks_and_run_to_run_stability():
    block, N, C, D = 32, 128, 128, 128
    (X, SX), (W, SW), _ = _quantized_layer(3100, N, C, D, block)
    X[:32] = 0
    SX[0] = 0.0                                                 # a whole row of all-zero input blocks -> zero output blocks
    Xd, SXd, Wd, SWd = map(dev, (X, SX, W, SW))
    q, s, f = jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True)
    assert not host(q)[:32].any() and not host(s)[0].any() and not host(f)[:32].any()
    assert np.all(np.isfinite(host(s)))
    _check_linear("fwd(zero rows)", (q, s, f), oracle.linear_fwd(X, SX, W, SW, block), block)
    q2, s2, f2 = jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True)
    assert torch.equal(q, q2) and torch.equal(s, s2) and torch.equal(f, f2)


def _sample_blocks(g, lm, ln, n):
    n = min(n, lm * ln)
    flat = g.choice(lm * ln, size=n, replace=False)
    return flat // ln, flat % ln


def _check_sampled(name, got, A, SA, Bm, SB, block, g, nblk=48, without_f32=None):
    """Full-size GPU result against the oracle on a sample of output blocks (each over the full K).
    without_f32: the same product launched without the FP32 output (the configuration the benchmark times); its
    codes and scales must equal those of the launch with it."""
    if without_f32 is not None:
        assert torch.equal(without_f32[0], got[0]) and torch.equal(without_f32[1], got[1]), name + ": INT8-only launch differs"
        assert without_f32[2] is None
    q, s, f = (host(t) for t in got)
    M, Nn = q.shape
    bp, bq = _sample_blocks(g, M // block, Nn // block, nblk)
    oq, os_, o32, o64 = oracle.linear_nt_blocks(A, SA, Bm, SB, bp, bq, block)
    nbad = 0
    for n, (p, c) in enumerate(zip(bp, bq)):
        sl = (slice(p * block, (p + 1) * block), slice(c * block, (c + 1) * block))
        np.testing.assert_array_equal(f[sl], o32[n], err_msg=name)
        assert_f32_close(f[sl], o64[n], block, name)
        assert_scales_close(s[p, c], os_[n], name)
        nbad += assert_codes_close(q[sl], oq[n], name, prequant=o32[n], scales=np.full((block, block), os_[n]))
    assert nbad == 0, name                                      # bit-identical accumulators, exact rounding
    # properties that hold everywhere: every non-zero block reaches +-127, scale = amax/127 of the FP32 output,
    # the half-step error bound.  Outputs above 2^25 elements are checked on eight random bands of block rows.
    if q.size > (1 << 25):
        rows_per_band = max(block, (1 << 22) // Nn // block * block)
        starts = g.choice(M // rows_per_band, size=min(8, M // rows_per_band), replace=False) * rows_per_band
        bands = [(int(r0), int(r0) + rows_per_band) for r0 in starts]
    else:
        bands = [(0, M)]
    for r0, r1 in bands:
        fb, qb, sb = f[r0:r1], q[r0:r1], s[r0 // block:r1 // block]
        amax = block_amax(fb, block)
        np.testing.assert_allclose(sb, amax / np.float32(127), rtol=1e-6)
        qa = block_amax(qb.astype(np.float32), block)
        assert np.all(qa[amax > 0] == 127)
        se = expand(sb.astype(np.float64), block)
        assert np.all(np.abs(qb.astype(np.float64) * se - fb) <= 0.5 * se * (1 + 1e-5))
    say(f"  {name}: {len(bp)} sampled blocks ok, {nbad} tie codes")


def test_linear_output_past_2_31_elements():
    """A forward product whose output has more than 2^31 elements (65536 x 32800, K = 64): the epilogue's
    addresses need 64 bits.  Sampled blocks and row bands, as for the large-GEMM sweep."""
    block, N, C, D = 32, 65536, 64, 32800
    say(f"linear fwd with a {N} x {D} output")
    g = workloads.rng(5300)
    (X, SX), (W, SW) = (oracle.quantize_block(workloads.gaussian(g, r, C, 1.0), block) for r in (N, D))
    got = jf.jf_linear_fwd(dev(X), dev(SX), dev(W), dev(SW), block, want_f32=True)
    assert got[0].numel() > (1 << 31)
    _check_sampled("fwd", got, X, SX, W, SW, block, g, 32)


def test_linear_config2_full_size_sampled():
    """GPT-2-small MLP shape (tokens 4096, in 768, out 3072, block 32) in the launch configuration the benchmark times."""
    block, N, C, D = 32, 4096, 768, 3072
    say("linear config 2 full size")
    (X, SX), (W, SW), (dY, SdY) = _quantized_layer(2, N, C, D, block)
    Xd, SXd, Wd, SWd, dYd, SdYd = map(dev, (X, SX, W, SW, dY, SdY))
    g = workloads.rng(4000)
    _check_sampled("fwd", jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True), X, SX, W, SW, block, g, 256,
                   without_f32=jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block))
    WT, SWT = oracle.transpose(W, SW, block)
    _check_sampled("dgrad", jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block, want_f32=True), dY, SdY, WT, SWT, block, g, 256,
                   without_f32=jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block))
    dYT, SdYT = oracle.transpose(dY, SdY, block)
    XT, SXT = oracle.transpose(X, SX, block)
    _check_sampled("wgrad", jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_f32=True), dYT, SdYT, XT, SXT, block, g, 256,
                   without_f32=jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block))


@pytest.mark.parametrize("block", [64, 128])
def test_linear_large_blocks_sampled(block):
    N, C, D = 1024, 1024, 512
    say(f"linear sampled block={block}")
    X, W, dY = workloads.linear_layer(50 + block, N, C, D, act_std=1.0, w_std=1.0, grad_std=1.0,
                                      outlier_fraction=0.005, outlier_factor=50.0)
    (X, SX), (W, SW), (dY, SdY) = (oracle.quantize_block(a, block) for a in (X, W, dY))
    Xd, SXd, Wd, SWd, dYd, SdYd = map(dev, (X, SX, W, SW, dY, SdY))
    g = workloads.rng(4100 + block)
    _check_sampled("fwd", jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True), X, SX, W, SW, block, g, 16)
    WT, SWT = oracle.transpose(W, SW, block)
    _check_sampled("dgrad", jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block, want_f32=True), dY, SdY, WT, SWT, block, g, 16)
    dYT, SdYT = oracle.transpose(dY, SdY, block)
    XT, SXT = oracle.transpose(X, SX, block)
    _check_sampled("wgrad", jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_f32=True), dYT, SdYT, XT, SXT, block, g, 16)


# --------------------------------------------------------------------------- GELU
def _check_eltwise(name, q, s, oq, os_, of64, block):
    assert_scales_close(host(s), os_, name + " scales")
    nbad = assert_codes_close(host(q), oq, name + " codes", prequant=of64, scales=os_, block=block)
    say(f"  {name}: {nbad} / {oq.size} codes differ by one")


# Blocks of 32 and 64 take one block per wave up to 24 M resp. 64 M elements; the last two cases are past that and
# run the 256-column workgroups, with a ragged last column group
@pytest.mark.parametrize("block,N,C", [(32, 96, 352), (64, 128, 192), (128, 256, 384), (32, 4096, 3072),
                                       (32, 32768, 1120), (64, 65536, 1088)])
def test_gelu_fwd_bwd(block, N, C):
    say(f"gelu block={block} {N}x{C}")
    x, gr = workloads.gelu_case(5000 + block + N, N, C)
    x[:block, :block] = 0.0
    x[block:2 * block, :block] = -np.abs(x[block:2 * block, :block]) - 6.0     # a block deep in the negative tail
    (X, SX), (G, SG) = oracle.quantize_block(x, block), oracle.quantize_block(gr, block)
    Xd, SXd, Gd, SGd = map(dev, (X, SX, G, SG))
    Y, SY = jf.jf_gelu_q(Xd, SXd, block)
    oY, oSY, oy = oracle.gelu_q(X, SX, block)
    _check_eltwise("gelu fwd", Y, SY, oY, oSY, oy, block)
    dX, SdX = jf.jf_gelu_q_bwd(Gd, SGd, Xd, SXd, block)
    odX, oSdX, odx = oracle.gelu_q_bwd(G, SG, X, SX, block)
    _check_eltwise("gelu bwd", dX, SdX, odX, oSdX, odx, block)


# --------------------------------------------------------------------------- LayerNorm
@pytest.mark.parametrize("block,N,C", [(32, 96, 352), (32, 64, 1280), (64, 128, 192), (128, 256, 384), (32, 4096, 768),
                                       (32, 64, 4096), (64, 128, 2304), (32, 19200, 96)])
def test_layernorm_fwd_bwd(block, N, C):
    say(f"layernorm block={block} {N}x{C}")
    x, gamma, beta, gr = workloads.layernorm_case(6000 + block + N, N, C)
    x[0, :] = 3.0                                               # a constant row: variance 0
    (X, SX), (G, SG) = oracle.quantize_block(x, block), oracle.quantize_block(gr, block)
    Xd, SXd, Gd, SGd, gd, bd = map(dev, (X, SX, G, SG, gamma, beta))
    eps = 1e-5
    Y, SY, mean, rstd = jf.jf_layernorm_q(Xd, SXd, gd, bd, eps, block)
    oY, oSY, omean, orstd, oy = oracle.layernorm_q(X, SX, gamma, beta, eps, block)
    np.testing.assert_allclose(host(mean), omean, rtol=0, atol=1e-5 * np.abs(oracle.dequantize(X, SX, block)).max())
    np.testing.assert_allclose(host(rstd), orstd, rtol=1e-5)
    _check_eltwise("layernorm fwd", Y, SY, oY, oSY, oy, block)
    # backward from the ORACLE's saved statistics, so that both sides start from identical inputs
    dX, SdX, dgam, dbet = jf.jf_layernorm_q_bwd(Gd, SGd, Xd, SXd, gd, dev(omean), dev(orstd), block)
    odX, oSdX, odg, odb, odx = oracle.layernorm_q_bwd(G, SG, X, SX, gamma, omean, orstd, block)
    _check_eltwise("layernorm bwd", dX, SdX, odX, oSdX, odx, block)
    gdq = oracle.dequantize(G, SG, block)
    xh = (oracle.dequantize(X, SX, block) - omean[:, None].astype(np.float64)) * orstd[:, None].astype(np.float64)
    assert_layernorm_param_grads_close(host(dgam), host(dbet), odg, odb, gdq, xh, "layernorm bwd")
    # run-to-run bit stability of the column reductions
    dX2, SdX2, dgam2, dbet2 = jf.jf_layernorm_q_bwd(Gd, SGd, Xd, SXd, gd, dev(omean), dev(orstd), block)
    assert torch.equal(dgam, dgam2) and torch.equal(dbet, dbet2) and torch.equal(dX, dX2)


@pytest.mark.parametrize("block,N,C", [(32, 64, 8192), (32, 96, 5152), (32, 128, 3072), (64, 128, 8192), (64, 192, 4800),
                                       (128, 256, 8192), (128, 128, 5248)])
def test_layernorm_wide_rows(block, N, C):
    """LayerNorm works on tiles after a pass that only leaves sums, so rows may be wider than a workgroup could hold
    (hidden 8192 is the widest LayerNorm the paper's speed comparison quotes); 5152 / 4800 / 5248 leave a ragged last
    strip and a last column range that uses a part of its waves."""
    say(f"layernorm wide rows {N}x{C}")
    x, gamma, beta, gr = workloads.layernorm_case(6500 + C, N, C)
    (X, SX), (G, SG) = oracle.quantize_block(x, block), oracle.quantize_block(gr, block)
    Y, SY, mean, rstd = jf.jf_layernorm_q(dev(X), dev(SX), dev(gamma), dev(beta), 1e-5, block)
    oY, oSY, omean, orstd, oy = oracle.layernorm_q(X, SX, gamma, beta, 1e-5, block)
    np.testing.assert_allclose(host(mean), omean, rtol=0, atol=1e-5 * np.abs(oracle.dequantize(X, SX, block)).max())
    np.testing.assert_allclose(host(rstd), orstd, rtol=1e-5)
    _check_eltwise("layernorm fwd", Y, SY, oY, oSY, oy, block)
    dX, SdX, dgam, dbet = jf.jf_layernorm_q_bwd(dev(G), dev(SG), dev(X), dev(SX), dev(gamma), dev(omean), dev(orstd), block)
    odX, oSdX, odg, odb, odx = oracle.layernorm_q_bwd(G, SG, X, SX, gamma, omean, orstd, block)
    _check_eltwise("layernorm bwd", dX, SdX, odX, oSdX, odx, block)
    xh = (oracle.dequantize(X, SX, block) - omean[:, None].astype(np.float64)) * orstd[:, None].astype(np.float64)
    assert_layernorm_param_grads_close(host(dgam), host(dbet), odg, odb, oracle.dequantize(G, SG, block), xh, "layernorm bwd")


# --------------------------------------------------------------------------- Add with row partials, LayerNorm from them
@pytest.mark.parametrize("block,N,C", [(32, 96, 352), (64, 128, 192), (128, 256, 384), (32, 8192, 1280)])
def test_add_and_layernorm_from_partials(block, N, C):
    say(f"add + layernorm from partials block={block} {N}x{C}")
    g = workloads.rng(7000 + block + N)
    x1 = workloads.gaussian(g, N, C, 1.0)
    workloads.with_outlier_columns(g, x1, 0.01, 20.0)
    x2 = workloads.gaussian(g, N, C, 0.3, mean=0.1)
    x1[:block, :block] = 0.0
    x2[:block, :block] = 0.0                                    # an all-zero output block
    (X1, S1), (X2, S2) = oracle.quantize_block(x1, block), oracle.quantize_block(x2, block)
    gamma = (1.0 + 0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)
    beta = (0.1 * g.standard_normal(C, dtype=np.float32)).astype(np.float32)
    X1d, S1d, X2d, S2d, gd, bd = map(dev, (X1, S1, X2, S2, gamma, beta))
    Y, SY, rm, rq = jf.jf_add_q(X1d, S1d, X2d, S2d, block, want_partials=True)
    oY, oSY, orm, orq, of = oracle.add_q(X1, S1, X2, S2, block)
    _check_eltwise("add", Y, SY, oY, oSY, of, block)
    Yn, SYn = jf.jf_add_q(X1d, S1d, X2d, S2d, block)            # without partials: same codes
    assert torch.equal(Y, Yn) and torch.equal(SY, SYn)
    # partials are FP32 sums of B terms: tolerance relative to the sum of magnitudes
    absum = np.abs(of).reshape(N, C // block, block).sum(axis=2)
    # (the library stores the partials block column by block column: (C / block, N))
    assert np.all(np.abs(host(rm).T.astype(np.float64) - orm) <= 1e-5 * absum / block + 1e-30)
    assert np.all(np.abs(host(rq).T.astype(np.float64) - orq) <= 1e-5 * orq + 1e-30)
    # LayerNorm from the ORACLE's partials, so that both sides start from identical inputs
    eps = 1e-5
    Z, SZ, mean, rstd = jf.jf_layernorm_q_partials(dev(oY), dev(oSY), dev(orm.T), dev(orq.T), gd, bd, eps, block)
    omean, orstd = oracle.row_stats_from_partials(orm, orq, C, eps, block)
    oZ, oSZ, oz = oracle.layernorm_q_stats(oY, oSY, gamma, beta, omean, orstd, block)
    np.testing.assert_allclose(host(mean), omean, rtol=0, atol=1e-5 * np.abs(of).max())
    np.testing.assert_allclose(host(rstd), orstd, rtol=1e-5)
    _check_eltwise("layernorm from partials", Z, SZ, oZ, oSZ, oz, block)


# --------------------------------------------------------------------------- Dropout
@pytest.mark.parametrize("block,N,C,p", [(32, 96, 352, 0.1), (64, 128, 192, 0.5), (128, 256, 384, 0.0), (32, 4096, 3072, 0.1)])
def test_dropout_fwd_and_as_its_own_backward(block, N, C, p):
    say(f"dropout block={block} {N}x{C} p={p}")
    g = workloads.rng(8000 + block + N)
    x, gr = workloads.gelu_case(8100 + block, N, C)
    bits, keep = workloads.dropout_mask_bits(g, N, C, p)
    keep[:block, :block] = False                                # a block that is dropped entirely
    bits = np.packbits(keep, axis=1, bitorder="little")
    for name, t in (("dropout fwd", x), ("dropout bwd", gr)):
        X, SX = oracle.quantize_block(t, block)
        Y, SY = jf.jf_dropout_q(dev(X), dev(SX), dev(bits), p, block)
        oY, oSY, of = oracle.dropout_q(X, SX, bits, p, block)
        _check_eltwise(name, Y, SY, oY, oSY, of, block)
        assert not host(Y)[:block, :block].any() and host(SY)[0, 0] == 0


# --------------------------------------------------------------------------- large-GEMM sweep (config 5)
# Every shape of the sweep at every block size, at full size.  Each product is checked on 256 sampled output
# blocks (each over the full K, FP32 accumulator bit-exact, codes identical), on properties of the whole output,
# and against the launch without the FP32 output, which is the configuration the benchmark times.
_SWEEP_SHAPES = [(2048, 2048, 2048), (4096, 4096, 4096), (8192, 8192, 8192),
                 (16384, 4096, 4096), (16384, 4096, 11008), (16384, 11008, 4096)]
_SWEEP_CASES = [(N, C, D, block) for (N, C, D) in _SWEEP_SHAPES for block in (32, 64, 128)]


@pytest.mark.parametrize("N,C,D,block", _SWEEP_CASES)
def test_linear_config5_sweep_sampled(N, C, D, block):
    """Large-GEMM sweep shapes at full size: N(0,1) data with 0.5 % outlier columns x50, all three products."""
    say(f"linear sweep N={N} C={C} D={D} block={block}: drawing and quantizing inputs")
    X, W, dY = workloads.linear_layer(5000 + N // 64 + C // 32 + block, N, C, D, act_std=1.0, w_std=1.0, grad_std=1.0,
                                      outlier_fraction=0.005, outlier_factor=50.0)
    (X, SX), (W, SW), (dY, SdY) = (oracle.quantize_block(a, block) for a in (X, W, dY))
    Xd, SXd, Wd, SWd, dYd, SdYd = map(dev, (X, SX, W, SW, dY, SdY))
    g = workloads.rng(5100 + block)
    nblk = 256
    say("  forward")
    _check_sampled("fwd", jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block, want_f32=True), X, SX, W, SW, block, g, nblk,
                   without_f32=jf.jf_linear_fwd(Xd, SXd, Wd, SWd, block))
    say("  dgrad")
    WT, SWT = oracle.transpose(W, SW, block)
    _check_sampled("dgrad", jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block, want_f32=True), dY, SdY, WT, SWT, block, g, nblk,
                   without_f32=jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block))
    del WT, SWT
    say("  wgrad")
    dYT, SdYT = oracle.transpose(dY, SdY, block)
    XT, SXT = oracle.transpose(X, SX, block)
    _check_sampled("wgrad", jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_f32=True), dYT, SdYT, XT, SXT, block, g, nblk,
                   without_f32=jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block))
    torch.cuda.empty_cache()


# --------------------------------------------------------------------------- both backward products in one call
@pytest.mark.parametrize("block,N,C,D", [(32, 4096, 768, 3072), (32, 416, 96, 224), (32, 512, 640, 256), (32, 2048, 2048, 2048),
                                         (64, 256, 192, 320), (128, 384, 256, 640)])
def test_linear_bwd_equals_dgrad_and_wgrad(block, N, C, D):
    """jf_linear_bwd (one launch for both products where each alone is too small to fill the chip, else two) gives
    what jf_linear_dgrad and jf_linear_wgrad give, bit for bit; those are checked against the oracle above."""
    say(f"linear bwd block={block} N={N} C={C} D={D}")
    (X, SX), (W, SW), (dY, SdY) = _quantized_layer(4700 + N + block, N, C, D, block)
    Xd, SXd, Wd, SWd, dYd, SdYd = map(dev, (X, SX, W, SW, dY, SdY))
    for want_f32 in (True, False):
        wd = jf.jf_linear_dgrad(dYd, SdYd, Wd, SWd, block, want_f32=want_f32)
        ww = jf.jf_linear_wgrad(dYd, SdYd, Xd, SXd, block, want_f32=want_f32)
        gd, gw = jf.jf_linear_bwd(dYd, SdYd, Wd, SWd, Xd, SXd, block, want_f32=want_f32)
        for got, want in ((gd, wd), (gw, ww)):
            for g_, w_ in zip(got, want):
                assert (g_ is None and w_ is None) or torch.equal(g_, w_)
    if (block, N, C, D) == (32, 416, 96, 224):                 # ragged tiles in both products: also against the oracle
        _check_linear("bwd: dgrad", jf.jf_linear_bwd(dYd, SdYd, Wd, SWd, Xd, SXd, block, want_f32=True)[0],
                      oracle.linear_dgrad(dY, SdY, W, SW, block), block)
        _check_linear("bwd: wgrad", jf.jf_linear_bwd(dYd, SdYd, Wd, SWd, Xd, SXd, block, want_f32=True)[1],
                      oracle.linear_wgrad(dY, SdY, X, SX, block), block)
