"""Pins of the CPU oracle against things other than itself (no GPU needed).

The paper prints no numeric example, so each oracle function is pinned by
closed forms, invariants, brute force on tiny inputs and library routines
(numpy float64 matmul, math.erf, torch CPU float64 layer_norm / gelu autograd).
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2403_12422_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_q(g, rows, cols, block, spread=True):
    """Random valid per-block tensor (codes in [-127,127], positive scales of mixed magnitude)."""
    q = g.integers(-127, 128, size=(rows, cols), dtype=np.int64).astype(np.int8)
    s = np.exp(g.uniform(-6, 1, size=(rows // block, cols // block))).astype(np.float32) if spread else np.ones(
        (rows // block, cols // block), np.float32)
    return q, s


def _dq(q, s, block):
    return q.astype(np.float64) * np.kron(s.astype(np.float64), np.ones((block, block)))


# --------------------------------------------------------------------------- O1 quantizer (Sec. 4, Eq. 1)
def test_quantizer_hand_cases():
    for line in open(os.path.join(GOLDEN, "quantizer_cases.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        vals, codes = line.split("|")
        vals = np.array([float(v) for v in vals.split()], np.float32)
        codes = np.array([int(c) for c in codes.split()], np.int8)
        reps = -(-1024 // vals.size)
        x = np.tile(vals, reps)[:1024].reshape(32, 32)
        want = np.tile(codes, reps)[:1024].reshape(32, 32)
        q, s = oracle.quantize_block(x, 32)
        assert s.shape == (1, 1) and s[0, 0] == np.float32(abs(vals[0])) / np.float32(127)
        np.testing.assert_array_equal(q, want)


@pytest.mark.parametrize("block", [32, 64, 128])
def test_quantizer_invariants(block):
    g = workloads.rng(101 + block)
    x = workloads.gaussian(g, 2 * block, 3 * block, 1.0)
    workloads.with_outlier_columns(g, x, 0.02, 20.0)
    q, s = oracle.quantize_block(x, block)
    assert q.dtype == np.int8 and s.dtype == np.float32
    assert q.min() >= -127 and q.max() <= 127
    S = np.kron(s.astype(np.float64), np.ones((block, block)))
    err = np.abs(x.astype(np.float64) - q.astype(np.float64) * S)
    assert np.all(err <= 0.5 * S * (1 + 2.0 ** -22))          # dequantization error at most half a step
    for bi in range(2):
        for bj in range(3):
            blk = x[bi * block:(bi + 1) * block, bj * block:(bj + 1) * block]
            qb = q[bi * block:(bi + 1) * block, bj * block:(bj + 1) * block]
            amax = np.abs(blk).max()
            assert np.abs(qb).max() == 127                       # the extreme element maps to +-127
            assert s[bi, bj] == np.float32(amax) / np.float32(127)
            assert abs(float(s[bi, bj]) * 127 - float(amax)) <= float(amax) * 2.0 ** -23
            # elementwise definition, written independently with numpy (np.rint is half-to-even)
            want = np.clip(np.rint(blk.astype(np.float64) / np.float64(s[bi, bj])), -127, 127)
            np.testing.assert_array_equal(qb, want.astype(np.int8))


def test_quantizer_zero_block_and_single_outlier():
    x = np.zeros((64, 64), np.float32)
    x[32:, 32:] = 0.001
    x[40, 50] = -1000.0                    # single outlier in block (1,1)
    x[0:32, 32:64] = 3.0                   # constant block
    q, s = oracle.quantize_block(x, 32)
    assert s[0, 0] == 0.0 and not q[:32, :32].any()            # all-zero block: scale 0, codes 0, no NaN
    assert s[1, 0] == 0.0 and not q[32:, :32].any()
    assert np.all(q[:32, 32:] == 127) and s[0, 1] == np.float32(3.0) / np.float32(127)
    assert q[40, 50] == -127
    rest = q[32:, 32:].copy()
    rest[8, 18] = 0
    assert not rest.any()                  # 0.001 / (1000/127) rounds to 0: the outlier only costs its own block
    assert np.all(np.isfinite(s))


def test_quantizer_transpose_commutes():
    g = workloads.rng(7)
    x = workloads.gaussian(g, 96, 160, 1.0)
    workloads.with_outlier_columns(g, x, 0.05, 20.0)
    q, s = oracle.quantize_block(x, 32)
    qT, sT = oracle.transpose(q, s, 32)
    q2, s2 = oracle.quantize_block(np.ascontiguousarray(x.T), 32)
    np.testing.assert_array_equal(qT, q2)
    np.testing.assert_array_equal(sT, s2)
    np.testing.assert_array_equal(qT, q.T)                      # transpose is literally the numpy transpose
    np.testing.assert_array_equal(sT, s.T)


def test_quantizer_requantize_is_idempotent():
    g = workloads.rng(8)
    x = workloads.gaussian(g, 64, 64, 3.0)
    q, s = oracle.quantize_block(x, 32)
    xd = oracle.dequantize(q, s, 32)
    np.testing.assert_array_equal(xd, _dq(q, s, 32))             # Q^-1 is code * scale
    q2, s2 = oracle.quantize_block(xd.astype(np.float32), 32)
    np.testing.assert_array_equal(q2, q)
    np.testing.assert_allclose(s2, s, rtol=2.0 ** -22)


def test_quantizer_per_tensor_special_case():
    # one block covering the whole matrix = the textbook symmetric per-tensor INT8 quantizer
    g = workloads.rng(9)
    x = workloads.gaussian(g, 128, 128, 1.0)
    q, s = oracle.quantize_block(x, 128)
    scale = np.float32(np.abs(x).max()) / np.float32(127)
    assert s.shape == (1, 1) and s[0, 0] == scale
    np.testing.assert_array_equal(q, np.rint(x.astype(np.float64) / np.float64(scale)).astype(np.int8))


def test_quantizer_rejects_ragged_shapes():
    with pytest.raises(ValueError):
        oracle.quantize_block(np.zeros((48, 64), np.float32), 32)


# --------------------------------------------------------------------------- O3 blocked INT8 matmul (Sec. 5.3, Alg. 1)
def test_block_partials_brute_force():
    g = workloads.rng(11)
    M, Nn, K, B = 64, 32, 96, 32
    A = g.integers(-127, 128, size=(M, K)).astype(np.int8)
    Bm = g.integers(-127, 128, size=(Nn, K)).astype(np.int8)
    A[:32, :32] = 127                      # adversarial fills reach the extreme +-B*127^2
    Bm[:32, :32] = -127
    for kb in range(K // B):
        got = oracle.block_partials(A, Bm, B, kb)
        want = np.zeros((M, Nn), np.int64)
        for i in range(M):                 # literal triple loop in Python integers
            for j in range(Nn):
                acc = 0
                for kk in range(kb * B, (kb + 1) * B):
                    acc += int(A[i, kk]) * int(Bm[j, kk])
                want[i, j] = acc
        np.testing.assert_array_equal(got.astype(np.int64), want)
    assert oracle.block_partials(A, Bm, B, 0)[0, 0] == -32 * 127 * 127


@pytest.mark.parametrize("block", [32, 64])
def test_linear_unit_scales_is_integer_matmul(block):
    g = workloads.rng(12)
    M, Nn, K = 2 * block, 3 * block, 4 * block
    A, SA = _rand_q(g, M, K, block, spread=False)
    Bm, SB = _rand_q(g, Nn, K, block, spread=False)
    q, s, a32, a64 = oracle.linear_nt(A, SA, Bm, SB, block)
    want = A.astype(np.int64) @ Bm.astype(np.int64).T
    np.testing.assert_array_equal(a64, want.astype(np.float64))
    np.testing.assert_array_equal(a32.astype(np.float64), want.astype(np.float64))   # |sum| < 2^24: exact in FP32 too
    # uniform scales factor out
    SA2 = np.full_like(SA, 0.5)
    SB2 = np.full_like(SB, 0.25)
    _, _, b32, b64 = oracle.linear_nt(A, SA2, Bm, SB2, block)
    np.testing.assert_array_equal(b64, want * 0.125)


@pytest.mark.parametrize("block", [32, 64, 128])
def test_linear_equals_dense_matmul_of_dequantized(block):
    g = workloads.rng(13 + block)
    M, Nn, K = 2 * block, block, 3 * block
    A, SA = _rand_q(g, M, K, block)
    Bm, SB = _rand_q(g, Nn, K, block)
    q, s, a32, a64 = oracle.linear_nt(A, SA, Bm, SB, block)
    dense = _dq(A, SA, block) @ _dq(Bm, SB, block).T            # numpy float64 library matmul
    scale = np.abs(dense).max()
    assert np.abs(a64 - dense).max() <= 1e-12 * scale
    # FP32 accumulator: K/B fused multiply-adds per element, each within half an ulp
    assert np.abs(a32.astype(np.float64) - dense).max() <= (K // block + 1) * 2.0 ** -24 * 4 * scale
    # output quantizer = Eq. 1 applied to the FP32 accumulator
    q2, s2 = oracle.quantize_block(a32, block)
    np.testing.assert_array_equal(q, q2)
    np.testing.assert_array_equal(s, s2)


def test_linear_fma_order_is_k_ascending_single_accumulator():
    # two K blocks, one output element followed by hand: acc = fma(t1, v1, fma(t0, v0, 0))
    B = 32
    A = np.zeros((B, 2 * B), np.int8)
    Bm = np.zeros((B, 2 * B), np.int8)
    A[0, 0], Bm[0, 0] = 127, 127            # v0 = 16129
    A[0, B], Bm[0, B] = 113, -97            # v1 = -10961
    SA = np.array([[0.1, 0.3]], np.float32)
    SB = np.array([[0.7, 0.9]], np.float32)
    _, _, a32, a64 = oracle.linear_nt(A, SA, Bm, SB, B)
    t0 = np.float32(SA[0, 0] * SB[0, 0])
    t1 = np.float32(SA[0, 1] * SB[0, 1])
    step0 = np.float32(np.float64(t0) * 16129.0)                 # fma with zero addend = rounded product
    want = np.float32(np.float64(t1) * -10961.0 + np.float64(step0))   # exact in float64, then one rounding
    assert a32[0, 0] == want
    assert a64[0, 0] == np.float64(SA[0, 0]) * np.float64(SB[0, 0]) * 16129.0 + np.float64(SA[0, 1]) * np.float64(SB[0, 1]) * -10961.0


def test_linear_blocks_subset_matches_full():
    g = workloads.rng(14)
    B = 32
    A, SA = _rand_q(g, 96, 64, B)
    Bm, SB = _rand_q(g, 128, 64, B)
    q, s, a32, a64 = oracle.linear_nt(A, SA, Bm, SB, B)
    bp, bq = np.array([0, 2, 1]), np.array([3, 0, 1])
    qb, sb, f32, f64 = oracle.linear_nt_blocks(A, SA, Bm, SB, bp, bq, B)
    for n, (p, c) in enumerate(zip(bp, bq)):
        np.testing.assert_array_equal(qb[n], q[p * B:(p + 1) * B, c * B:(c + 1) * B])
        np.testing.assert_array_equal(f32[n], a32[p * B:(p + 1) * B, c * B:(c + 1) * B])
        assert sb[n] == s[p, c]


def test_three_products_against_dense_reference():
    # Sec. 4: Y = X W^T, dX = dY W, dW = dY^T X on dequantized operands (numpy float64)
    g = workloads.rng(15)
    B, N, C, D = 32, 64, 96, 128
    X, SX = _rand_q(g, N, C, B)
    W, SW = _rand_q(g, D, C, B)
    dY, SdY = _rand_q(g, N, D, B)
    Xd, Wd, dYd = _dq(X, SX, B), _dq(W, SW, B), _dq(dY, SdY, B)
    for got, want in ((oracle.linear_fwd(X, SX, W, SW, B), Xd @ Wd.T),
                      (oracle.linear_dgrad(dY, SdY, W, SW, B), dYd @ Wd),
                      (oracle.linear_wgrad(dY, SdY, X, SX, B), dYd.T @ Xd)):
        q, s, a32, a64 = got
        assert a64.shape == want.shape
        assert np.abs(a64 - want).max() <= 1e-12 * np.abs(want).max()
        q2, s2 = oracle.quantize_block(a32, B)
        np.testing.assert_array_equal(q, q2)
        np.testing.assert_array_equal(s, s2)


def test_whole_linear_quantization_error_is_small_and_outlier_robust():
    # sanity of the method itself (Sec. 4 claim): per-block INT8 keeps ~1% error with outlier channels
    for frac in (0.0, 0.01):
        g = workloads.rng(16)
        X = workloads.gaussian(g, 128, 256, 1.0)
        if frac:
            workloads.with_outlier_columns(g, X, frac, 20.0)
        W = workloads.gaussian(g, 128, 256, 0.02)
        Xq, SX = oracle.quantize_block(X, 32)
        Wq, SW = oracle.quantize_block(W, 32)
        _, _, _, y = oracle.linear_fwd(Xq, SX, Wq, SW, 32)
        ref = X.astype(np.float64) @ W.astype(np.float64).T
        rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
        assert rel < 0.03


# --------------------------------------------------------------------------- O4 GELU (App. A)
def _golden_cdf():
    rows = []
    for line in open(os.path.join(GOLDEN, "std_normal_cdf.txt")):
        if line.strip() and not line.startswith("#"):
            rows.append([float(v) for v in line.split()])
    return np.array(rows)


def test_gelu_closed_form_values():
    tab = _golden_cdf()
    # a block whose codes 0..127 times scale hit the tabulated x exactly: scale = 1/32, code = 32 x
    B = 32
    Xq = np.zeros((B, B), np.int8)
    SX = np.array([[1.0 / 32]], np.float32)
    for i, (x, cdf, pdf) in enumerate(tab):
        Xq[0, i] = int(round(x * 32))
    gq = np.full((B, B), 127, np.int8)
    SG = np.array([[1.0 / 127]], np.float32)          # upstream gradient == 1 (up to FP32 rounding of 1/127)
    _, _, y = oracle.gelu_q(Xq, SX, B)
    _, _, dx = oracle.gelu_q_bwd(gq, SG, Xq, SX, B)
    gval = 127 * float(np.float32(1.0 / 127))
    for i, (x, cdf, pdf) in enumerate(tab):
        assert abs(y[0, i] - x * cdf) < 1e-14
        assert abs(dx[0, i] - gval * (x * pdf + cdf)) < 1e-14
    assert y[1, 1] == 0.0                               # GELU(0) = 0


def test_gelu_matches_math_erf_torch_and_finite_differences():
    g = workloads.rng(21)
    B = 32
    x, gr = workloads.gelu_case(21, 64, 64)
    Xq, SX = oracle.quantize_block(x, B)
    Gq, SG = oracle.quantize_block(gr, B)
    xd, gd = _dq(Xq, SX, B), _dq(Gq, SG, B)
    Yq, SY, y = oracle.gelu_q(Xq, SX, B)
    dXq, SdX, dx = oracle.gelu_q_bwd(Gq, SG, Xq, SX, B)
    want = np.vectorize(lambda v: v * 0.5 * (1.0 + math.erf(v / math.sqrt(2.0))))(xd)
    assert np.abs(y - want).max() < 1e-14
    xt = torch.tensor(xd, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.gelu(xt, approximate="none")
    yt.backward(torch.tensor(gd))
    assert np.abs(y - yt.detach().numpy()).max() < 1e-13
    assert np.abs(dx - xt.grad.numpy()).max() < 1e-13 * max(1.0, np.abs(gd).max())
    h = 1e-6                                            # derivative by central differences
    f = lambda v: v * 0.5 * (1.0 + math.erf(v / math.sqrt(2.0)))
    fd = np.vectorize(lambda v: (f(v + h) - f(v - h)) / (2 * h))(xd)
    assert np.abs(dx - gd * fd).max() < 1e-8 * np.abs(gd).max()
    # limits: GELU(x) -> x for large x, -> 0- for very negative x
    assert abs(f(9.0) - 9.0) < 1e-15 and -1e-15 < f(-9.0) <= 0.0
    # the quantize step of Alg. 2 is Eq. 1 on the FP32 result
    q2, s2 = oracle.quantize_block(y.astype(np.float32), B)
    np.testing.assert_array_equal(Yq, q2)
    np.testing.assert_array_equal(SY, s2)
    q3, s3 = oracle.quantize_block(dx.astype(np.float32), B)
    np.testing.assert_array_equal(dXq, q3)
    np.testing.assert_array_equal(SdX, s3)


# --------------------------------------------------------------------------- O5 LayerNorm (App. A)
def test_layernorm_matches_torch_float64():
    B, N, C = 32, 64, 160
    x, gamma, beta, gr = workloads.layernorm_case(31, N, C, outlier_fraction=0.02)
    Xq, SX = oracle.quantize_block(x, B)
    Gq, SG = oracle.quantize_block(gr, B)
    xd, gd = _dq(Xq, SX, B), _dq(Gq, SG, B)
    eps = 1e-5
    Yq, SY, mean, rstd, y = oracle.layernorm_q(Xq, SX, gamma, beta, eps, B)
    xt = torch.tensor(xd, dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(gamma, dtype=torch.float64, requires_grad=True)
    bt = torch.tensor(beta, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.layer_norm(xt, (C,), gt, bt, eps=float(np.float32(eps)))
    assert np.abs(y - yt.detach().numpy()).max() < 1e-12 * np.abs(y).max()
    np.testing.assert_allclose(mean, xd.mean(axis=1), rtol=0, atol=2e-7 * np.abs(xd).max())
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt(xd.var(axis=1) + float(np.float32(eps))), rtol=1e-7)
    q2, s2 = oracle.quantize_block(y.astype(np.float32), B)
    np.testing.assert_array_equal(Yq, q2)
    np.testing.assert_array_equal(SY, s2)

    # backward with the exact (float64) statistics fed back as float32, like the saved tensors
    yt.backward(torch.tensor(gd))
    dXq, SdX, dgam, dbet, dx = oracle.layernorm_q_bwd(Gq, SG, Xq, SX, gamma, mean, rstd, B)
    tol = 1e-6                                           # mean/rstd were rounded to FP32
    assert np.abs(dx - xt.grad.numpy()).max() < tol * np.abs(dx).max()
    assert np.abs(dgam - gt.grad.numpy()).max() < tol * np.abs(dgam).max()
    assert np.abs(dbet - bt.grad.numpy()).max() < tol * np.abs(dbet).max()
    q3, s3 = oracle.quantize_block(dx.astype(np.float32), B)
    np.testing.assert_array_equal(dXq, q3)
    np.testing.assert_array_equal(SdX, s3)


def test_layernorm_unit_affine_row_moments():
    B, N, C = 32, 32, 96
    x, _, _, _ = workloads.layernorm_case(32, N, C)
    Xq, SX = oracle.quantize_block(x, B)
    eps = 1e-5
    ones, zeros = np.ones(C, np.float32), np.zeros(C, np.float32)
    _, _, mean, rstd, y = oracle.layernorm_q(Xq, SX, ones, zeros, eps, B)
    var = _dq(Xq, SX, B).var(axis=1)
    np.testing.assert_allclose(y.mean(axis=1), 0.0, atol=1e-13)
    np.testing.assert_allclose(y.var(axis=1), var / (var + float(np.float32(eps))), rtol=1e-12)


def test_layernorm_backward_finite_difference():
    B, N, C = 32, 32, 64
    x, gamma, beta, gr = workloads.layernorm_case(33, N, C)
    Xq, SX = oracle.quantize_block(x, B)
    Gq, SG = oracle.quantize_block(gr, B)
    xd, gd = _dq(Xq, SX, B), _dq(Gq, SG, B)
    eps = float(np.float32(1e-5))

    def ln(v):
        mu = v.mean(axis=1, keepdims=True)
        var = v.var(axis=1, keepdims=True)
        return (v - mu) / np.sqrt(var + eps) * gamma.astype(np.float64) + beta.astype(np.float64)

    mu = xd.mean(axis=1)
    rs = 1.0 / np.sqrt(xd.var(axis=1) + eps)
    _, _, _, _, dx = oracle.layernorm_q_bwd(Gq, SG, Xq, SX, gamma, mu.astype(np.float32), rs.astype(np.float32), B)
    h = 1e-5
    for (i, j) in [(0, 0), (5, 17), (31, 63)]:
        e = np.zeros_like(xd)
        e[i, j] = h
        fd = ((ln(xd + e) - ln(xd - e)) * gd).sum() / (2 * h)
        assert abs(dx[i, j] - fd) < 2e-6 * np.abs(dx).max()


# --------------------------------------------------------------------------- Add with row partials (App. A)
def _two_tensors(seed, N, C, block):
    g = workloads.rng(seed)
    x1 = workloads.gaussian(g, N, C, 1.0)
    workloads.with_outlier_columns(g, x1, 0.01, 20.0)
    x2 = workloads.gaussian(g, N, C, 0.3, mean=0.1)
    return oracle.quantize_block(x1, block), oracle.quantize_block(x2, block)


@pytest.mark.parametrize("block", [32, 64])
def test_add_equals_numpy_sum_of_dequantized_and_commutes(block):
    N, C = 2 * block, 3 * block
    (X1, S1), (X2, S2) = _two_tensors(700 + block, N, C, block)
    Y, SY, rm, rq, f = oracle.add_q(X1, S1, X2, S2, block)
    want = oracle.dequantize(X1, S1, block) + oracle.dequantize(X2, S2, block)       # library float64 addition
    np.testing.assert_array_equal(f, want)
    # the output is Eq. 1 applied to the FP32 sum: same pins as the quantizer
    q, s = oracle.quantize_block(want.astype(np.float32), block)
    np.testing.assert_array_equal(Y, q)
    np.testing.assert_array_equal(SY, s)
    Y2, SY2, rm2, rq2, _ = oracle.add_q(X2, S2, X1, S1, block)
    np.testing.assert_array_equal(Y, Y2)
    np.testing.assert_array_equal(SY, SY2)
    np.testing.assert_array_equal(rm, rm2)
    np.testing.assert_array_equal(rq, rq2)


def test_add_of_zero_tensor_requantizes_to_the_same_codes():
    block, N, C = 32, 64, 96
    (X1, S1), _ = _two_tensors(711, N, C, block)
    Z, SZ = np.zeros((N, C), np.int8), np.zeros((N // block, C // block), np.float32)
    Y, SY, _, _, _ = oracle.add_q(X1, S1, Z, SZ, block)
    np.testing.assert_array_equal(Y, X1)
    np.testing.assert_allclose(SY, S1, rtol=2e-7)


def test_add_row_partials_against_numpy_and_row_statistics():
    """Row partials: mean and sum of squares over each block's columns; combining them gives the row mean and
    the biased row variance of the whole row (checked against numpy on the full rows)."""
    block, N, C = 32, 64, 160
    (X1, S1), (X2, S2) = _two_tensors(720, N, C, block)
    Y, SY, rm, rq, f = oracle.add_q(X1, S1, X2, S2, block)
    y32 = f.astype(np.float32).astype(np.float64)
    blocks = y32.reshape(N, C // block, block)
    np.testing.assert_allclose(rm, blocks.mean(axis=2), rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(rq, (blocks ** 2).sum(axis=2), rtol=1e-6)
    eps = 1e-5
    mean, rstd = oracle.row_stats_from_partials(rm, rq, C, eps, block)
    np.testing.assert_allclose(mean, y32.mean(axis=1), rtol=0, atol=2e-6)
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt(y32.var(axis=1) + eps), rtol=1e-5)
    # a constant row has variance 0 whatever its mean
    rm_c = np.full((block, C // block), 7.0, np.float32)
    rq_c = np.full((block, C // block), 49.0 * block, np.float32)
    mean_c, rstd_c = oracle.row_stats_from_partials(rm_c, rq_c, C, eps, block)
    assert mean_c[0] == 7.0 and abs(rstd_c[0] - 1.0 / math.sqrt(eps)) < 1e-2


def test_layernorm_from_statistics_matches_torch_and_the_self_statistics_operator():
    block, N, C = 32, 64, 96
    x, gamma, beta, _ = workloads.layernorm_case(730, N, C)
    X, SX = oracle.quantize_block(x, block)
    xd = oracle.dequantize(X, SX, block)
    eps = 1e-5
    # statistics of the dequantized tensor itself, via ADD with a zero tensor: then the operator must agree with
    # the LayerNorm that computes its own statistics, and with torch's float64 layer_norm
    Z, SZ = np.zeros((N, C), np.int8), np.zeros((N // block, C // block), np.float32)
    _, _, rm, rq, _ = oracle.add_q(X, SX, Z, SZ, block)
    mean, rstd = oracle.row_stats_from_partials(rm, rq, C, eps, block)
    Y, SY, f = oracle.layernorm_q_stats(X, SX, gamma, beta, mean, rstd, block)
    Y0, SY0, mean0, rstd0, f0 = oracle.layernorm_q(X, SX, gamma, beta, eps, block)
    np.testing.assert_allclose(mean, mean0, rtol=0, atol=1e-6 * np.abs(xd).max())
    np.testing.assert_allclose(rstd, rstd0, rtol=1e-5)
    want = torch.nn.functional.layer_norm(torch.from_numpy(xd), (C,), torch.from_numpy(gamma.astype(np.float64)),
                                          torch.from_numpy(beta.astype(np.float64)), eps).numpy()
    np.testing.assert_allclose(f, want, rtol=0, atol=2e-5 * np.abs(want).max())
    assert np.abs(Y.astype(int) - Y0.astype(int)).max() <= 1
    np.testing.assert_allclose(SY, SY0, rtol=1e-5)
    # statistics that differ from the tensor's own are used as given: y = (x - m) r gamma + beta
    m2 = (mean + 0.25).astype(np.float32)
    r2 = (rstd * 0.5).astype(np.float32)
    _, _, f2 = oracle.layernorm_q_stats(X, SX, gamma, beta, m2, r2, block)
    np.testing.assert_allclose(f2, (xd - m2[:, None].astype(np.float64)) * r2[:, None].astype(np.float64) * gamma + beta,
                               rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------------- Dropout (App. A)
def test_dropout_against_numpy_identity_zero_and_linearity():
    block, N, C, p = 32, 64, 96, 0.1
    g = workloads.rng(740)
    x = workloads.gaussian(g, N, C, 1.0)
    X, SX = oracle.quantize_block(x, block)
    xd = oracle.dequantize(X, SX, block)
    bits, keep = workloads.dropout_mask_bits(g, N, C, p)
    assert 0.8 < keep.mean() < 0.97
    Y, SY, f = oracle.dropout_q(X, SX, bits, p, block)
    # library arithmetic on the dequantized tensor; p is an FP32 number
    np.testing.assert_allclose(f, np.where(keep, xd / (1.0 - float(np.float32(p))), 0.0), rtol=1e-15, atol=0)
    q, s = oracle.quantize_block(f.astype(np.float32), block)
    np.testing.assert_array_equal(Y, q)
    np.testing.assert_array_equal(SY, s)
    # the bit order: dropping exactly column 9 zeroes exactly that column
    only9 = np.ones((N, C), bool)
    only9[:, 9] = False
    _, _, f9 = oracle.dropout_q(X, SX, np.packbits(only9, axis=1, bitorder="little"), 0.0, block)
    assert np.all(f9[:, 9] == 0) and np.array_equal(np.delete(f9, 9, axis=1), np.delete(xd, 9, axis=1))
    # p = 0 with everything kept is the identity on the codes; everything dropped gives zero codes and zero scales
    ones = np.full((N, C // 8), 255, np.uint8)
    Y1, SY1, _ = oracle.dropout_q(X, SX, ones, 0.0, block)
    np.testing.assert_array_equal(Y1, X)
    np.testing.assert_allclose(SY1, SX, rtol=2e-7)
    Y0, SY0, _ = oracle.dropout_q(X, SX, np.zeros((N, C // 8), np.uint8), p, block)
    assert not Y0.any() and not SY0.any()
    # the operator is linear in x, so it is its own backward: d/dx sum(w * Drop(x)) = Drop(w) element-wise
    assert 0.9 < f.sum() / (xd * keep).sum() * (1 - p) < 1.1
    with pytest.raises(ValueError):
        oracle.dropout_q(X, SX, bits, 1.0, block)
