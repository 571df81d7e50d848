"""Comparison rules shared by the GPU parity tests.

Tolerances (from the benchmark spec of this build):
  * INT32 block partial sums: bit-exact;
  * re-quantized INT8 codes: identical except +-1 at rounding ties on at most 0.1 % of the elements;
  * scales and FP32 outputs: 1e-5 relative (FP32 outputs relative to the max-abs of their quantization block,
    which is what the quantizer sees; element-wise relative error is meaningless where the sum cancels);
  * column sums (dgamma, dbeta of LayerNorm backward): FP32 sums of N signed terms, 1e-5 relative to the sum of
    the terms' magnitudes -- the one rule for them in every test.
"""
import numpy as np

CODE_MISMATCH_FRACTION = 1e-3
REL_TOL = 1e-5


def block_amax(a, block):
    r, c = a.shape
    return np.abs(a).reshape(r // block, block, c // block, block).max(axis=(1, 3))


def expand(grid, block):
    return np.kron(grid, np.ones((block, block), grid.dtype))


def assert_scales_close(got, want, what=""):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - want)
    assert np.all(err <= REL_TOL * np.abs(want)), f"{what}: scale rel err {np.max(err / np.maximum(np.abs(want), 1e-300)):.3e}"
    assert np.all((want == 0) == (got == 0)), f"{what}: zero-scale blocks differ"


def assert_codes_close(got, want, what="", prequant=None, scales=None, block=None):
    """got/want int8 arrays.  If the oracle's pre-quantization values and scales are given, every
    mismatch must also sit at a rounding tie of value/scale (within 2e-3 of a half-integer)."""
    got = np.asarray(got).astype(np.int16)
    want = np.asarray(want).astype(np.int16)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    diff = np.abs(got - want)
    nbad = int(np.count_nonzero(diff))
    assert diff.max(initial=0) <= 1, f"{what}: code differs by {diff.max()}"
    assert nbad <= CODE_MISMATCH_FRACTION * diff.size, f"{what}: {nbad}/{diff.size} codes differ"
    if nbad and prequant is not None:
        s = expand(np.asarray(scales, np.float64), block) if block else np.asarray(scales, np.float64)
        idx = np.nonzero(diff)
        ratio = np.asarray(prequant, np.float64)[idx] / s[idx]
        dist = np.abs(np.abs(ratio - np.floor(ratio)) - 0.5)
        assert np.all(dist < 2e-3), f"{what}: a mismatching code is not at a rounding tie (distance {dist.max():.3e})"
    return nbad


def assert_f32_close(got, want64, block, what=""):
    """FP32 accumulator against the float64 oracle value, relative to the block's max-abs."""
    got = np.asarray(got, np.float64)
    want64 = np.asarray(want64, np.float64)
    amax = expand(block_amax(want64, block), block)
    err = np.abs(got - want64)
    ok = err <= REL_TOL * amax
    assert np.all(ok), f"{what}: max err/amax {np.max(err / np.maximum(amax, 1e-300)):.3e}"
    big = (np.abs(want64) >= 1e-2 * amax) & (amax > 0)
    rel = err[big] / np.abs(want64[big])
    assert rel.size == 0 or rel.max() <= 1e-3, f"{what}: element-wise rel err {rel.max():.3e}"


def assert_layernorm_param_grads_close(dgamma, dbeta, want_dgamma, want_dbeta, g64, xhat64, what=""):
    """dgamma = sum_N g * xhat and dbeta = sum_N g against the oracle's double sums: within REL_TOL of the sum of
    the magnitudes of the terms (g64, xhat64: the dequantized upstream gradient and the normalised input)."""
    tol_g = REL_TOL * np.abs(g64 * xhat64).sum(axis=0) + 1e-30
    tol_b = REL_TOL * np.abs(g64).sum(axis=0) + 1e-30
    err_g = np.abs(np.asarray(dgamma, np.float64) - want_dgamma)
    err_b = np.abs(np.asarray(dbeta, np.float64) - want_dbeta)
    assert np.all(err_g <= tol_g), f"{what}: dgamma error / tolerance {np.max(err_g / tol_g):.3f}"
    assert np.all(err_b <= tol_b), f"{what}: dbeta error / tolerance {np.max(err_b / tol_b):.3f}"
