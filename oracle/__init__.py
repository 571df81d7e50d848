"""CPU oracle of the per-block INT8 data flow (arxiv 2403.12422) -- test infrastructure.

A ctypes front-end over ``jetfire_oracle.c``.  Inputs and outputs are numpy
arrays in host memory.  Only tests, the smoke check and the benchmark's
CPU-baseline leg may import this package; the GPU library never does, and this
package imports nothing from the GPU package.

Function names follow the C-ABI of the GPU library without the ``jf_`` prefix.
Each function's docstring names the passage of the paper it follows; the
arithmetic itself lives in the C file.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB if os.path.exists(_build.LIB) and os.path.getmtime(_build.LIB) >= os.path.getmtime(
            _build.SRC) else _build.build()
        _lib = ctypes.CDLL(path)
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.int8, a.dtype
    return a


def _f32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, a.dtype
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc} (2 = shape not divisible by block)")


_I64 = ctypes.c_int64
_I32 = ctypes.c_int


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def set_threads(n: int) -> None:
    _load().oracle_set_threads(_I32(n))


def quantize_block(x, block=32):
    """Sec. 4, Eq. 1: per-block quantizer Q.  x: (rows, cols) float32 -> (codes int8, scales float32 grid)."""
    x = _f32(x)
    rows, cols = x.shape
    q = np.empty((rows, cols), np.int8)
    s = np.empty((rows // block, cols // block), np.float32)
    _check(_load().oracle_quantize_block(_p(x), _I64(rows), _I64(cols), _I32(block), _p(q), _p(s)), "quantize_block")
    return q, s


def dequantize(q, s, block=32):
    """Sec. 4, Eq. 1: dequantizer Q^-1 = code * scale, exact in float64."""
    q, s = _i8(q), _f32(s)
    rows, cols = q.shape
    out = np.empty((rows, cols), np.float64)
    _check(_load().oracle_dequantize(_p(q), _p(s), _I64(rows), _I64(cols), _I32(block), _p(out)), "dequantize")
    return out


def transpose(q, s, block=32):
    """Transpose of a per-block tensor (codes and scale grid), the operand reshaping of Sec. 4's backward products."""
    q, s = _i8(q), _f32(s)
    rows, cols = q.shape
    qT = np.empty((cols, rows), np.int8)
    sT = np.empty((cols // block, rows // block), np.float32)
    _check(_load().oracle_transpose(_p(q), _p(s), _I64(rows), _I64(cols), _I32(block), _p(qT), _p(sT)), "transpose")
    return qT, sT


def block_partials(A, Bm, block, kb):
    """Sec. 5.3: INT32 product A_{p,kb} Bm_{q,kb}^T of K-block kb for every output block; A (M,K), Bm (Nn,K)."""
    A, Bm = _i8(A), _i8(Bm)
    M, K = A.shape
    Nn, K2 = Bm.shape
    assert K == K2
    out = np.empty((M, Nn), np.int32)
    _check(_load().oracle_block_partials(_p(A), _p(Bm), _I64(M), _I64(Nn), _I64(K), _I32(block), _I64(kb), _p(out)),
           "block_partials")
    return out


def _linear(fn, a, sa, b, sb, out_shape, dims, block):
    q = np.empty(out_shape, np.int8)
    s = np.empty((out_shape[0] // block, out_shape[1] // block), np.float32)
    a32 = np.empty(out_shape, np.float32)
    a64 = np.empty(out_shape, np.float64)
    _check(fn(_p(a), _p(sa), _p(b), _p(sb), _I64(dims[0]), _I64(dims[1]), _I64(dims[2]), _I32(block), _p(q), _p(s),
              _p(a32), _p(a64)), "linear")
    return q, s, a32, a64


def linear_nt(A, SA, Bm, SB, block=32):
    """Alg. 1 in NT form out = A Bm^T.  Returns (codes, scales, FP32 accumulator, float64 accumulator)."""
    A, SA, Bm, SB = _i8(A), _f32(SA), _i8(Bm), _f32(SB)
    M, K = A.shape
    Nn = Bm.shape[0]
    assert Bm.shape[1] == K
    return _linear(_load().oracle_linear_nt, A, SA, Bm, SB, (M, Nn), (M, Nn, K), block)


def linear_nt_blocks(A, SA, Bm, SB, bp, bq, block=32):
    """Alg. 1 for the listed output blocks only; returns per-block tiles (nblk,B,B) and scales (nblk,)."""
    A, SA, Bm, SB = _i8(A), _f32(SA), _i8(Bm), _f32(SB)
    bp = np.ascontiguousarray(bp, dtype=np.int64)
    bq = np.ascontiguousarray(bq, dtype=np.int64)
    M, K = A.shape
    Nn = Bm.shape[0]
    n = bp.size
    q = np.empty((n, block, block), np.int8)
    s = np.empty((n,), np.float32)
    a32 = np.empty((n, block, block), np.float32)
    a64 = np.empty((n, block, block), np.float64)
    _check(_load().oracle_linear_nt_blocks(_p(A), _p(SA), _p(Bm), _p(SB), _I64(M), _I64(Nn), _I64(K), _I32(block),
                                           _p(bp), _p(bq), _I64(n), _p(q), _p(s), _p(a32), _p(a64)),
           "linear_nt_blocks")
    return q, s, a32, a64


def linear_fwd(X, SX, W, SW, block=32):
    """Sec. 4 / Alg. 1: Y = X W^T.  X (N,C), W (D,C) -> Y (N,D)."""
    X, SX, W, SW = _i8(X), _f32(SX), _i8(W), _f32(SW)
    N, C = X.shape
    D = W.shape[0]
    assert W.shape[1] == C
    return _linear(_load().oracle_linear_fwd, X, SX, W, SW, (N, D), (N, C, D), block)


def linear_dgrad(dY, SdY, W, SW, block=32):
    """Sec. 4: dX = dY W.  dY (N,D), W (D,C) -> dX (N,C)."""
    dY, SdY, W, SW = _i8(dY), _f32(SdY), _i8(W), _f32(SW)
    N, D = dY.shape
    C = W.shape[1]
    assert W.shape[0] == D
    return _linear(_load().oracle_linear_dgrad, dY, SdY, W, SW, (N, C), (N, C, D), block)


def linear_wgrad(dY, SdY, X, SX, block=32):
    """Sec. 4: dW = dY^T X.  dY (N,D), X (N,C) -> dW (D,C)."""
    dY, SdY, X, SX = _i8(dY), _f32(SdY), _i8(X), _f32(SX)
    N, D = dY.shape
    C = X.shape[1]
    assert X.shape[0] == N
    return _linear(_load().oracle_linear_wgrad, dY, SdY, X, SX, (D, C), (N, C, D), block)


def gelu_q(X, SX, block=32):
    """App. A + Alg. 2: INT8 GELU forward.  Returns (codes, scales, float64 pre-quantization values)."""
    X, SX = _i8(X), _f32(SX)
    N, C = X.shape
    Y = np.empty((N, C), np.int8)
    SY = np.empty((N // block, C // block), np.float32)
    yf = np.empty((N, C), np.float64)
    _check(_load().oracle_gelu_q(_p(X), _p(SX), _I64(N), _I64(C), _I32(block), _p(Y), _p(SY), _p(yf)), "gelu_q")
    return Y, SY, yf


def gelu_q_bwd(dY, SdY, X, SX, block=32):
    """App. A + Alg. 2: INT8 GELU backward dx = g * GELU'(x)."""
    dY, SdY, X, SX = _i8(dY), _f32(SdY), _i8(X), _f32(SX)
    N, C = X.shape
    dX = np.empty((N, C), np.int8)
    SdX = np.empty((N // block, C // block), np.float32)
    f = np.empty((N, C), np.float64)
    _check(_load().oracle_gelu_q_bwd(_p(dY), _p(SdY), _p(X), _p(SX), _I64(N), _I64(C), _I32(block), _p(dX), _p(SdX),
                                     _p(f)), "gelu_q_bwd")
    return dX, SdX, f


def layernorm_q(X, SX, gamma, beta, eps=1e-5, block=32):
    """App. A (LayerNorm) + Alg. 2.  Returns (codes, scales, mean, rstd, float64 pre-quantization values)."""
    X, SX, gamma, beta = _i8(X), _f32(SX), _f32(gamma), _f32(beta)
    N, C = X.shape
    Y = np.empty((N, C), np.int8)
    SY = np.empty((N // block, C // block), np.float32)
    mean = np.empty((N,), np.float32)
    rstd = np.empty((N,), np.float32)
    f = np.empty((N, C), np.float64)
    _check(_load().oracle_layernorm_q(_p(X), _p(SX), _p(gamma), _p(beta), ctypes.c_float(eps), _I64(N), _I64(C),
                                      _I32(block), _p(Y), _p(SY), _p(mean), _p(rstd), _p(f)), "layernorm_q")
    return Y, SY, mean, rstd, f


def layernorm_q_bwd(dY, SdY, X, SX, gamma, mean, rstd, block=32):
    """LayerNorm backward (standard gradient) + Alg. 2.  Returns (codes, scales, dgamma, dbeta, float64 dx)."""
    dY, SdY, X, SX = _i8(dY), _f32(SdY), _i8(X), _f32(SX)
    gamma, mean, rstd = _f32(gamma), _f32(mean), _f32(rstd)
    N, C = X.shape
    dX = np.empty((N, C), np.int8)
    SdX = np.empty((N // block, C // block), np.float32)
    dg = np.empty((C,), np.float32)
    db = np.empty((C,), np.float32)
    f = np.empty((N, C), np.float64)
    _check(_load().oracle_layernorm_q_bwd(_p(dY), _p(SdY), _p(X), _p(SX), _p(gamma), _p(mean), _p(rstd), _I64(N),
                                          _I64(C), _I32(block), _p(dX), _p(SdX), _p(dg), _p(db), _p(f)),
           "layernorm_q_bwd")
    return dX, SdX, dg, db, f


def add_q(X1, S1, X2, S2, block=32):
    """App. A (Add, with the row partials of the LayerNorm paragraph) + Alg. 2.

    Returns (codes, scales, row_mean (N, C/B), row_sumsq (N, C/B), float64 sum)."""
    X1, S1, X2, S2 = _i8(X1), _f32(S1), _i8(X2), _f32(S2)
    N, C = X1.shape
    assert X2.shape == (N, C)
    Y = np.empty((N, C), np.int8)
    SY = np.empty((N // block, C // block), np.float32)
    rm = np.empty((N, C // block), np.float32)
    rq = np.empty((N, C // block), np.float32)
    f = np.empty((N, C), np.float64)
    _check(_load().oracle_add_q(_p(X1), _p(S1), _p(X2), _p(S2), _I64(N), _I64(C), _I32(block), _p(Y), _p(SY), _p(rm),
                                _p(rq), _p(f)), "add_q")
    return Y, SY, rm, rq, f


def row_stats_from_partials(row_mean, row_sumsq, C, eps=1e-5, block=32):
    """App. A (LayerNorm paragraph): per-row mean and rstd from ADD's per-block row partials."""
    row_mean, row_sumsq = _f32(row_mean), _f32(row_sumsq)
    N = row_mean.shape[0]
    assert row_mean.shape == row_sumsq.shape == (N, C // block)
    mean = np.empty((N,), np.float32)
    rstd = np.empty((N,), np.float32)
    _check(_load().oracle_row_stats_from_partials(_p(row_mean), _p(row_sumsq), _I64(N), _I64(C), _I32(block),
                                                  ctypes.c_float(eps), _p(mean), _p(rstd)), "row_stats_from_partials")
    return mean, rstd


def layernorm_q_stats(X, SX, gamma, beta, mean, rstd, block=32):
    """App. A: LayerNorm from given row statistics + Alg. 2.  Returns (codes, scales, float64 pre-quantization values)."""
    X, SX, gamma, beta, mean, rstd = _i8(X), _f32(SX), _f32(gamma), _f32(beta), _f32(mean), _f32(rstd)
    N, C = X.shape
    Y = np.empty((N, C), np.int8)
    SY = np.empty((N // block, C // block), np.float32)
    f = np.empty((N, C), np.float64)
    _check(_load().oracle_layernorm_q_stats(_p(X), _p(SX), _p(gamma), _p(beta), _p(mean), _p(rstd), _I64(N), _I64(C),
                                            _I32(block), _p(Y), _p(SY), _p(f)), "layernorm_q_stats")
    return Y, SY, f


def dropout_q(X, SX, mask_bits, p, block=32):
    """App. A (Dropout) + Alg. 2: y = x * m / (1 - p); the backward pass is the same call on the gradient.

    mask_bits: (N, C/8) uint8, bit (c mod 8) of byte c/8 of a row belongs to column c.
    Returns (codes, scales, float64 pre-quantization values)."""
    X, SX = _i8(X), _f32(SX)
    mask_bits = np.ascontiguousarray(mask_bits)
    N, C = X.shape
    assert mask_bits.dtype == np.uint8 and mask_bits.shape == (N, C // 8)
    Y = np.empty((N, C), np.int8)
    SY = np.empty((N // block, C // block), np.float32)
    f = np.empty((N, C), np.float64)
    _check(_load().oracle_dropout_q(_p(X), _p(SX), _p(mask_bits), ctypes.c_float(p), _I64(N), _I64(C), _I32(block),
                                    _p(Y), _p(SY), _p(f)), "dropout_q")
    return Y, SY, f
