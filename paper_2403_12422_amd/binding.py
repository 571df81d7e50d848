"""ctypes binding of ``libjetfire.so``: same names as the C ABI, argument marshalling only.

torch is used for device memory and the current stream; nothing here computes.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libjetfire.so")
_lib = None

# name -> argument ctypes, in the order of include/jetfire.h
_P, _I64, _I32, _F32, _SZ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
_SIGNATURES = {
    "jf_last_hip_error": (_I32, []),
    "jf_error_string": (ctypes.c_char_p, [_I32]),
    "jf_workspace_bytes": (_SZ, [_I32, _I64, _I64, _I64, _I32]),
    "jf_quantize_block": (_I32, [_P, _I32, _I64, _I64, _I64, _I32, _P, _I64, _P, _P, _I64, _P, _P]),
    "jf_dequantize_block": (_I32, [_P, _P, _I64, _I64, _I32, _P, _I32, _I64, _P]),
    "jf_linear_fwd": (_I32, [_P, _P, _P, _P, _I64, _I64, _I64, _I32, _P, _P, _P, _P, _SZ, _P]),
    "jf_linear_dgrad": (_I32, [_P, _P, _P, _P, _I64, _I64, _I64, _I32, _P, _P, _P, _P, _SZ, _P]),
    "jf_linear_wgrad": (_I32, [_P, _P, _P, _P, _I64, _I64, _I64, _I32, _P, _P, _P, _P, _SZ, _P]),
    "jf_linear_bwd": (_I32, [_P, _P, _P, _P, _P, _P, _I64, _I64, _I64, _I32, _P, _P, _P, _P, _P, _P, _P, _SZ, _P]),
    "jf_gelu_q": (_I32, [_P, _P, _I64, _I64, _I32, _P, _P, _P]),
    "jf_gelu_q_bwd": (_I32, [_P, _P, _P, _P, _I64, _I64, _I32, _P, _P, _P]),
    "jf_layernorm_q": (_I32, [_P, _P, _P, _P, _F32, _I64, _I64, _I32, _P, _P, _P, _P, _P]),
    "jf_layernorm_q_partials": (_I32, [_P, _P, _P, _P, _P, _P, _F32, _I64, _I64, _I32, _P, _P, _P, _P, _P]),
    "jf_dropout_q": (_I32, [_P, _P, _P, _F32, _I64, _I64, _I32, _P, _P, _P]),
    "jf_add_q": (_I32, [_P, _P, _P, _P, _I64, _I64, _I32, _P, _P, _P, _P, _P]),
    "jf_layernorm_q_bwd": (_I32, [_P, _P, _P, _P, _P, _P, _P, _I64, _I64, _I32, _P, _P, _P, _P, _P, _SZ, _P]),
    "jf_layernorm_q_bwd_static": (_I32, [_P, _P, _P, _P, _P, _P, _P, _I64, _I64, _I32, _P, _P, _P, _P, _P]),
    "jf_debug_linear_partials": (_I32, [_I32, _P, _P, _I64, _I64, _I64, _I32, _I64, _P, _P]),
    "jf_debug_set_gemm_shape": (_I32, [_I32]),
}
EXPORTED_SYMBOLS = tuple(_SIGNATURES)

JF_OP_QUANTIZE, JF_OP_LINEAR_FWD, JF_OP_LINEAR_DGRAD, JF_OP_LINEAR_WGRAD = 0, 1, 2, 3
JF_OP_GELU, JF_OP_GELU_BWD, JF_OP_LAYERNORM, JF_OP_LAYERNORM_BWD = 4, 5, 6, 7


class JetfireError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(message)
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load the built shared object; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise JetfireError(-1, f"{_LIB_PATH} is missing: run `python -m paper_2403_12422_amd.build` "
                                   "(or __graft_entry__.build()) first; there is no CPU fallback")
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(code):
    if code != 0:
        lib = load_library()
        msg = lib.jf_error_string(code).decode()
        if code == 6:
            msg += f" (hip error {lib.jf_last_hip_error()})"
        raise JetfireError(code, msg)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev(t, dtype, ndim):
    if not t.is_cuda:
        raise JetfireError(-2, "tensors must live on the GPU; this library has no CPU path")
    if t.dtype != dtype or t.dim() != ndim or not t.is_contiguous():
        raise JetfireError(-2, f"expected contiguous {ndim}-d {dtype} tensor, got {t.dtype} {tuple(t.shape)}")
    return t


def jf_workspace_bytes(op, N, C, D, block):
    return int(load_library().jf_workspace_bytes(op, N, C, D, block))


def jf_quantize_block(x, block=32, transposed_copy=False, out=None):
    """x: (rows, cols) float32 or float16 CUDA tensor -> (q, s) or (q, s, qT, sT).

    `out` (here and in every function below) is an optional tuple of preallocated output tensors, in the
    order they are returned; without it the outputs are allocated with torch."""
    lib = load_library()
    if x.dtype not in (torch.float32, torch.float16):
        raise JetfireError(7, "source must be float32 or float16")
    _dev(x, x.dtype, 2)
    rows, cols = x.shape
    qT = sT = None
    if out is not None:
        q, s = out[0], out[1]
        if transposed_copy:
            qT, sT = out[2], out[3]
    else:
        q = torch.empty((rows, cols), dtype=torch.int8, device=x.device)
        s = torch.empty((max(rows // block, 0), max(cols // block, 0)), dtype=torch.float32, device=x.device)
    if transposed_copy and out is None:
        qT = torch.empty((cols, rows), dtype=torch.int8, device=x.device)
        sT = torch.empty((max(cols // block, 0), max(rows // block, 0)), dtype=torch.float32, device=x.device)
    _check(lib.jf_quantize_block(_ptr(x), 0 if x.dtype == torch.float32 else 1, rows, cols, cols, block, _ptr(q), cols,
                                 _ptr(s), _ptr(qT), rows, _ptr(sT), _stream()))
    return (q, s, qT, sT) if transposed_copy else (q, s)


def jf_dequantize_block(q, s, block=32, dtype=torch.float32, out=None):
    """(codes, scales) -> float32 or float16 tensor of code * scale."""
    _dev(q, torch.int8, 2), _dev(s, torch.float32, 2)
    if dtype not in (torch.float32, torch.float16):
        raise JetfireError(7, "output must be float32 or float16")
    rows, cols = q.shape
    if out is None:
        out = torch.empty((rows, cols), dtype=dtype, device=q.device)
    _check(load_library().jf_dequantize_block(_ptr(q), _ptr(s), rows, cols, block, _ptr(out),
                                              0 if dtype == torch.float32 else 1, cols, _stream()))
    return out


def _linear(fn, a, sa, b, sb, N, C, D, block, out_shape, want_q, want_f32, out=None):
    dev = a.device
    if out is not None:
        q, s, f = out
    else:
        q = torch.empty(out_shape, dtype=torch.int8, device=dev) if want_q else None
        s = torch.empty((out_shape[0] // block, out_shape[1] // block), dtype=torch.float32, device=dev) if want_q else None
        f = torch.empty(out_shape, dtype=torch.float32, device=dev) if want_f32 else None
    _check(fn(_ptr(a), _ptr(sa), _ptr(b), _ptr(sb), N, C, D, block, _ptr(q), _ptr(s), _ptr(f), None, 0, _stream()))
    return q, s, f


def jf_linear_fwd(X, SX, W, SW, block=32, want_f32=False, out=None):
    """Y = X W^T.  X (N,C) int8, W (D,C) int8 -> (Y int8 (N,D), SY, Y_f32 or None)."""
    _dev(X, torch.int8, 2), _dev(W, torch.int8, 2), _dev(SX, torch.float32, 2), _dev(SW, torch.float32, 2)
    N, C = X.shape
    D = W.shape[0]
    if W.shape[1] != C:
        raise JetfireError(2, "X and W disagree on C")
    return _linear(load_library().jf_linear_fwd, X, SX, W, SW, N, C, D, block, (N, D), True, want_f32, out)


def jf_linear_dgrad(dY, SdY, W, SW, block=32, want_f32=False, out=None):
    """dX = dY W.  dY (N,D) int8, W (D,C) int8 -> (dX int8 (N,C), SdX, dX_f32 or None)."""
    _dev(dY, torch.int8, 2), _dev(W, torch.int8, 2), _dev(SdY, torch.float32, 2), _dev(SW, torch.float32, 2)
    N, D = dY.shape
    C = W.shape[1]
    if W.shape[0] != D:
        raise JetfireError(2, "dY and W disagree on D")
    return _linear(load_library().jf_linear_dgrad, dY, SdY, W, SW, N, C, D, block, (N, C), True, want_f32, out)


def jf_linear_wgrad(dY, SdY, X, SX, block=32, want_q=True, want_f32=False, out=None):
    """dW = dY^T X.  dY (N,D) int8, X (N,C) int8 -> (dW int8 (D,C) or None, SdW or None, dW_f32 or None)."""
    _dev(dY, torch.int8, 2), _dev(X, torch.int8, 2), _dev(SdY, torch.float32, 2), _dev(SX, torch.float32, 2)
    N, D = dY.shape
    C = X.shape[1]
    if X.shape[0] != N:
        raise JetfireError(2, "dY and X disagree on N")
    return _linear(load_library().jf_linear_wgrad, dY, SdY, X, SX, N, C, D, block, (D, C), want_q, want_f32, out)


def jf_linear_bwd(dY, SdY, W, SW, X, SX, block=32, want_f32=False, out=None):
    """Both backward products in one call: returns ((dX, SdX, dX_f32 or None), (dW, SdW, dW_f32 or None)); `out` is the
    same pair of triples, preallocated."""
    for t in (dY, W, X):
        _dev(t, torch.int8, 2)
    for t in (SdY, SW, SX):
        _dev(t, torch.float32, 2)
    N, D = dY.shape
    C = W.shape[1]
    if W.shape[0] != D or tuple(X.shape) != (N, C):
        raise JetfireError(2, "dY, W and X disagree on N, C, D")
    dev = dY.device
    if out is not None:
        (dX, SdX, dXf), (dW, SdW, dWf) = out
    else:
        i8 = lambda r, c: torch.empty((r, c), dtype=torch.int8, device=dev)
        sc = lambda r, c: torch.empty((r // block, c // block), dtype=torch.float32, device=dev)
        f32 = lambda r, c: torch.empty((r, c), dtype=torch.float32, device=dev) if want_f32 else None
        dX, SdX, dXf, dW, SdW, dWf = i8(N, C), sc(N, C), f32(N, C), i8(D, C), sc(D, C), f32(D, C)
    _check(load_library().jf_linear_bwd(_ptr(dY), _ptr(SdY), _ptr(W), _ptr(SW), _ptr(X), _ptr(SX), N, C, D, block, _ptr(dX),
                                        _ptr(SdX), _ptr(dXf), _ptr(dW), _ptr(SdW), _ptr(dWf), None, 0, _stream()))
    return (dX, SdX, dXf), (dW, SdW, dWf)


def jf_gelu_q(X, SX, block=32, out=None):
    _dev(X, torch.int8, 2), _dev(SX, torch.float32, 2)
    N, C = X.shape
    Y, SY = out if out is not None else (torch.empty_like(X), torch.empty_like(SX))
    _check(load_library().jf_gelu_q(_ptr(X), _ptr(SX), N, C, block, _ptr(Y), _ptr(SY), _stream()))
    return Y, SY


def jf_gelu_q_bwd(dY, SdY, X, SX, block=32, out=None):
    _dev(X, torch.int8, 2), _dev(SX, torch.float32, 2), _dev(dY, torch.int8, 2), _dev(SdY, torch.float32, 2)
    N, C = X.shape
    if dY.shape != X.shape:
        raise JetfireError(2, "dY and X shapes differ")
    dX, SdX = out if out is not None else (torch.empty_like(X), torch.empty_like(SX))
    _check(load_library().jf_gelu_q_bwd(_ptr(dY), _ptr(SdY), _ptr(X), _ptr(SX), N, C, block, _ptr(dX), _ptr(SdX),
                                        _stream()))
    return dX, SdX


def jf_layernorm_q(X, SX, gamma, beta, eps=1e-5, block=32, out=None):
    _dev(X, torch.int8, 2), _dev(SX, torch.float32, 2), _dev(gamma, torch.float32, 1), _dev(beta, torch.float32, 1)
    N, C = X.shape
    if out is not None:
        Y, SY, mean, rstd = out
    else:
        Y = torch.empty_like(X)
        SY = torch.empty_like(SX)
        mean = torch.empty((N,), dtype=torch.float32, device=X.device)
        rstd = torch.empty((N,), dtype=torch.float32, device=X.device)
    _check(load_library().jf_layernorm_q(_ptr(X), _ptr(SX), _ptr(gamma), _ptr(beta), eps, N, C, block, _ptr(Y),
                                         _ptr(SY), _ptr(mean), _ptr(rstd), _stream()))
    return Y, SY, mean, rstd


def jf_layernorm_q_partials(X, SX, row_mean, row_sumsq, gamma, beta, eps=1e-5, block=32, out=None):
    """LayerNorm whose row statistics come from the row partials written by jf_add_q."""
    _dev(X, torch.int8, 2), _dev(SX, torch.float32, 2), _dev(gamma, torch.float32, 1), _dev(beta, torch.float32, 1)
    _dev(row_mean, torch.float32, 2), _dev(row_sumsq, torch.float32, 2)
    N, C = X.shape
    if tuple(row_mean.shape) != (C // block, N) or tuple(row_sumsq.shape) != (C // block, N):
        raise JetfireError(2, "row partials must be (C / block, N), as jf_add_q writes them")
    if out is not None:
        Y, SY, mean, rstd = out
    else:
        Y = torch.empty_like(X)
        SY = torch.empty_like(SX)
        mean = torch.empty((N,), dtype=torch.float32, device=X.device)
        rstd = torch.empty((N,), dtype=torch.float32, device=X.device)
    _check(load_library().jf_layernorm_q_partials(_ptr(X), _ptr(SX), _ptr(row_mean), _ptr(row_sumsq), _ptr(gamma),
                                                  _ptr(beta), eps, N, C, block, _ptr(Y), _ptr(SY), _ptr(mean),
                                                  _ptr(rstd), _stream()))
    return Y, SY, mean, rstd


def jf_dropout_q(X, SX, mask_bits, p, block=32, out=None):
    """Y = Q(X * m / (1 - p)); mask_bits (N, C/8) uint8, bit c % 8 of byte c // 8 of a row is column c's keep bit."""
    _dev(X, torch.int8, 2), _dev(SX, torch.float32, 2), _dev(mask_bits, torch.uint8, 2)
    N, C = X.shape
    if tuple(mask_bits.shape) != (N, C // 8):
        raise JetfireError(2, "mask_bits must be (N, C / 8)")
    Y, SY = out if out is not None else (torch.empty_like(X), torch.empty_like(SX))
    _check(load_library().jf_dropout_q(_ptr(X), _ptr(SX), _ptr(mask_bits), p, N, C, block, _ptr(Y), _ptr(SY), _stream()))
    return Y, SY


def jf_add_q(X1, S1, X2, S2, block=32, want_partials=False, out=None):
    """Y = Q(X1 + X2); with want_partials also the row partials (mean, sum of squares) of the sum, stored block column by
    block column: two (C/block, N) tensors."""
    _dev(X1, torch.int8, 2), _dev(S1, torch.float32, 2), _dev(X2, torch.int8, 2), _dev(S2, torch.float32, 2)
    N, C = X1.shape
    if X2.shape != X1.shape:
        raise JetfireError(2, "X1 and X2 shapes differ")
    rm = rq = None
    if out is not None:
        Y, SY = out[0], out[1]
        if want_partials:
            rm, rq = out[2], out[3]
    else:
        Y, SY = torch.empty_like(X1), torch.empty_like(S1)
        if want_partials:
            rm = torch.empty((C // block, N), dtype=torch.float32, device=X1.device)
            rq = torch.empty((C // block, N), dtype=torch.float32, device=X1.device)
    _check(load_library().jf_add_q(_ptr(X1), _ptr(S1), _ptr(X2), _ptr(S2), N, C, block, _ptr(Y), _ptr(SY), _ptr(rm),
                                   _ptr(rq), _stream()))
    return (Y, SY, rm, rq) if want_partials else (Y, SY)


def jf_layernorm_q_bwd(dY, SdY, X, SX, gamma, mean, rstd, block=32, workspace=None, out=None):
    _dev(X, torch.int8, 2), _dev(SX, torch.float32, 2), _dev(dY, torch.int8, 2), _dev(SdY, torch.float32, 2)
    _dev(gamma, torch.float32, 1), _dev(mean, torch.float32, 1), _dev(rstd, torch.float32, 1)
    N, C = X.shape
    if dY.shape != X.shape:
        raise JetfireError(2, "dY and X shapes differ")
    need = jf_workspace_bytes(JF_OP_LAYERNORM_BWD, N, C, 0, block)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=X.device)
    if out is not None:
        dX, SdX, dgamma, dbeta = out
    else:
        dX = torch.empty_like(X)
        SdX = torch.empty_like(SX)
        dgamma = torch.empty((C,), dtype=torch.float32, device=X.device)
        dbeta = torch.empty((C,), dtype=torch.float32, device=X.device)
    _check(load_library().jf_layernorm_q_bwd(_ptr(dY), _ptr(SdY), _ptr(X), _ptr(SX), _ptr(gamma), _ptr(mean),
                                             _ptr(rstd), N, C, block, _ptr(dX), _ptr(SdX), _ptr(dgamma), _ptr(dbeta),
                                             _ptr(workspace), workspace.numel(), _stream()))
    return dX, SdX, dgamma, dbeta


def jf_layernorm_q_bwd_static(dY, SdY, X, SX, gamma, mean, rstd, out, block=32):
    """jf_layernorm_q_bwd without a workspace: the library's static device scratch holds the partial sums, and
    nothing is allocated -- `out` = (dX, SdX, dgamma, dbeta), preallocated, is therefore required."""
    _dev(X, torch.int8, 2), _dev(SX, torch.float32, 2), _dev(dY, torch.int8, 2), _dev(SdY, torch.float32, 2)
    _dev(gamma, torch.float32, 1), _dev(mean, torch.float32, 1), _dev(rstd, torch.float32, 1)
    N, C = X.shape
    if dY.shape != X.shape:
        raise JetfireError(2, "dY and X shapes differ")
    dX, SdX, dgamma, dbeta = out
    _dev(dX, torch.int8, 2), _dev(SdX, torch.float32, 2), _dev(dgamma, torch.float32, 1), _dev(dbeta, torch.float32, 1)
    _check(load_library().jf_layernorm_q_bwd_static(_ptr(dY), _ptr(SdY), _ptr(X), _ptr(SX), _ptr(gamma), _ptr(mean),
                                                    _ptr(rstd), N, C, block, _ptr(dX), _ptr(SdX), _ptr(dgamma),
                                                    _ptr(dbeta), _stream()))
    return dX, SdX, dgamma, dbeta


def jf_debug_linear_partials(which, A, Bm, N, C, D, block, kb):
    """INT32 product of K-block kb (test hook); which: 0 fwd, 1 dgrad, 2 wgrad."""
    _dev(A, torch.int8, 2), _dev(Bm, torch.int8, 2)
    shape = {0: (N, D), 1: (N, C), 2: (D, C)}[which]
    out = torch.empty(shape, dtype=torch.int32, device=A.device)
    _check(load_library().jf_debug_linear_partials(which, _ptr(A), _ptr(Bm), N, C, D, block, kb, _ptr(out), _stream()))
    return out


def jf_debug_set_gemm_shape(shape):
    """Test hook: 0 automatic, 1 128x128, 4 64x64, 6 256x128, 7 64x64 with a deep stage, 8 128x64."""
    _check(load_library().jf_debug_set_gemm_shape(shape))
