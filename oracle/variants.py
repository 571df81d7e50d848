"""Other scale shapes of Sec. 4 (per-tensor, per-token, per-channel), as plain numpy, for the quantization-error
comparison of Sec. 7.3 -- test infrastructure like the rest of this package; no GPU counterpart.

Each function quantizes with the same symmetric max-abs / 127 scale and round-half-to-even as Eq. 1, only the set
of elements that share a scale differs, and returns the dequantized tensor in float64.
"""
import numpy as np


def _qdq(x, amax):
    x = np.asarray(x, np.float32)
    s = (amax.astype(np.float32) / np.float32(127)).astype(np.float32)
    safe = np.where(s > 0, s, np.float32(1)).astype(np.float64)
    q = np.clip(np.rint(x.astype(np.float64) / safe), -127, 127)
    return np.where(s > 0, q * s.astype(np.float64), 0.0)


def per_tensor(x):
    """One scale for the whole matrix."""
    return _qdq(x, np.abs(x).max(keepdims=True))


def per_token(x):
    """One scale per row (token)."""
    return _qdq(x, np.abs(x).max(axis=1, keepdims=True))


def per_channel(x):
    """One scale per column (channel)."""
    return _qdq(x, np.abs(x).max(axis=0, keepdims=True))
