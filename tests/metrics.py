"""Error metrics used by the parity tests."""
import numpy as np


def rel_err(y, r):
    """max_i |y_i - r_i| / max(|r_i|, rms(r)) per token vector (rows), worst row returned.

    Elements much smaller than the vector's RMS are judged at the vector's scale, and a vector
    that lies entirely below what an fp32 output can hold (|r| < 1e-30) is judged at that scale.
    """
    y = np.atleast_2d(np.asarray(y, dtype=np.float64))
    r = np.atleast_2d(np.asarray(r, dtype=np.float64))
    assert y.shape == r.shape
    y = y.reshape(y.shape[0], -1)
    r = r.reshape(r.shape[0], -1)
    rms = np.sqrt((r ** 2).mean(axis=1, keepdims=True))
    den = np.maximum(np.abs(r), np.maximum(rms, 1e-30))
    return float((np.abs(y - r) / den).max())


def max_rel_err(y, r):
    """max_i |y_i - r_i| / max_i |r_i| over the whole array."""
    y = np.asarray(y, dtype=np.float64)
    r = np.asarray(r, dtype=np.float64)
    return float(np.abs(y - r).max() / max(np.abs(r).max(), 1e-300))
