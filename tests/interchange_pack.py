"""Test-side packers for quantised blocks in GGUF block order, written from the layout text alone
(oracle/interchange.py's docstring), one weight at a time.  Independent of the oracle's reader and of the HIP path.

Fields are plain Python / numpy integers; binary16 numbers are given as uint16 bit patterns.
"""
from fractions import Fraction

import numpy as np

from q4k_pack import half_fraction


def _put_scales(sc, m):
    """six-bit sc_0..7, m_0..7 -> the 12 bytes"""
    s = [0] * 12
    for j in range(8):
        a, b = int(sc[j]), int(m[j])
        assert 0 <= a < 64 and 0 <= b < 64
        if j < 4:
            s[j] |= a
            s[j + 4] |= b
        else:
            s[j + 4] |= (a & 15) | ((b & 15) << 4)
            s[j - 4] |= (a >> 4) << 6
            s[j] |= (b >> 4) << 6
    return s


def _put_low4(q):
    """256 quants -> the 128 bytes holding their low four bits (q4_k / q5_k)"""
    qs = [0] * 128
    for t in range(256):
        c, l = t // 64, t % 32
        v = int(q[t]) & 15
        qs[32 * c + l] |= v if t % 64 < 32 else v << 4
    return qs


def block_q4k(d_bits, dmin_bits, sc, m, q):
    assert all(0 <= int(v) < 16 for v in q)
    b = [d_bits & 255, d_bits >> 8, dmin_bits & 255, dmin_bits >> 8] + _put_scales(sc, m) + _put_low4(q)
    assert len(b) == 144
    return bytes(b)


def block_q5k(d_bits, dmin_bits, sc, m, q):
    assert all(0 <= int(v) < 32 for v in q)
    qh = [0] * 32
    for t in range(256):
        c, l = t // 64, t % 32
        if int(q[t]) & 16:
            qh[l] |= 1 << (2 * c + (1 if t % 64 >= 32 else 0))
    b = [d_bits & 255, d_bits >> 8, dmin_bits & 255, dmin_bits >> 8] + _put_scales(sc, m) + qh + _put_low4(q)
    assert len(b) == 176
    return bytes(b)


def block_q6k(d_bits, sc, q):
    """sc: 16 signed bytes; q: 256 values in 0..63"""
    ql, qh = [0] * 128, [0] * 64
    for t in range(256):
        v = int(q[t])
        assert 0 <= v < 64
        h, k, l = t // 128, (t % 128) // 32, t % 32
        ql[64 * h + 32 * (k & 1) + l] |= (v & 15) if k < 2 else (v & 15) << 4
        qh[32 * h + l] |= (v >> 4) << (2 * k)
    b = ql + qh + [int(s) & 255 for s in sc] + [d_bits & 255, d_bits >> 8]
    assert len(b) == 210
    return bytes(b)


def block_q80(d_bits, q):
    b = [d_bits & 255, d_bits >> 8] + [int(v) & 255 for v in q]
    assert len(b) == 34
    return bytes(b)


# exact values of the weights (Fractions), from the fields
def values_k(d_bits, dmin_bits, sc, m, q):
    d, dmin = half_fraction(d_bits), half_fraction(dmin_bits)
    return [d * int(sc[t // 32]) * int(q[t]) - dmin * int(m[t // 32]) for t in range(256)]


def values_q6k(d_bits, sc, q):
    d = half_fraction(d_bits)
    return [d * int(sc[t // 16]) * (int(q[t]) - 32) for t in range(256)]


def values_q80(d_bits, q):
    d = half_fraction(d_bits)
    return [d * int(v) for v in q]


def random_tensor(fmt, n_rows, n_cols, seed):
    """bytes of a tensor in GGUF block order with random fields, and the fields' exact values as float64 [n_rows, n_cols]
    (every value here is a ratio of small integers and a binary16 number: exact in float64)."""
    rng = np.random.default_rng(seed)
    per = 32 if fmt == "q8_0" else 256
    out, vals = [], []
    half = lambda: int(np.float16(rng.uniform(1e-3, 4e-3)).view(np.uint16))
    for _ in range(n_rows * (n_cols // per)):
        if fmt in ("q4_k", "q5_k"):
            d, dm = half(), half()
            sc, m = rng.integers(0, 64, 8), rng.integers(0, 64, 8)
            q = rng.integers(0, 16 if fmt == "q4_k" else 32, 256)
            out.append((block_q4k if fmt == "q4_k" else block_q5k)(d, dm, sc, m, q))
            vals.extend(values_k(d, dm, sc, m, q))
        elif fmt == "q6_k":
            d, sc, q = half(), rng.integers(-128, 128, 16), rng.integers(0, 64, 256)
            out.append(block_q6k(d, sc, q))
            vals.extend(values_q6k(d, sc, q))
        elif fmt == "q8_0":
            d, q = half(), rng.integers(-128, 128, 32)
            out.append(block_q80(d, q))
            vals.extend(values_q80(d, q))
        else:
            raise ValueError(fmt)
    v = np.array([float(x) for x in vals], dtype=np.float64).reshape(n_rows, n_cols)
    return np.frombuffer(b"".join(out), dtype=np.uint8).copy(), v
