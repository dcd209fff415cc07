"""Test-side packer / unpacker of Q4_K super-blocks, written from the layout text alone.

Independent of both the oracle and the HIP path: it exists so that tests can build
super-blocks field by field and know every dequantised value in advance.

Layout (144 bytes): bytes 0-1 d (binary16 LE), 2-3 dmin, 4-15 a 96-bit little-endian
bit stream of sixteen 6-bit fields (field i at stream bits [6i, 6i+6); 0-7 sub-scales,
8-15 sub-mins), 16-143 quants (weight t in byte 16 + t//2, low nibble when t is even).
"""
from fractions import Fraction

import numpy as np


def pack_block(d_bits, dmin_bits, sc, m, q):
    assert len(sc) == 8 and len(m) == 8 and len(q) == 256
    out = bytearray(144)
    out[0:2] = int(d_bits).to_bytes(2, "little")
    out[2:4] = int(dmin_bits).to_bytes(2, "little")
    stream = 0
    for i, f in enumerate(list(sc) + list(m)):
        assert 0 <= int(f) < 64
        stream |= int(f) << (6 * i)
    out[4:16] = stream.to_bytes(12, "little")
    for t in range(256):
        assert 0 <= int(q[t]) < 16
        out[16 + t // 2] |= int(q[t]) << (4 * (t & 1))
    return np.frombuffer(bytes(out), dtype=np.uint8).copy()


def unpack_block(blk):
    b = bytes(np.asarray(blk, dtype=np.uint8))
    d_bits = int.from_bytes(b[0:2], "little")
    dmin_bits = int.from_bytes(b[2:4], "little")
    stream = int.from_bytes(b[4:16], "little")
    f = [(stream >> (6 * i)) & 63 for i in range(16)]
    q = [(b[16 + t // 2] >> (4 * (t & 1))) & 15 for t in range(256)]
    return d_bits, dmin_bits, f[:8], f[8:], q


def half_bits(x):
    return int(np.array(x, dtype=np.float16).view(np.uint16))


def half_fraction(bits):
    """Exact rational value of a finite binary16 bit pattern."""
    sign = -1 if bits >> 15 else 1
    ex = (bits >> 10) & 31
    man = bits & 1023
    assert ex != 31
    if ex == 0:
        return sign * Fraction(man, 1 << 24)
    return sign * Fraction(1024 + man, 1024) * (Fraction(2) ** (ex - 15))


def exact_weight(d_bits, dmin_bits, sc, m, q):
    """Exact rational d*sc*q - dmin*m."""
    return half_fraction(d_bits) * sc * q - half_fraction(dmin_bits) * m


def fraction_to_f32(fr):
    """Nearest-even fp32 of a rational whose exact value fits in the fp64 significand."""
    v = float(fr)
    assert Fraction(v) == fr, "rational not exactly representable in fp64"
    return np.float32(v)


def dense_from_blocks(W):
    """Second, independent dequantisation loop -> float64 [rows, cols] of the *fp32-rounded* weights."""
    W = np.asarray(W, dtype=np.uint8)
    rows, nb, _ = W.shape
    out = np.zeros((rows, nb * 256), dtype=np.float64)
    for r in range(rows):
        for b in range(nb):
            d_bits, dmin_bits, sc, m, q = unpack_block(W[r, b])
            d = np.float32(np.array(d_bits, dtype=np.uint16).view(np.float16))
            dm = np.float32(np.array(dmin_bits, dtype=np.uint16).view(np.float16))
            for t in range(256):
                s = t // 32
                out[r, b * 256 + t] = np.float32(np.float32(np.float32(d * np.float32(sc[s])) * np.float32(q[t]))
                                                 - np.float32(dm * np.float32(m[s])))
    return out
