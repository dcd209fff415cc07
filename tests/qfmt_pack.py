"""Test-side packers of the weight formats beside Q4_K, written from the layout text alone.

Independent of both the oracle and the HIP path: tests build tensors field by field and know every
dequantised value in advance (exact rational arithmetic on the fields).

Layout (version 1): every field of a tensor is a plane of its own, planes follow one another without
padding, blocks inside a plane are in row-major order.  n = rows * cols / 256 super-blocks.
Quant bits of q5_k / q6_k sit in 32-bit words, weight t always in byte t%4 of its word:
  low 4 bits: word t//8, low nibble when t%8 < 4 else high nibble;
  bits 4..5 (q6_k): word t//16, bits 2g, 2g+1 with g = (t%16)//4;   bit 4 (q5_k): word t//32, bit g = (t%32)//4.
  q5_k: [n][16] header (binary16 d, dmin, then a 96-bit little-endian stream of sixteen 6-bit fields:
        sc_0..7, m_0..7) | [n][128] low 4 bits | [n][32] bit 4.        w = d*sc_s*q - dmin*m_s, s = t//32
  q6_k: [n][128] low 4 bits | [n][64] bits 4..5 | [n][16] int8 sub-scales (s = t//16) | [n] binary16 d.
                                                                       w = d*sc_s*(q-32)
  q8_0: [rows*cols] int8 | [rows*cols/32] binary16 d.          w = d*q
  f16 / f32: row-major numbers.
Fields are given as integer arrays shaped [rows, nb, ...]; half values as uint16 bit patterns.
"""
from fractions import Fraction

import numpy as np

from q4k_pack import half_fraction


def _words(bits, per_word, width):
    """bits [..., 256] -> bytes [..., 256 // per_word * 4]: weight t goes to byte t%4 of word t//per_word,
    at bit position width * ((t % per_word) // 4)."""
    b = np.asarray(bits, dtype=np.uint8)
    g = b.reshape(b.shape[:-1] + (256 // per_word, per_word // 4, 4))       # [word][position g][byte j]
    out = np.zeros(b.shape[:-1] + (256 // per_word, 4), dtype=np.uint8)
    for pos in range(per_word // 4):
        out |= (g[..., pos, :] << (width * pos)).astype(np.uint8)
    return out.reshape(b.shape[:-1] + (-1,))


def _nibbles(q_lo):
    return _words(q_lo, 8, 4)


def pack_q5k(d_bits, dmin_bits, sc, m, q):
    """d_bits, dmin_bits [rows, nb]; sc, m [rows, nb, 8] in 0..63; q [rows, nb, 256] in 0..31."""
    q = np.asarray(q)
    rows, nb, _ = q.shape
    hdr = np.zeros((rows, nb, 16), dtype=np.uint8)
    for r in range(rows):
        for b in range(nb):
            stream = 0
            for i, f in enumerate(list(sc[r][b]) + list(m[r][b])):
                assert 0 <= int(f) < 64
                stream |= int(f) << (6 * i)
            hdr[r, b] = np.frombuffer(int(d_bits[r][b]).to_bytes(2, "little") + int(dmin_bits[r][b]).to_bytes(2, "little")
                                      + stream.to_bytes(12, "little"), dtype=np.uint8)
    lo = _nibbles(q & 15)
    hi = _words((q >> 4) & 1, 32, 1)
    return np.concatenate([hdr.reshape(-1), lo.reshape(-1), hi.reshape(-1)])


def pack_q6k(d_bits, sc, q):
    """d_bits [rows, nb]; sc [rows, nb, 16] in -128..127; q [rows, nb, 256] in 0..63."""
    q = np.asarray(q)
    lo = _nibbles(q & 15)
    hi = _words((q >> 4) & 3, 16, 2)
    scb = np.asarray(sc, dtype=np.int8).view(np.uint8)
    db = np.asarray(d_bits, dtype="<u2").view(np.uint8)
    return np.concatenate([lo.reshape(-1), hi.reshape(-1), scb.reshape(-1), db.reshape(-1)])


def pack_q80(d_bits, q):
    """d_bits [rows, cols/32]; q [rows, cols] in -128..127."""
    return np.concatenate([np.asarray(q, dtype=np.int8).view(np.uint8).reshape(-1), np.asarray(d_bits, dtype="<u2").view(np.uint8).reshape(-1)])


def exact_q5k(d_bits, dmin_bits, sc, m, q):
    return half_fraction(int(d_bits)) * int(sc) * int(q) - half_fraction(int(dmin_bits)) * int(m)


def exact_q6k(d_bits, sc, q):
    return half_fraction(int(d_bits)) * int(sc) * (int(q) - 32)


def exact_q80(d_bits, q):
    return half_fraction(int(d_bits)) * int(q)
