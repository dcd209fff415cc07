"""The layout text of include/prima.h for Q5_K and Q6_K, taken at its word.

A caller packs tensors from the public header, so the header's wording is packed here byte by byte with
plain loops (a third packer, sharing nothing with tests/qfmt_pack.py's reshapes or the oracle's C) and the
oracle must decode every weight to the exact value the header's rule gives.  The sentences this file
follows are asserted to be present in the header, so that the two cannot drift apart silently.
"""
import os
import re

import numpy as np

import oracle
from q4k_pack import fraction_to_f32, half_fraction

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _header_text():
    with open(os.path.join(ROOT, "include", "prima.h")) as f:
        return re.sub(r"[\s*]+", " ", f.read())


def test_the_header_says_what_this_file_packs():
    text = _header_text()
    for sentence in (
        "weight t (0..255 inside its super-block) always sits in byte t%4 of its word",
        "low 4 bits (Q5_K, Q6_K): word t/8 (128 bytes per super-block); the low nibble of byte t%4 when t%8 < 4, the high nibble when t%8 >= 4",
        "bits 4..5 (Q6_K): word t/16 (64 bytes); bits 2g and 2g+1 of byte t%4, g = (t%16)/4",
        "bit 4 (Q5_K): word t/32 (32 bytes); bit g of byte t%4, g = (t%32)/4",
        "Q5_K [n][16]: d, dmin (binary16, little endian), then sixteen 6-bit fields sc_0..7, m_0..7 as a 96-bit little-endian stream",
        "| [n][128]: the low 4 bits | [n][32]: bit 4. q = low + 16 bit4 in 0..31; w = d sc_s q - dmin m_s, s = t/32",
        "Q6_K [n][128]: the low 4 bits | [n][64]: bits 4..5 | [n][16]: signed bytes sc_s, s = t/16 | [n]: d (binary16, little endian). q = low + 16 bits45 in 0..63; w = d sc_s (q - 32)",
        "blocks inside a plane are in row-major order (row r, block b -> r n_cols / block + b)",
    ):
        assert sentence in text, sentence


def _put_low4(plane, block, t, low):
    """low 4 bits: word t/8 of the block's 128 bytes, byte t%4, low nibble when t%8 < 4"""
    at = block * 128 + 4 * (t // 8) + t % 4
    plane[at] |= low if t % 8 < 4 else low << 4


def pack_q5k_from_header(rows, nb, d_bits, dmin_bits, sc, m, q):
    n = rows * nb
    hdr, lo, hi = bytearray(16 * n), bytearray(128 * n), bytearray(32 * n)
    for r in range(rows):
        for b in range(nb):
            blk = r * nb + b                       # row-major blocks inside a plane
            stream = 0
            for i in range(8):
                stream |= int(sc[r][b][i]) << (6 * i)
                stream |= int(m[r][b][i]) << (6 * (8 + i))
            hdr[16 * blk:16 * blk + 16] = (int(d_bits[r][b]).to_bytes(2, "little") + int(dmin_bits[r][b]).to_bytes(2, "little")
                                          + stream.to_bytes(12, "little"))
            for t in range(256):
                v = int(q[r][b][t])
                _put_low4(lo, blk, t, v & 15)
                g = (t % 32) // 4                  # bit 4: word t/32 of 32 bytes, bit g of byte t%4
                hi[blk * 32 + 4 * (t // 32) + t % 4] |= ((v >> 4) & 1) << g
    return np.frombuffer(bytes(hdr + lo + hi), dtype=np.uint8).copy()


def pack_q6k_from_header(rows, nb, d_bits, sc, q):
    n = rows * nb
    lo, hi, scb, db = bytearray(128 * n), bytearray(64 * n), bytearray(16 * n), bytearray(2 * n)
    for r in range(rows):
        for b in range(nb):
            blk = r * nb + b
            for t in range(256):
                v = int(q[r][b][t])
                _put_low4(lo, blk, t, v & 15)
                g = (t % 16) // 4                  # bits 4..5: word t/16 of 64 bytes, bits 2g, 2g+1 of byte t%4
                hi[blk * 64 + 4 * (t // 16) + t % 4] |= ((v >> 4) & 3) << (2 * g)
            for s in range(16):
                scb[blk * 16 + s] = int(sc[r][b][s]) & 0xFF
            db[2 * blk:2 * blk + 2] = int(d_bits[r][b]).to_bytes(2, "little")
    return np.frombuffer(bytes(lo + hi + scb + db), dtype=np.uint8).copy()


def _half_bits(rng, shape):
    return ((rng.integers(0, 2, shape) << 15) | (rng.integers(5, 21, shape) << 10) | rng.integers(0, 1024, shape)).astype(np.uint16)


def test_q5k_packed_from_the_header_decodes_to_the_header_rule():
    rng = np.random.default_rng(2504)
    rows, nb = 3, 2
    d, dm = _half_bits(rng, (rows, nb)) & 0x7FFF, _half_bits(rng, (rows, nb)) & 0x7FFF
    sc, m = rng.integers(0, 64, (rows, nb, 8)), rng.integers(0, 64, (rows, nb, 8))
    q = rng.integers(0, 32, (rows, nb, 256))
    W = pack_q5k_from_header(rows, nb, d, dm, sc, m, q)
    assert W.size == oracle.fmt_tensor_bytes("q5_k", rows, nb * 256)
    w = oracle.fmt_dequant("q5_k", W, rows, nb * 256)
    for r in range(rows):
        for b in range(nb):
            for t in range(256):
                s = t // 32
                exact = half_fraction(int(d[r, b])) * int(sc[r, b, s]) * int(q[r, b, t]) - half_fraction(int(dm[r, b])) * int(m[r, b, s])
                assert w[r, b * 256 + t] == fraction_to_f32(exact), (r, b, t)


def test_q6k_packed_from_the_header_decodes_to_the_header_rule():
    rng = np.random.default_rng(8791)
    rows, nb = 3, 2
    d = _half_bits(rng, (rows, nb))
    sc = rng.integers(-128, 128, (rows, nb, 16))
    q = rng.integers(0, 64, (rows, nb, 256))
    W = pack_q6k_from_header(rows, nb, d, sc, q)
    assert W.size == oracle.fmt_tensor_bytes("q6_k", rows, nb * 256)
    w = oracle.fmt_dequant("q6_k", W, rows, nb * 256)
    for r in range(rows):
        for b in range(nb):
            for t in range(256):
                exact = half_fraction(int(d[r, b])) * int(sc[r, b, t // 16]) * (int(q[r, b, t]) - 32)
                assert w[r, b * 256 + t] == fraction_to_f32(exact), (r, b, t)


def test_the_header_packer_and_the_test_packer_agree_byte_for_byte():
    import qfmt_pack as fp
    rng = np.random.default_rng(7)
    rows, nb = 2, 3
    d, dm = _half_bits(rng, (rows, nb)) & 0x7FFF, _half_bits(rng, (rows, nb)) & 0x7FFF
    sc, m = rng.integers(0, 64, (rows, nb, 8)), rng.integers(0, 64, (rows, nb, 8))
    q5 = rng.integers(0, 32, (rows, nb, 256))
    assert np.array_equal(pack_q5k_from_header(rows, nb, d, dm, sc, m, q5), fp.pack_q5k(d, dm, sc, m, q5))
    sc6 = rng.integers(-128, 128, (rows, nb, 16))
    q6 = rng.integers(0, 64, (rows, nb, 256))
    assert np.array_equal(pack_q6k_from_header(rows, nb, d, sc6, q6), fp.pack_q6k(d, sc6, q6))
