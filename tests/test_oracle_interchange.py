"""Pins of the oracle's reading of tensors in GGUF block order (oracle/interchange.py).

The block formats are restated from their public description; there is no real file and no specification in reach,
so agreement with real checkpoints is PARITY UNPINNED.  What is pinned: the arithmetic and the placement as
described, by a packer written separately from the same text (tests/interchange_pack.py), values known by mental
arithmetic, every weight position and every field distinguishable, exact rationals, bits per weight."""
import os
import sys
from fractions import Fraction

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
from oracle import interchange as ix
import interchange_pack as ip
from q4k_pack import fraction_to_f32, half_bits


def _u8(b):
    return np.frombuffer(b, dtype=np.uint8)


def test_bits_per_weight():
    for fmt, bits in [("q4_k", 4.5), ("q5_k", 5.5), ("q6_k", 6.5625), ("q8_0", 8.5), ("f16", 16), ("f32", 32)]:
        assert ix.tensor_bytes(fmt, 6, 1024) * 8 == bits * 6 * 1024


def test_q4k_by_hand():
    # d = 2, dmin = 1; sub-block s: sc = s + 1, m = 2 s; quant t = t % 16
    sc, m = [s + 1 for s in range(8)], [2 * s for s in range(8)]
    q = [t % 16 for t in range(256)]
    w = ix.dequant("q4_k", _u8(ip.block_q4k(half_bits(2.0), half_bits(1.0), sc, m, q)), 1, 256)[0]
    for t in (0, 1, 15, 31, 32, 47, 63, 64, 100, 255):
        s = t // 32
        assert w[t] == 2.0 * (s + 1) * (t % 16) - 2 * s, t


def test_six_bit_fields_all_values_all_slots():
    # every slot (sc_j, m_j) takes every value 0..63 while the others hold a different pattern: the slot alone moves
    base_sc, base_m = [(7 * j + 3) % 64 for j in range(8)], [(11 * j + 5) % 64 for j in range(8)]
    q = [1] * 256
    for j in range(8):
        for v in (0, 1, 15, 16, 31, 32, 47, 48, 63):
            for which in ("sc", "m"):
                sc, m = list(base_sc), list(base_m)
                (sc if which == "sc" else m)[j] = v
                w = ix.dequant("q4_k", _u8(ip.block_q4k(half_bits(1.0), half_bits(1.0), sc, m, q)), 1, 256)[0]
                for s in range(8):
                    assert np.all(w[32 * s:32 * s + 32] == sc[s] - m[s]), (j, v, which, s)


@pytest.mark.parametrize("fmt", ["q4_k", "q5_k", "q6_k"])
def test_every_position_is_its_own(fmt):
    # a single quant differs from the background at position t: exactly weight t differs
    for t in list(range(0, 256, 7)) + [31, 32, 63, 64, 127, 128, 255]:
        if fmt == "q6_k":
            mk = lambda q: ip.block_q6k(half_bits(1.0), [1] * 16, q)
            bg, val = 32, 63
        else:
            mk = lambda q: (ip.block_q4k if fmt == "q4_k" else ip.block_q5k)(half_bits(1.0), half_bits(0.0), [1] * 8, [0] * 8, q)
            bg, val = 0, 15 if fmt == "q4_k" else 31
        q = [bg] * 256
        q[t] = val
        w = ix.dequant(fmt, _u8(mk(q)), 1, 256)[0]
        expect = np.zeros(256, dtype=np.float32)
        expect[t] = val - bg
        assert np.array_equal(w, expect), (fmt, t)


@pytest.mark.parametrize("fmt", ["q5_k", "q6_k"])
def test_every_bit_of_a_quant_counts(fmt):
    # quants 1, 2, 4, ... at one position: the value doubles each time (a high bit landing in the wrong place shows)
    for t in (0, 5, 37, 70, 101, 130, 170, 200, 255):
        bits = 5 if fmt == "q5_k" else 6
        for k in range(bits):
            q = [0] * 256
            q[t] = 1 << k
            if fmt == "q5_k":
                w = ix.dequant(fmt, _u8(ip.block_q5k(half_bits(1.0), half_bits(0.0), [1] * 8, [0] * 8, q)), 1, 256)[0]
                assert w[t] == (1 << k) and np.count_nonzero(w) == 1
            else:
                w = ix.dequant(fmt, _u8(ip.block_q6k(half_bits(1.0), [1] * 16, q)), 1, 256)[0]
                assert w[t] == (1 << k) - 32 and np.count_nonzero(w + 32) == 1


def test_q6k_by_hand():
    # d = 0.5, sub-scale of the 16 weights from 16 s on: s - 8 (signed); quant t = t % 64
    sc = [s - 8 for s in range(16)]
    q = [t % 64 for t in range(256)]
    w = ix.dequant("q6_k", _u8(ip.block_q6k(half_bits(0.5), sc, q)), 1, 256)[0]
    for t in (0, 1, 16, 31, 33, 64, 96, 127, 128, 200, 255):
        assert w[t] == 0.5 * (t // 16 - 8) * (t % 64 - 32), t


def test_q80_by_hand():
    q = [0] * 32
    q[0], q[1], q[31] = -128, 127, 3
    w = ix.dequant("q8_0", _u8(ip.block_q80(half_bits(0.25), q) + ip.block_q80(half_bits(2.0), q)), 1, 64)[0]
    assert w[0] == -32.0 and w[1] == 31.75 and w[31] == 0.75 and w[32] == -256.0 and w[63] == 6.0
    assert np.count_nonzero(w) == 6


@pytest.mark.parametrize("fmt", ["q4_k", "q5_k", "q6_k", "q8_0"])
def test_random_tensor_exact(fmt):
    raw, vals = ip.random_tensor(fmt, 3, 512, seed=11)
    w = ix.dequant(fmt, raw, 3, 512)
    # the exact value, rounded once to fp32 (d*sc*q and dmin*m are exact in fp32, their difference is rounded once)
    assert np.array_equal(w, vals.astype(np.float32))


def test_rows_and_blocks_in_order():
    # row r, block b of a q8_0 tensor holds the constant 8 r + b
    rows, cols = 4, 256
    raw = b"".join(ip.block_q80(half_bits(1.0), [8 * r + b] * 32) for r in range(rows) for b in range(cols // 32))
    w = ix.dequant("q8_0", _u8(raw), rows, cols)
    for r in range(rows):
        for b in range(cols // 32):
            assert np.all(w[r, 32 * b:32 * b + 32] == 8 * r + b)


def test_f16_f32_pass_through():
    a = np.arange(512, dtype=np.float32).reshape(2, 256) / 3
    assert np.array_equal(ix.dequant("f32", a.view(np.uint8), 2, 256), a)
    h = a.astype(np.float16)
    assert np.array_equal(ix.dequant("f16", h.view(np.uint8), 2, 256), h.astype(np.float32))
