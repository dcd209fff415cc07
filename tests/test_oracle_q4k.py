"""Pins for the oracle's Q4_K decoding and mat-vec (CPU only).

Semantics pinned: 256 weights per super-block, w = d*sc_s*q - dmin*m_s with s = t // 32
(config 0 of workloads/configs.py); the paper itself only names the format (App. A.3, computation latency).
"""
import os
import random
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from q4k_pack import (dense_from_blocks, exact_weight, fraction_to_f32, half_bits, pack_block,
                      unpack_block)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "q4k_handbuilt.txt")


def _one(blk):
    return oracle.dequant(blk.reshape(1, 1, 144))[0]


def test_handbuilt_known_value():
    # d = 2^-8, sc = 3, q = 5, dmin = 2^-9, m = 7  ->  15/256 - 7/512 = 23/512 everywhere
    blk = pack_block(half_bits(2.0 ** -8), half_bits(2.0 ** -9), [3] * 8, [7] * 8, [5] * 256)
    w = _one(blk)
    assert np.all(w == np.float32(23.0 / 512.0))


def test_handbuilt_zero_and_max():
    z = _one(np.zeros(144, dtype=np.uint8))
    assert np.all(z == 0.0)
    # d = 1, dmin = 0.5, all fields at maximum: 63*15 - 0.5*63 = 913.5
    blk = pack_block(half_bits(1.0), half_bits(0.5), [63] * 8, [63] * 8, [15] * 256)
    assert np.all(_one(blk) == np.float32(913.5))
    # the packed maximum block is all ones in bytes 4..143
    assert np.all(blk[4:] == 255)


def test_single_nibble_each_position():
    # one nonzero quant at position t: catches any index mapping mistake
    for t in range(256):
        q = [0] * 256
        q[t] = 9
        blk = pack_block(half_bits(1.0), half_bits(0.0), [1] * 8, [0] * 8, q)
        w = _one(blk)
        expect = np.zeros(256, dtype=np.float32)
        expect[t] = 9.0
        assert np.array_equal(w, expect), t


def test_single_field_each_position():
    # one nonzero 6-bit field: sub-scale s scales weights 32s..32s+31 only, sub-min likewise
    for s in range(8):
        sc = [0] * 8
        sc[s] = 37
        w = _one(pack_block(half_bits(0.25), half_bits(1.0), sc, [0] * 8, [2] * 256))
        expect = np.zeros(256, dtype=np.float32)
        expect[32 * s:32 * s + 32] = 0.25 * 37 * 2
        assert np.array_equal(w, expect), ("sc", s)
        m = [0] * 8
        m[s] = 41
        w = _one(pack_block(half_bits(0.25), half_bits(2.0), [0] * 8, m, [2] * 256))
        expect = np.zeros(256, dtype=np.float32)
        expect[32 * s:32 * s + 32] = -2.0 * 41
        assert np.array_equal(w, expect), ("m", s)


def test_golden_handbuilt_file():
    """Blocks listed field by field in tests/golden with their values worked out by hand."""
    n = 0
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if not line:
            continue
        d, dmin, sc, m, q, num, den = line.split()
        blk = pack_block(half_bits(float(Fraction(d))), half_bits(float(Fraction(dmin))),
                         [int(sc)] * 8, [int(m)] * 8, [int(q)] * 256)
        assert np.all(_one(blk) == np.float32(int(num) / int(den))), line
        n += 1
    assert n >= 6


def test_exact_rational_random_half_values():
    """Every finite fp16 d/dmin: oracle bits == nearest fp32 of the exact rational."""
    rnd = random.Random(1234)
    checked = 0
    for _ in range(300):
        while True:
            d_bits, dmin_bits = rnd.randrange(0, 1 << 16), rnd.randrange(0, 1 << 16)
            if (d_bits >> 10) & 31 != 31 and (dmin_bits >> 10) & 31 != 31:
                break
        sc = [rnd.randrange(64) for _ in range(8)]
        m = [rnd.randrange(64) for _ in range(8)]
        q = [rnd.randrange(16) for _ in range(256)]
        w = _one(pack_block(d_bits, dmin_bits, sc, m, q))
        for t in range(0, 256, 5):
            fr = exact_weight(d_bits, dmin_bits, sc[t // 32], m[t // 32], q[t])
            v = float(fr)
            if Fraction(v) != fr:      # needs > 53 bits: extreme exponent gap, skip
                continue
            if abs(v) > 3e38:
                continue
            assert np.float32(v).tobytes() == w[t].tobytes() or (v == 0 and w[t] == 0), (d_bits, dmin_bits, t)
            checked += 1
    assert checked > 10000


def test_exact_config_range_vectorised():
    """10^6 weights in the benchmark's value range: fp64 evaluation is exact there."""
    rng = np.random.default_rng(7)
    nb = 4096
    W = rng.integers(0, 256, size=(nb, 1, 144), dtype=np.uint8)
    dd = (1e-3 + 3e-3 * rng.random((nb, 2), dtype=np.float32)).astype(np.float16)
    W[:, 0, 0:4] = dd.view(np.uint8).reshape(nb, 4)
    got = oracle.dequant(W)                         # [nb, 256]
    # independent vectorised unpack
    stream = np.zeros(nb, dtype=object)
    for i in range(12):
        stream = stream + (W[:, 0, 4 + i].astype(object) << (8 * i))
    f = np.array([[(int(s) >> (6 * i)) & 63 for i in range(16)] for s in stream], dtype=np.float64)
    qb = W[:, 0, 16:]
    q = np.empty((nb, 256), dtype=np.float64)
    q[:, 0::2] = qb & 15
    q[:, 1::2] = qb >> 4
    d = dd[:, 0].astype(np.float64)[:, None]
    dm = dd[:, 1].astype(np.float64)[:, None]
    sc = np.repeat(f[:, :8], 32, axis=1)
    m = np.repeat(f[:, 8:], 32, axis=1)
    exact = d * sc * q - dm * m                     # exact in fp64 (<= 21 + small exponent span bits)
    assert np.array_equal(exact.astype(np.float32).view(np.uint32), got.view(np.uint32))


def test_unpack_roundtrip():
    rnd = random.Random(5)
    sc = [rnd.randrange(64) for _ in range(8)]
    m = [rnd.randrange(64) for _ in range(8)]
    q = [rnd.randrange(16) for _ in range(256)]
    blk = pack_block(0x1234, 0x2345, sc, m, q)
    assert unpack_block(blk) == (0x1234, 0x2345, sc, m, q)


def _rand_tensor(rng, rows, nb):
    W = rng.integers(0, 256, size=(rows, nb, 144), dtype=np.uint8)
    dd = (1e-3 + 3e-3 * rng.random((rows * nb, 2), dtype=np.float32)).astype(np.float16)
    W.reshape(-1, 144)[:, 0:4] = dd.view(np.uint8).reshape(-1, 4)
    return W


def test_gemv_bruteforce_dense():
    rng = np.random.default_rng(11)
    for rows, nb, T in [(3, 1, 1), (8, 2, 3), (5, 3, 2)]:
        W = _rand_tensor(rng, rows, nb)
        x = rng.standard_normal((T, nb * 256))
        dense = dense_from_blocks(W)
        ref = np.zeros((T, rows))
        for t in range(T):
            for r in range(rows):
                acc = 0.0
                for c in range(nb * 256):
                    acc += dense[r, c] * x[t, c]
                ref[t, r] = acc
        got = oracle.gemv(W, x)
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_gemv_integer_exact():
    """d, dmin powers of two and small integer x: every partial sum is exact, any order."""
    rng = np.random.default_rng(3)
    rows, nb = 6, 2
    W = rng.integers(0, 256, size=(rows, nb, 144), dtype=np.uint8)
    for r in range(rows):
        for b in range(nb):
            W[r, b, 0:2] = np.frombuffer(int(half_bits(2.0 ** -(r % 3))).to_bytes(2, "little"), dtype=np.uint8)
            W[r, b, 2:4] = np.frombuffer(int(half_bits(2.0 ** -(b + 1))).to_bytes(2, "little"), dtype=np.uint8)
    x = rng.integers(-8, 9, size=(2, nb * 256)).astype(np.float64)
    dense = dense_from_blocks(W)
    ref = (dense.astype(object) @ x.T.astype(object)).T.astype(np.float64)   # python-number arithmetic
    got = oracle.gemv(W, x)
    assert np.array_equal(got, ref)


def test_gemv_vs_torch_float64_matmul():
    rng = np.random.default_rng(21)
    W = _rand_tensor(rng, 96, 5)
    x = rng.standard_normal((4, 5 * 256))
    dense = torch.from_numpy(oracle.dequant(W)).to(torch.float64)
    ref = (torch.from_numpy(x) @ dense.T).numpy()
    got = oracle.gemv(W, x)
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-9)


def test_dequant_matches_second_loop():
    rng = np.random.default_rng(2)
    W = _rand_tensor(rng, 4, 2)
    assert np.array_equal(oracle.dequant(W).astype(np.float64), dense_from_blocks(W))


def test_gemv_rejects_bad_cols():
    import ctypes as C
    W = np.zeros(144, dtype=np.uint8)
    y = np.zeros(1)
    x = np.zeros(300)
    rc = oracle.lib().orc_q4k_gemv(W.ctypes.data_as(C.c_void_p), C.c_int64(1), C.c_int64(300),
                                   x.ctypes.data_as(C.c_void_p), C.c_int64(300), C.c_int32(1),
                                   y.ctypes.data_as(C.c_void_p), C.c_int64(1))
    assert rc != 0
