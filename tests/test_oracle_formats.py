"""Pins of the oracle's decoding of the weight formats beside Q4_K (the set of formats in the profiler
paragraph of Sec. 4 / App. A.3; layouts: this repository's version 1, see oracle/prima_oracle.c).

What pins it: tensors built field by field by an independent packer (tests/qfmt_pack.py) whose every
weight is known as an exact rational; values known by mental arithmetic; bits per weight; a dense fp64
matrix product from a library."""
import sys
import os

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
import oracle
import qfmt_pack as fp
from q4k_pack import fraction_to_f32, half_bits


def _finite_half_bits(rng, shape):
    """random finite binary16 patterns of moderate size (exponent field 5..20), either sign"""
    return ((rng.integers(0, 2, shape) << 15) | (rng.integers(5, 21, shape) << 10) | rng.integers(0, 1024, shape)).astype(np.uint16)


def test_bits_per_weight():
    n = 6 * 1024
    for fmt, bits in [("q4_k", 4.5), ("q5_k", 5.5), ("q6_k", 6.5625), ("q8_0", 8.5), ("f16", 16), ("f32", 32)]:
        assert oracle.fmt_tensor_bytes(fmt, 6, 1024) * 8 == bits * n
    assert oracle.fmt_tensor_bytes("q6_k", 3, 100) == -1     # columns: whole super-blocks only


def test_q80_by_hand():
    # one row of 256 weights, 8 scales: d_i = 0.5 * (i + 1); q = -128, 127, 1, 0, ...
    q = np.zeros((1, 256), dtype=np.int64)
    q[0, 0], q[0, 1], q[0, 2], q[0, 33], q[0, 255] = -128, 127, 1, -3, 5
    d = np.array([[half_bits(0.5 * (i + 1)) for i in range(8)]])
    w = oracle.fmt_dequant("q8_0", fp.pack_q80(d, q), 1, 256)
    assert w[0, 0] == -64.0 and w[0, 1] == 63.5 and w[0, 2] == 0.5 and w[0, 33] == -3.0 and w[0, 255] == 20.0
    assert np.count_nonzero(w) == 5


def test_q6k_by_hand():
    # d = 2, sc of sub-block 0 = -3, of sub-block 15 = 5: q = 0 -> 2*-3*-32 = 192; q = 63 -> -186; q = 32 -> 0
    q = np.full((1, 1, 256), 32, dtype=np.int64)
    sc = np.zeros((1, 1, 16), dtype=np.int64)
    sc[0, 0, 0], sc[0, 0, 15] = -3, 5
    q[0, 0, 0], q[0, 0, 1], q[0, 0, 15], q[0, 0, 16], q[0, 0, 255] = 0, 63, 33, 0, 48
    w = oracle.fmt_dequant("q6_k", fp.pack_q6k(np.array([[half_bits(2.0)]]), sc, q), 1, 256)
    assert w[0, 0] == 192.0 and w[0, 1] == -186.0 and w[0, 15] == -6.0
    assert w[0, 16] == 0.0            # sub-block 1 has scale 0
    assert w[0, 255] == 160.0         # 2 * 5 * 16
    assert np.count_nonzero(w) == 4


def test_q5k_by_hand():
    # d = 1, dmin = 0.5; sub-block 0: sc 2, m 3; sub-block 7: sc 63, m 0
    sc = np.zeros((1, 1, 8), dtype=np.int64)
    m = np.zeros((1, 1, 8), dtype=np.int64)
    sc[0, 0, 0], m[0, 0, 0], sc[0, 0, 7] = 2, 3, 63
    q = np.zeros((1, 1, 256), dtype=np.int64)
    q[0, 0, 0], q[0, 0, 1], q[0, 0, 31], q[0, 0, 224], q[0, 0, 255] = 31, 16, 15, 17, 1
    W = fp.pack_q5k(np.array([[half_bits(1.0)]]), np.array([[half_bits(0.5)]]), sc, m, q)
    w = oracle.fmt_dequant("q5_k", W, 1, 256)
    assert w[0, 0] == 60.5 and w[0, 1] == 30.5 and w[0, 31] == 28.5 and w[0, 2] == -1.5
    assert w[0, 224] == 63.0 * 17 and w[0, 255] == 63.0 and w[0, 225] == 0.0
    assert np.all(w[0, 32:224] == 0.0)


@pytest.mark.parametrize("fmt", ["q5_k", "q6_k", "q8_0"])
def test_dequant_is_the_exact_value_rounded_once(fmt):
    """Random fields over their whole ranges, 3 rows x 2 super-blocks: every weight equals the exact
    rational value of the format's rule, rounded to fp32 once (positions included: the packer places
    row r, block b, weight t from the layout text)."""
    rng = np.random.default_rng(11)
    rows, nb = 3, 2
    if fmt == "q5_k":
        d, dm = _finite_half_bits(rng, (rows, nb)) & 0x7FFF, _finite_half_bits(rng, (rows, nb)) & 0x7FFF
        sc, m = rng.integers(0, 64, (rows, nb, 8)), rng.integers(0, 64, (rows, nb, 8))
        q = rng.integers(0, 32, (rows, nb, 256))
        W = fp.pack_q5k(d, dm, sc, m, q)
        exact = lambda r, b, t: fp.exact_q5k(d[r, b], dm[r, b], sc[r, b, t // 32], m[r, b, t // 32], q[r, b, t])
    elif fmt == "q6_k":
        d = _finite_half_bits(rng, (rows, nb))
        sc = rng.integers(-128, 128, (rows, nb, 16))
        q = rng.integers(0, 64, (rows, nb, 256))
        W = fp.pack_q6k(d, sc, q)
        exact = lambda r, b, t: fp.exact_q6k(d[r, b], sc[r, b, t // 16], q[r, b, t])
    else:
        d = _finite_half_bits(rng, (rows, nb * 8))
        q = rng.integers(-128, 128, (rows, nb * 256))
        W = fp.pack_q80(d, q)
        exact = lambda r, b, t: fp.exact_q80(d[r, b * 8 + t // 32], q[r, b * 256 + t])
    w = oracle.fmt_dequant(fmt, W, rows, nb * 256)
    for r in range(rows):
        for b in range(nb):
            for t in range(256):
                want = fraction_to_f32(exact(r, b, t))
                assert w[r, b * 256 + t] == want, (r, b, t, w[r, b * 256 + t], want)


def test_plain_number_formats():
    rng = np.random.default_rng(5)
    a = rng.standard_normal((3, 512)).astype(np.float32)
    assert np.array_equal(oracle.fmt_dequant("f32", a.view(np.uint8), 3, 512), a)
    h = a.astype(np.float16)
    assert np.array_equal(oracle.fmt_dequant("f16", h.view(np.uint8), 3, 512), h.astype(np.float32))


def test_q4k_through_the_format_calls_is_the_q4k_decoder():
    from workloads import synth
    W = synth.q4k_tensor(0, 0, "wq", 5, 512)
    assert np.array_equal(oracle.fmt_dequant("q4_k", W, 5, 512), oracle.dequant(W))


@pytest.mark.parametrize("fmt", ["q5_k", "q6_k", "q8_0", "f16", "f32"])
def test_gemv_is_the_dense_product(fmt):
    """The mat-vec of every format equals a library fp64 product with the dequantised matrix."""
    from workloads import synth
    rows, cols, T = 37, 768, 3
    W = synth.fmt_tensor(0, 0, "wq", fmt, rows, cols)
    x = synth.normal_f32(0, 0, "q", (T, cols)).astype(np.float64)
    dense = oracle.fmt_dequant(fmt, W, rows, cols).astype(np.float64)
    assert np.isfinite(dense).all() and np.abs(dense).max() > 0
    y = oracle.fmt_gemv(fmt, W, rows, cols, x)
    ref = x @ dense.T
    assert np.abs(y - ref).max() <= 1e-12 * np.abs(ref).max()


def test_lm_head_in_another_format_is_norm_then_product():
    from workloads import synth
    from workloads.configs import CONFIGS
    d = CONFIGS["c0"].dims
    vocab = 300
    W = synth.fmt_tensor(0, 0, "w_lm", "q6_k", vocab, d.e)
    g = synth.gain_f32(0, 0, "g_final", d.e)
    x = synth.normal_f32(0, 0, "x_in", (2, d.e)).astype(np.float64)
    got = oracle.lm_head_fmt(d, "q6_k", g, W, vocab, x)
    n = x / np.sqrt((x ** 2).mean(axis=1, keepdims=True) + float(np.float32(d.rms_eps))) * g.astype(np.float64)
    ref = n @ oracle.fmt_dequant("q6_k", W, vocab, d.e).astype(np.float64).T
    assert np.abs(got - ref).max() <= 1e-12 * np.abs(ref).max()


def test_layer_does_not_depend_on_the_format_of_a_matrix():
    """A layer whose matrix is stored as the fp32 numbers that its Q4_K tensor decodes to gives the same bits as
    the Q4_K layer, for each of the seven matrices in turn (a format routed to the wrong projection would decode
    garbage), and for all seven at once."""
    from workloads import synth
    from workloads.configs import CONFIGS
    cfg = CONFIGS["c0"]
    d = cfg.dims
    t = synth.layer_tensors(cfg, 0)
    x = synth.window_input(cfg).astype(np.float64)
    caches = (t["k_cache"].copy(), t["v_cache"].copy())
    ref = oracle.layer(d, t, x, cfg.n_past)
    names = list(oracle.WEIGHTS)
    for subset in [[n] for n in names] + [names]:
        t2 = dict(t)
        t2["k_cache"], t2["v_cache"] = caches[0].copy(), caches[1].copy()
        for n in subset:
            t2[n] = oracle.dequant(t[n]).view(np.uint8).reshape(-1)
        got = oracle.layer(d, t2, x, cfg.n_past, formats={n: "f32" for n in subset})
        assert np.array_equal(got, ref), subset


# ---- do the pins bite?  Plausible mistakes planted in a copy of the oracle's source (on the CPU, in a temporary
# ---- library; the oracle itself is untouched): each must fail the exact-value pin.
_MUTANTS = [
    ("q6_k", "(qh[(t / 16) * 4 + t % 4] >> (2 * ((t % 16) / 4))) & 3", "(qh[t / 4] >> (2 * (t % 4))) & 3", "high bits read from another placement"),
    ("q6_k", "d * (float)sc[t / 16]", "d * (float)sc[t / 32]", "sub-scale of the wrong sub-block"),
    ("q6_k", "(lo | (hi << 4)) - 32)", "(lo | (hi << 4)) - 31)", "offset 31 instead of 32"),
    ("q6_k", "(lo | (hi << 4)) - 32)", "(lo | (hi << 2)) - 32)", "high bits shifted to the wrong place"),
    ("q5_k", "(qh[(t / 32) * 4 + t % 4] >> ((t % 32) / 4)) & 1", "(qh[t / 8] >> (t % 8)) & 1", "fifth bit read from another placement"),
    ("q5_k", "field6(hdr, 8 + s); /* field6 skips", "field6(hdr, s); /* field6 skips", "sub-min taken from the sub-scale's field"),
    ("q5_k", "return (t % 8 < 4) ? (byte & 15) : (byte >> 4);", "return (t % 8 < 4) ? (byte >> 4) : (byte & 15);", "nibbles swapped"),
    ("q5_k", "uint8_t byte = nib[(t / 8) * 4 + t % 4];", "uint8_t byte = nib[t / 2];", "low bits read from another placement"),
    ("q8_0", "half_at(dp + 2 * (t / 32))", "half_at(dp + 2 * (t / 64))", "scale of the wrong block"),
    ("q8_0", "const int8_t *q = (const int8_t *)W + blk * QK;", "const uint8_t *q = (const uint8_t *)W + blk * QK;", "quants read as unsigned"),
]


@pytest.mark.parametrize("fmt,old,new,what", _MUTANTS, ids=[m[3] for m in _MUTANTS])
def test_a_planted_mistake_fails_the_exact_value_pin(tmp_path, fmt, old, new, what):
    import ctypes as C
    import subprocess
    src = open(os.path.join(os.path.dirname(oracle.__file__), "prima_oracle.c")).read()
    assert src.count(old) == 1, "the oracle's text has changed: update this mutant"
    bad_c, bad_so = tmp_path / "mutant.c", tmp_path / "mutant.so"
    bad_c.write_text(src.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-o", str(bad_so), str(bad_c), "-lm"])
    lib = C.CDLL(str(bad_so))
    rng = np.random.default_rng(11)
    rows, nb = 3, 2
    if fmt == "q5_k":
        d, dm = _finite_half_bits(rng, (rows, nb)) & 0x7FFF, _finite_half_bits(rng, (rows, nb)) & 0x7FFF
        sc, m = rng.integers(0, 64, (rows, nb, 8)), rng.integers(0, 64, (rows, nb, 8))
        q = rng.integers(0, 32, (rows, nb, 256))
        W = fp.pack_q5k(d, dm, sc, m, q)
        exact = lambda r, b, t: fp.exact_q5k(d[r, b], dm[r, b], sc[r, b, t // 32], m[r, b, t // 32], q[r, b, t])
    elif fmt == "q6_k":
        d = _finite_half_bits(rng, (rows, nb))
        sc = rng.integers(-128, 128, (rows, nb, 16))
        q = rng.integers(0, 64, (rows, nb, 256))
        W = fp.pack_q6k(d, sc, q)
        exact = lambda r, b, t: fp.exact_q6k(d[r, b], sc[r, b, t // 16], q[r, b, t])
    else:
        d = _finite_half_bits(rng, (rows, nb * 8))
        q = rng.integers(-128, 128, (rows, nb * 256))
        W = fp.pack_q80(d, q)
        exact = lambda r, b, t: fp.exact_q80(d[r, b * 8 + t // 32], q[r, b * 256 + t])
    W = np.ascontiguousarray(W, dtype=np.uint8)
    out = np.empty((rows, nb * 256), dtype=np.float32)
    rc = lib.orc_fmt_dequant(C.c_int32(oracle.FORMATS[fmt]), W.ctypes.data_as(C.c_void_p), C.c_int64(rows), C.c_int64(nb * 256),
                             out.ctypes.data_as(C.c_void_p))
    assert rc == 0
    wrong = sum(out[r, b * 256 + t] != fraction_to_f32(exact(r, b, t)) for r in range(rows) for b in range(nb) for t in range(256))
    assert wrong > 0, what
    # and the untouched oracle passes the same check
    good = oracle.fmt_dequant(fmt, W, rows, nb * 256)
    assert all(good[r, b * 256 + t] == fraction_to_f32(exact(r, b, t)) for r in range(rows) for b in range(nb) for t in range(256))
