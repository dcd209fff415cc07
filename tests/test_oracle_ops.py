"""Pins for the oracle's small operators: fp16 conversion, RMSNorm, RoPE, SwiGLU, softmax, attention.

The paper fixes the KV cache precision (fp16) and its byte volumes (App. A.3, memory access
latency); the operator formulas are the standard Llama/Qwen definitions.
"""
import math

import numpy as np
import torch

import oracle
from workloads.configs import ModelDims


def test_half_to_double_exhaustive_vs_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    for b in range(0, 65536, 7):
        v = oracle.half_to_double(b)
        assert (math.isnan(v) and math.isnan(ref[b])) or v == ref[b], b


def test_float_to_half_vs_numpy():
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(4000).astype(np.float32),
        (rng.standard_normal(2000) * 1e-6).astype(np.float32),      # subnormal half range
        (rng.standard_normal(2000) * 3e4).astype(np.float32),       # near overflow
        np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                  1.0009765625, 1.00048828125, 1.00146484375], dtype=np.float32),   # ties to even
    ])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    for v, r in zip(vals, ref):
        assert oracle.float_to_half(v) == int(r), float(v)


def test_rmsnorm_invariants():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((3, 640)) * 50.0
    g1 = np.ones(640, dtype=np.float32)
    eps = 1e-5
    y = oracle.rmsnorm(x, g1, eps)
    ms = (x ** 2).mean(axis=1)
    # RMS of the output before gain equals sqrt(ms / (ms + eps))
    assert np.allclose(np.sqrt((y ** 2).mean(axis=1)), np.sqrt(ms / (ms + np.float32(eps))), rtol=1e-13)
    # gain multiplies elementwise afterwards
    g = (1 + 0.1 * rng.standard_normal(640)).astype(np.float32)
    assert np.allclose(oracle.rmsnorm(x, g, eps), y * g.astype(np.float64), rtol=1e-14)
    # eps sits inside the root, added to the mean of squares: tiny input is damped, not normalised
    tiny = np.full((1, 16), 1e-4)
    out = oracle.rmsnorm(tiny, np.ones(16, dtype=np.float32), eps)
    assert np.allclose(out, 1e-4 / math.sqrt(1e-8 + float(np.float32(eps))), rtol=1e-12)
    # torch reference
    xt = torch.from_numpy(x)
    ref = xt * torch.rsqrt(xt.pow(2).mean(-1, keepdim=True) + float(np.float32(eps))) * torch.from_numpy(g).double()
    assert np.allclose(oracle.rmsnorm(x, g, eps), ref.numpy(), rtol=1e-13)


def test_rope_invariants():
    rng = np.random.default_rng(2)
    H, D, theta = 3, 64, 1e4
    v = rng.standard_normal(H * D)
    for mode in (0, 1):
        # position 0 is the identity
        assert np.array_equal(oracle.rope(v, H, D, 0, theta, mode), v)
        r = oracle.rope(v, H, D, 977, theta, mode).reshape(H, D)
        v2 = v.reshape(H, D)
        for i in range(D // 2):
            ia, ib = (2 * i, 2 * i + 1) if mode else (i, i + D // 2)
            # each pair keeps its norm
            assert np.allclose(r[:, ia] ** 2 + r[:, ib] ** 2, v2[:, ia] ** 2 + v2[:, ib] ** 2, rtol=1e-12)
            # and is turned by exactly pos * theta^(-2i/D)
            ang = 977 * theta ** (-2.0 * i / D)
            assert np.allclose(r[:, ia], v2[:, ia] * math.cos(ang) - v2[:, ib] * math.sin(ang), rtol=1e-9, atol=1e-12)
            assert np.allclose(r[:, ib], v2[:, ia] * math.sin(ang) + v2[:, ib] * math.cos(ang), rtol=1e-9, atol=1e-12)
        # relative-position property: <rope(q,p), rope(k,p')> depends on p - p' only
        q, k = rng.standard_normal(D), rng.standard_normal(D)
        a = oracle.rope(q, 1, D, 100, theta, mode) @ oracle.rope(k, 1, D, 60, theta, mode)
        b = oracle.rope(q, 1, D, 1040, theta, mode) @ oracle.rope(k, 1, D, 1000, theta, mode)
        assert abs(a - b) < 1e-9
    # the two pairings differ (a wrong default would be seen)
    assert not np.allclose(oracle.rope(v, H, D, 5, theta, 0), oracle.rope(v, H, D, 5, theta, 1))


def test_rope_closed_forms():
    """The angle schedule pinned without retyping it: a unit vector in every pair shows its angle directly (atan2);
    pair 0 turns by `pos` radians, the pair a quarter of the way through the head by pos / sqrt(theta) (theta = 1e4:
    pos / 100, so position 200 turns it by 2 rad, cos 2 and sin 2 as printed in any table), and the angles fall
    geometrically with a constant ratio that would reach pos / theta one pair past the last."""
    H, D, theta = 1, 64, 1e4
    for mode in (0, 1):
        pair = lambda i: (2 * i, 2 * i + 1) if mode else (i, i + D // 2)
        v = np.zeros(D)
        for i in range(D // 2):
            v[pair(i)[0]] = 1.0                      # (1, 0) in every pair
        r = oracle.rope(v, H, D, 200, theta, mode)
        a16, b16 = pair(16)
        assert abs(r[a16] - (-0.4161468365471424)) < 1e-12 and abs(r[b16] - 0.9092974268256817) < 1e-12
        # small position: every angle below pi, so atan2 returns it
        pos = 3
        r = oracle.rope(v, H, D, pos, theta, mode)
        ang = np.array([math.atan2(r[pair(i)[1]], r[pair(i)[0]]) for i in range(D // 2)])
        assert abs(ang[0] - pos) < 1e-12                                  # pair 0: pos radians, counter-clockwise
        ratio = ang[1:] / ang[:-1]
        assert np.allclose(ratio, ratio[0], rtol=1e-9) and ratio[0] < 1   # geometric, falling
        assert abs(ang[-1] * ratio[0] - pos / theta) < 1e-15              # D/2 steps from pos to pos / theta
        assert abs(ang[D // 4] - pos / 100.0) < 1e-13


def test_silu_swiglu():
    z = np.array([0.0, 30.0, -30.0, 1.5, -1.5, 700.0, -700.0])
    one = np.ones_like(z)
    s = oracle.swiglu(z, one)
    assert s[0] == 0.0
    assert abs(s[1] - 30.0) < 1e-11 and abs(s[2]) < 1e-11
    assert abs((s[3] - s[4]) - 1.5) < 1e-15          # silu(z) - silu(-z) = z
    assert s[5] == 700.0 and abs(s[6]) < 1e-290
    rng = np.random.default_rng(3)
    g, u = rng.standard_normal(1000) * 5, rng.standard_normal(1000)
    ref = (torch.nn.functional.silu(torch.from_numpy(g)) * torch.from_numpy(u)).numpy()
    assert np.allclose(oracle.swiglu(g, u), ref, rtol=1e-13, atol=1e-15)


def test_softmax_rows_sum_to_one():
    rng = np.random.default_rng(4)
    for scale in (1.0, 80.0, 1e4):
        w = oracle.softmax(rng.standard_normal(513) * scale)
        assert abs(w.sum() - 1.0) < 1e-12 and np.all(w >= 0)
    # shift invariance (max subtraction)
    l = rng.standard_normal(10)
    assert np.allclose(oracle.softmax(l), oracle.softmax(l + 1e6), rtol=1e-9)


def _dims(Hq=8, Hkv=2, D=64):
    return ModelDims(Hq * D, Hq, Hkv, D, 256, 1e4)


def _torch_attn(dims, q, K, V, n_past, T):
    Hq, Hkv, D = dims.n_q_heads, dims.n_kv_heads, dims.head_dim
    grp = Hq // Hkv
    qt = torch.from_numpy(np.asarray(q, dtype=np.float64)).reshape(T, Hq, D)
    Kt = torch.from_numpy(K.astype(np.float64))
    Vt = torch.from_numpy(V.astype(np.float64))
    out = torch.zeros(T, Hq, D, dtype=torch.float64)
    for j in range(T):
        n = n_past + j + 1
        for h in range(Hq):
            s = (Kt[h // grp, :n] @ qt[j, h]) / math.sqrt(D)
            out[j, h] = torch.softmax(s, 0) @ Vt[h // grp, :n]
    return out.numpy()


def test_attention_vs_torch_float64():
    rng = np.random.default_rng(5)
    for (Hq, Hkv, D, n_past, T) in [(8, 2, 64, 37, 1), (10, 2, 128, 130, 4), (8, 1, 128, 0, 3), (4, 4, 32, 5, 2)]:
        dims = _dims(Hq, Hkv, D)
        cap = n_past + T + 3
        K = rng.standard_normal((Hkv, cap, D)).astype(np.float16)
        V = rng.standard_normal((Hkv, cap, D)).astype(np.float16)
        q = rng.standard_normal((T, Hq, D))
        got = oracle.attn_decode(dims, q, K, V, n_past, T)
        assert np.allclose(got, _torch_attn(dims, q, K, V, n_past, T), rtol=1e-11, atol=1e-12)


def test_attention_special_cases():
    rng = np.random.default_rng(6)
    dims = _dims(8, 2, 64)
    D = 64
    # one key: output is that V row exactly
    K = rng.standard_normal((2, 4, D)).astype(np.float16)
    V = rng.standard_normal((2, 4, D)).astype(np.float16)
    q = rng.standard_normal((1, 8, D))
    o = oracle.attn_decode(dims, q, K, V, 0, 1)
    for h in range(8):
        assert np.array_equal(o[0, h], V[h // 4, 0].astype(np.float64))
    # all K rows equal: output is the mean of the V rows
    n = 50
    K = np.repeat(rng.standard_normal((2, 1, D)).astype(np.float16), n, axis=1)
    V = rng.standard_normal((2, n, D)).astype(np.float16)
    o = oracle.attn_decode(dims, q, K, V, n - 1, 1)
    for h in range(8):
        assert np.allclose(o[0, h], V[h // 4].astype(np.float64).mean(axis=0), rtol=1e-12, atol=1e-13)
    # identical queries within a group give identical outputs; different groups differ
    K = rng.standard_normal((2, n, D)).astype(np.float16)
    qq = np.repeat(rng.standard_normal((1, 1, D)), 8, axis=1)
    o = oracle.attn_decode(dims, qq, K, V, n - 1, 1)
    assert np.array_equal(o[0, 0], o[0, 3]) and np.array_equal(o[0, 4], o[0, 7])
    assert not np.allclose(o[0, 0], o[0, 4])
    # permuting cached positions (K and V together) leaves the output unchanged
    perm = rng.permutation(n)
    o1 = oracle.attn_decode(dims, q, K, V, n - 1, 1)
    o2 = oracle.attn_decode(dims, q, K[:, perm], V[:, perm], n - 1, 1)
    assert np.allclose(o1, o2, rtol=1e-11, atol=1e-13)


def test_attention_causal_tail_and_gap():
    """Token j sees rows 0..n_past+j only: later rows may hold anything."""
    rng = np.random.default_rng(7)
    dims = _dims(4, 2, 32)
    n_past, T = 9, 3
    K = rng.standard_normal((2, n_past + T, 32)).astype(np.float16)
    V = rng.standard_normal((2, n_past + T, 32)).astype(np.float16)
    q = rng.standard_normal((T, 4, 32))
    o, gap = oracle.attn_decode(dims, q, K, V, n_past, T, return_gap=True)
    assert gap > 0
    K2, V2 = K.copy(), V.copy()
    K2[:, n_past + 1:] = 77.0       # rows after token 0's own row
    V2[:, n_past + 1:] = -55.0
    o2 = oracle.attn_decode(dims, q, K2, V2, n_past, T)
    assert np.array_equal(o[0], o2[0]) and not np.allclose(o[1], o2[1])
