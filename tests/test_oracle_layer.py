"""Pins for the oracle's decoder layer and window (CPU only).

The window is the unit a device advances per round (paper Sec. 3.1, Def. 1); it takes and
returns e FP32 values per token (App. A.3, communication latency); its KV cache grows by
2(h_k e_k + h_v e_v) bytes per layer per token (App. A.3, memory access latency); verifying
several tokens in one batch must leave outputs unchanged (App. A.12).
"""
import copy
import math

import numpy as np
import torch

import oracle
from workloads import synth
from workloads.configs import CONFIGS, TINY


def _torch_layer(dims, t, x, n_past):
    """The same layer written independently with torch float64 ops on dense weights."""
    T = x.shape[0]
    D, Hq, Hkv = dims.head_dim, dims.n_q_heads, dims.n_kv_heads
    W = {k: torch.from_numpy(oracle.dequant(t[k])).double() for k in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")}
    ga, gf = torch.from_numpy(t["g_attn"]).double(), torch.from_numpy(t["g_ffn"]).double()
    eps = float(np.float32(dims.rms_eps))
    xt = torch.from_numpy(x)

    def norm(v, g):
        return v * torch.rsqrt(v.pow(2).mean(-1, keepdim=True) + eps) * g

    def rope(v, H):
        v = v.reshape(T, H, D).clone()
        i = torch.arange(D // 2, dtype=torch.float64)
        freq = float(np.float32(dims.rope_theta)) ** (-2.0 * i / D)
        pos = torch.arange(n_past, n_past + T, dtype=torch.float64)
        ang = pos[:, None] * freq[None, :]
        c, s = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
        if dims.rope_mode == 0:
            a, b = v[..., :D // 2], v[..., D // 2:]
            return torch.cat([a * c - b * s, a * s + b * c], dim=-1)
        a, b = v[..., 0::2], v[..., 1::2]
        out = torch.empty_like(v)
        out[..., 0::2] = a * c - b * s
        out[..., 1::2] = a * s + b * c
        return out

    n1 = norm(xt, ga)
    q = rope(n1 @ W["wq"].T, Hq)
    k = rope(n1 @ W["wk"].T, Hkv)
    v = (n1 @ W["wv"].T).reshape(T, Hkv, D)
    K = torch.from_numpy(t["k_cache"].astype(np.float64)).clone()
    V = torch.from_numpy(t["v_cache"].astype(np.float64)).clone()
    for j in range(T):
        K[:, n_past + j] = k[j].float().half().double()
        V[:, n_past + j] = v[j].float().half().double()
    o = torch.zeros(T, Hq, D, dtype=torch.float64)
    grp = Hq // Hkv
    for j in range(T):
        n = n_past + j + 1
        for h in range(Hq):
            s = (K[h // grp, :n] @ q[j, h]) / math.sqrt(D)
            o[j, h] = torch.softmax(s, 0) @ V[h // grp, :n]
    h1 = xt + o.reshape(T, -1) @ W["wo"].T
    n2 = norm(h1, gf)
    y = h1 + (torch.nn.functional.silu(n2 @ W["wgate"].T) * (n2 @ W["wup"].T)) @ W["wdown"].T
    return y.numpy(), o.reshape(T, -1).numpy()


def _layers(cfg, cap=None):
    return [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]


def test_layer_vs_torch_float64():
    for name in ("t0", "t1", "t2"):
        cfg = TINY[name]
        t = synth.layer_tensors(cfg, 0)
        x = synth.window_input(cfg).astype(np.float64)
        ref, ref_o = _torch_layer(cfg.dims, t, x, cfg.n_past)
        got, taps = oracle.layer(cfg.dims, copy.deepcopy(t), x, cfg.n_past, taps=True)
        scale = np.abs(ref).max()
        assert np.abs(got - ref).max() / scale < 1e-10, name
        assert np.abs(taps["o"] - ref_o).max() / np.abs(ref_o).max() < 1e-10, name


def test_joint_equals_sequential():
    """T tokens in one batch == T successive single-token steps (speculative verification)."""
    cfg = TINY["t1"]
    x = synth.window_input(cfg).astype(np.float64)
    joint_layers = _layers(cfg)
    seq_layers = copy.deepcopy(joint_layers)
    y_joint = oracle.window(cfg.dims, joint_layers, x, cfg.n_past)
    y_seq = np.empty_like(y_joint)
    for j in range(cfg.T):
        y_seq[j] = oracle.window(cfg.dims, seq_layers, x[j:j + 1], cfg.n_past + j)[0]
    assert np.abs(y_joint - y_seq).max() / np.abs(y_seq).max() < 1e-12
    for a, b in zip(joint_layers, seq_layers):
        assert np.array_equal(a["k_cache"].view(np.uint16), b["k_cache"].view(np.uint16))
        assert np.array_equal(a["v_cache"].view(np.uint16), b["v_cache"].view(np.uint16))


def test_batch_of_sequences_is_independent_one_token_steps():
    """A batch step (one token for each of B sequences with their own caches and lengths) is, per sequence, the
    one-token window step of that sequence alone: same bits, same appended rows, whatever the other sequences
    are and in whatever order they stand; nothing else in a cache changes."""
    cfg = TINY["t1"]
    cap = 40
    n_past = [0, 7, 39, 21]
    B = len(n_past)
    layers = _layers(cfg)
    x = synth.batch_input(cfg, B).astype(np.float64)
    caches = synth.batch_caches(cfg, len(layers), n_past, cap)
    before = copy.deepcopy(caches)
    y = oracle.window_batch(cfg.dims, layers, caches, x, n_past)
    perm = [2, 0, 3, 1]
    caches_p = [[copy.deepcopy(before[l][b]) for b in perm] for l in range(len(layers))]
    y_p = oracle.window_batch(cfg.dims, layers, caches_p, x[perm], [n_past[b] for b in perm])
    assert np.array_equal(y_p, y[perm])
    for b in range(B):
        alone = [dict(t) for t in layers]
        for l, t in enumerate(alone):
            t["k_cache"], t["v_cache"] = copy.deepcopy(before[l][b])
        y_b = oracle.window(cfg.dims, alone, x[b:b + 1], n_past[b])
        assert np.array_equal(y_b[0], y[b])
        for l, t in enumerate(alone):
            for got, ref, old in zip(caches[l][b], (t["k_cache"], t["v_cache"]), before[l][b]):
                assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))
                keep = np.ones(cap, dtype=bool)
                keep[n_past[b]] = False
                assert np.array_equal(got[:, keep].view(np.uint16), old[:, keep].view(np.uint16))
                assert np.any(got[:, n_past[b]] != 0)


def test_window_is_composition_of_layers():
    cfg = TINY["t0"]
    x = synth.window_input(cfg).astype(np.float64)
    la = _layers(cfg)
    lb = copy.deepcopy(la)
    y = oracle.window(cfg.dims, la, x, cfg.n_past)
    h = x
    for t in lb:
        h = oracle.window(cfg.dims, [t], h, cfg.n_past)
    assert np.array_equal(y, h)


def test_kv_append_bytes_and_rows():
    """Only rows n_past..n_past+T-1 change: 2(h_k e_k + h_v e_v) bytes per token per layer."""
    cfg = TINY["t1"]
    d = cfg.dims
    cap = cfg.n_past + cfg.T + 5
    t = synth.layer_tensors(cfg, 0, kv_cap=cap)
    before_k, before_v = t["k_cache"].copy(), t["v_cache"].copy()
    oracle.layer(d, t, synth.window_input(cfg).astype(np.float64), cfg.n_past)
    ck = t["k_cache"].view(np.uint16) != before_k.view(np.uint16)
    cv = t["v_cache"].view(np.uint16) != before_v.view(np.uint16)
    rows = np.zeros(cap, dtype=bool)
    rows[cfg.n_past:cfg.n_past + cfg.T] = True
    assert not ck[:, ~rows].any() and not cv[:, ~rows].any()
    assert ck[:, rows].mean() > 0.99 and cv[:, rows].mean() > 0.99
    changed_bytes = 2 * (rows.sum() * d.n_kv_heads * d.head_dim) * 2
    assert changed_bytes == cfg.T * 2 * (d.kvd + d.kvd)
    assert d.kv_bytes_per_layer(1) == 2 * (d.n_kv_heads * d.head_dim + d.n_kv_heads * d.head_dim)


def test_rewind_after_rejection():
    """Run T=4, reject the last two drafts, continue with T=2 at n_past+2 with other inputs:
    equals a run that never saw the rejected tokens (stale rows are overwritten, never read)."""
    cfg = TINY["t1"]
    d = cfg.dims
    cap = cfg.n_past + 8
    x4 = synth.window_input(cfg).astype(np.float64)
    xb = synth.normal_f32(cfg.config_id, 1, "x_in", (2, d.e)).astype(np.float64)
    la = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(2)]
    lb = copy.deepcopy(la)
    oracle.window(d, la, x4, cfg.n_past)
    ya = oracle.window(d, la, xb, cfg.n_past + 2)
    oracle.window(d, lb, x4[:2], cfg.n_past)
    yb = oracle.window(d, lb, xb, cfg.n_past + 2)
    assert np.array_equal(ya, yb)


def test_lm_head_is_norm_then_gemv():
    cfg = TINY["t0"].with_(vocab=300)
    out = synth.output_layer_tensors(cfg)
    x = synth.window_input(cfg).astype(np.float64)
    got = oracle.lm_head(cfg.dims, out["g_final"], out["w_lm"], x)
    ref = oracle.gemv(out["w_lm"], oracle.rmsnorm(x, out["g_final"], cfg.dims.rms_eps))
    assert np.array_equal(got, ref) and got.shape == (cfg.T, 300)


def test_byte_accounting_matches_paper_formula():
    """b + 2(h_k e_k + h_v e_v) n_kv per layer (App. A.3, device loading time)."""
    expect = {"c0": 122683392, "c1": 154828800, "c2": 274268160, "c3": 481296384}
    for name, b in expect.items():
        cfg = CONFIGS[name]
        assert cfg.dims.q4k_bytes_per_layer() == b
        assert cfg.dims.kv_bytes_per_layer(cfg.n_past) == 4096 * cfg.n_past
    c3 = CONFIGS["c3"]
    assert abs(c3.bytes_per_step() / 1e9 - 9.961) < 0.01
    t = synth.layer_tensors(TINY["t0"], 0)
    nbytes = sum(t[k].nbytes for k in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown"))
    assert nbytes == TINY["t0"].dims.q4k_bytes_per_layer()


def test_synthetic_distribution():
    """Generator recipe: d, dmin in [1e-3, 4e-3]; fields uniform over their full range."""
    W = synth.q4k_tensor(0, 0, "wq", 64, 1024)
    dd = W.reshape(-1, 144)[:, 0:4].copy().view(np.float16).astype(np.float64)
    assert dd.min() >= 1e-3 - 1e-6 and dd.max() <= 4e-3 + 1e-5
    w = oracle.dequant(W)
    # E[w] = E[d] E[sc] E[q] - E[dmin] E[m] = 2.5e-3 * 31.5 * 7.5 - 2.5e-3 * 31.5 ~= 0.512
    assert abs(w.mean() - 0.512) < 0.02
    again = synth.q4k_tensor(0, 0, "wq", 64, 1024)
    assert np.array_equal(W, again)
    assert not np.array_equal(W, synth.q4k_tensor(0, 1, "wq", 64, 1024))
