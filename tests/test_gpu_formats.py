"""GPU parity of the other weight formats (Q5_K, Q6_K, Q8_0, FP16, FP32) against the CPU oracle, through
the C ABI: dequantisation bit for bit, mat-vec and output layer within the mat-vec tolerance."""
import numpy as np
import pytest
import torch

import oracle
from metrics import rel_err
from tolerance import EPS_FP32, check_hidden
from workloads import synth
from workloads.configs import CONFIGS, TINY

pytestmark = pytest.mark.gpu

FORMATS = ["q5_k", "q6_k", "q8_0", "f16", "f32"]
GEMV_TOL = 1e-4      # fp32 sums of up to 28672 terms against fp64 (the Q4_K mat-vec tests use the same bound)


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _rand_tensor(rng, fmt, rows, cols):
    """every field uniform over its range, scales any finite binary16 of moderate size (either sign)"""
    n = rows * cols // 256
    nbytes = int(n * 256 * synth.FORMAT_BITS[fmt] / 8)
    if fmt == "f32":
        return rng.standard_normal((rows, cols)).astype(np.float32).view(np.uint8).reshape(-1)
    if fmt == "f16":
        return rng.standard_normal((rows, cols)).astype(np.float16).view(np.uint8).reshape(-1)
    raw = rng.integers(0, 256, nbytes, dtype=np.uint8)

    def halves(count):
        return ((rng.integers(0, 2, count) << 15) | (rng.integers(8, 18, count) << 10) | rng.integers(0, 1024, count)).astype("<u2").view(np.uint8)

    if fmt == "q5_k":
        raw[:16 * n].reshape(n, 16)[:, 0:4] = halves(2 * n).reshape(n, 4)
    elif fmt == "q6_k":
        raw[208 * n:] = halves(n)
    else:
        raw[rows * cols:] = halves(8 * n)
    return raw


@pytest.mark.parametrize("fmt", FORMATS + ["q4_k"])
def test_dequant_bit_exact(gpu_lib, fmt):
    rng = np.random.default_rng(3)
    for rows, cols in [(1, 256), (5, 768), (67, 2048), (3, 28672)]:
        W = synth.fmt_tensor(0, 1, "wq", fmt, rows, cols) if fmt == "q4_k" else _rand_tensor(rng, fmt, rows, cols)
        ref = oracle.fmt_dequant(fmt, W, rows, cols)
        got = gpu_lib.fmt_dequant(fmt, _dev(W), rows, cols).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), ref.view(np.uint32)), (fmt, rows, cols)


@pytest.mark.parametrize("fmt", FORMATS)
def test_gemv_shapes_and_token_counts(gpu_lib, fmt):
    """Rows ragged against the 4-, 2- and 1-row groups (few and many rows: both choices of rows per wave), K from one
    super-block to 40960 (whole and partial pieces of 1024 weights, one and several chunks of K in LDS), every token
    count (passes of up to 8), activations with a different scale per token: each against the oracle, and twice with
    identical bits."""
    rng = np.random.default_rng(77)
    cases = [(1, 256, 1), (2, 256, 16), (3, 512, 2), (5, 768, 3), (37, 1024, 4), (130, 1280, 5), (64, 4096, 6), (63, 4352, 7),
             (257, 8192, 8), (33, 8192, 9), (7, 28672, 1), (18, 28672, 12), (1000, 3584, 1), (4096, 2048, 1),
             # K beyond what LDS holds for one and two tokens (chunks of 32768 and 16384 weights), 16 tokens in two passes
             (9, 40960, 1), (6, 33024, 2), (5, 12288, 16), (40000, 256, 1), (33000, 512, 3)]
    for rows, cols, T in cases:
        W = _rand_tensor(rng, fmt, rows, cols)
        x = (rng.standard_normal((T, cols)) * np.exp(2 * rng.standard_normal((T, 1)))).astype(np.float32)
        ref = oracle.fmt_gemv(fmt, W, rows, cols, x.astype(np.float64))
        Wd, xd = _dev(W), _dev(x)
        got = gpu_lib.fmt_gemv(fmt, Wd, rows, cols, xd).cpu().numpy()
        again = gpu_lib.fmt_gemv(fmt, Wd, rows, cols, xd).cpu().numpy()
        assert rel_err(got, ref) < GEMV_TOL, (fmt, rows, cols, T, rel_err(got, ref))
        assert np.array_equal(got.view(np.uint32), again.view(np.uint32)), (fmt, rows, cols, T)


def test_gemv_strided_activations_and_outputs(gpu_lib):
    rng = np.random.default_rng(8)
    rows, cols, T = 50, 1024, 3
    W = _rand_tensor(rng, "q6_k", rows, cols)
    xbig = torch.full((T, cols + 64), float("nan"), device="cuda")
    x = rng.standard_normal((T, cols)).astype(np.float32)
    xbig[:, :cols] = _dev(x)
    ybig = torch.full((T, rows + 7), -7.0, device="cuda")
    gpu_lib.fmt_gemv("q6_k", _dev(W), rows, cols, xbig[:, :cols], y=ybig[:, :rows])
    ref = oracle.fmt_gemv("q6_k", W, rows, cols, x.astype(np.float64))
    assert rel_err(ybig[:, :rows].cpu().numpy(), ref) < GEMV_TOL
    assert (ybig[:, rows:] == -7.0).all()


def test_gemv_argument_errors(gpu_lib):
    W = torch.zeros(gpu_lib.fmt_tensor_bytes("q8_0", 4, 256), dtype=torch.uint8, device="cuda")
    x = torch.zeros((1, 256), device="cuda")
    with pytest.raises(gpu_lib.PrimaError):
        gpu_lib.fmt_gemv("q8_0", W, 4, 256, torch.zeros((17, 256), device="cuda"))       # too many tokens
    with pytest.raises(gpu_lib.PrimaError):
        gpu_lib.fmt_gemv("q4_k", torch.zeros(4 * 144, dtype=torch.uint8, device="cuda"), 4, 256, x)   # has its own entry point
    with pytest.raises(ValueError):
        gpu_lib.fmt_gemv("q8_0", W[:-2], 4, 256, x)
    assert gpu_lib.fmt_tensor_bytes("q6_k", 4, 100) == 0


@pytest.mark.parametrize("fmt,T", [("q6_k", 1), ("q6_k", 8), ("q8_0", 3), ("f16", 1)])
def test_lm_head_in_another_format(gpu_lib, fmt, T):
    """Output layer: final RMSNorm fused in front of the mat-vec; vocabulary ragged against the row groups."""
    cfg = CONFIGS["c1"]
    d = cfg.dims
    vocab = 3001
    W = synth.fmt_tensor(cfg.config_id, 0, "w_lm", fmt, vocab, d.e)
    g = synth.gain_f32(cfg.config_id, 0, "g_final", d.e)
    x = (synth.normal_f32(cfg.config_id, 0, "x_in", (T, d.e)).astype(np.float64) * 1e3).astype(np.float32)
    ref = oracle.lm_head_fmt(d, fmt, g, W, vocab, x.astype(np.float64))
    got = gpu_lib.lm_head_fmt(d, fmt, _dev(g), _dev(W), vocab, _dev(x)).cpu().numpy()
    assert rel_err(got, ref) < 2e-3          # the hidden-state tolerance
    assert rel_err(got, ref) < 1e-4, rel_err(got, ref)


def test_lm_head_q6k_full_vocab_sampled(gpu_lib):
    """Config 4's output layer (128256 x 8192) in Q6_K, one token: logits sampled across the vocabulary and its
    ragged end recomputed one by one by a brute-force fp64 product on the dequantised rows."""
    cfg = CONFIGS["c4k1"]
    d = cfg.dims
    vocab = cfg.vocab
    W = synth.fmt_tensor(cfg.config_id, 0, "w_lm", "q6_k", vocab, d.e)
    g = synth.gain_f32(cfg.config_id, 0, "g_final", d.e)
    x = synth.normal_f32(cfg.config_id, 0, "x_in", (1, d.e))
    got = gpu_lib.lm_head_fmt(d, "q6_k", _dev(g), _dev(W), vocab, _dev(x)).cpu().numpy()[0]
    assert np.isfinite(got).all()
    rows = [0, 1, 2, 3, 4, 1023, 65535, 65536, 100000, vocab - 5, vocab - 4, vocab - 1]
    n = x[0].astype(np.float64)
    n = n / np.sqrt((n ** 2).mean() + float(np.float32(d.rms_eps))) * g.astype(np.float64)
    # rows one by one: a one-row tensor cut out of the planes
    nblk = d.e // 256
    N = vocab * nblk
    ref = []
    for r in rows:
        one = np.concatenate([W[r * nblk * 128:(r + 1) * nblk * 128], W[128 * N + r * nblk * 64:128 * N + (r + 1) * nblk * 64],
                              W[192 * N + r * nblk * 16:192 * N + (r + 1) * nblk * 16], W[208 * N + r * nblk * 2:208 * N + (r + 1) * nblk * 2]])
        ref.append(float(oracle.fmt_dequant("q6_k", one, 1, d.e)[0].astype(np.float64) @ n))
    ref = np.array(ref)
    scale = np.sqrt((ref ** 2).mean())
    assert np.abs(got[rows] - ref).max() / scale < 1e-4


MIXES = {
    # the usual mix of a "Q4K" model: V and down projections in Q6_K
    "q4_k_m": [{"wv": "q6_k", "wdown": "q6_k"}, {}, {"wv": "q6_k", "wdown": "q6_k"}],
    # every matrix in some other format, gate / up not both Q4_K (SwiGLU as its own launch), one Q4_K matrix alone in its group
    "all_kinds": [{"wq": "q8_0", "wk": "q5_k", "wv": "f16", "wo": "q6_k", "wgate": "q5_k", "wup": "q8_0", "wdown": "f32"},
                  {"wq": "q6_k", "wgate": "q6_k"},
                  {"wk": "q8_0", "wv": "q8_0", "wup": "f16", "wo": "f16", "wdown": "q5_k"}],
}


@pytest.mark.parametrize("mix", sorted(MIXES))
@pytest.mark.parametrize("name,T", [("t1", 1), ("t2", 5), ("c1", 4), ("c0", 11)])
def test_window_with_mixed_formats(gpu_lib, mix, name, T):
    """Three layers with matrices in several formats, one and several tokens (passes of 8 in the format mat-vec):
    hidden state against the oracle within the hidden-state tolerance; the appended K/V rows too."""
    n_layers = 3
    formats = MIXES[mix][-n_layers:]
    cfg = {**CONFIGS, **TINY}[name].with_(n_layers=n_layers, T=T)
    d = cfg.dims
    cap = cfg.n_past + T
    x = synth.window_input(cfg)
    host = [synth.layer_tensors(cfg, l, kv_cap=cap, formats=formats[l]) for l in range(n_layers)]
    dev_layers = [{k: _dev(v) for k, v in t.items()} for t in host]
    ref = oracle.window(d, host, x.astype(np.float64), cfg.n_past, formats=formats)     # appends to the host caches
    win = gpu_lib.Window(d, dev_layers, cap, T_max=T, formats=formats)
    win.workspace.fill_(0xFF)
    y = win.decode(_dev(x), cfg.n_past).cpu().numpy()
    err = rel_err(y, ref)
    print("mixed formats", mix, name, T, "hidden-state max rel err", err, flush=True)
    check_hidden(f"mixed {mix} {name} T={T}", err, d, host, x.astype(np.float64), cfg.n_past, formats=formats, eps=EPS_FP32)
    # the first layer's appended rows (deeper layers' rows inherit the hidden state's error)
    for c in ("k_cache", "v_cache"):
        new_ref = host[0][c][:, cfg.n_past:cfg.n_past + T].astype(np.float64).reshape(1, -1)
        new_got = dev_layers[0][c][:, cfg.n_past:cfg.n_past + T].float().cpu().numpy().reshape(1, -1)
        assert rel_err(new_got, new_ref) < 2e-3


def test_mixed_window_of_q4k_only_equals_the_q4k_window(gpu_lib):
    """With every format Q4_K the mixed entry point runs the same launches: identical bits."""
    cfg = CONFIGS["c1"].with_(n_layers=2)
    d = cfg.dims
    cap = cfg.n_past + cfg.T
    xd = _dev(synth.window_input(cfg))
    dev_layers = [{k: _dev(v) for k, v in synth.layer_tensors(cfg, l, kv_cap=cap).items()} for l in range(2)]
    a = gpu_lib.Window(d, dev_layers, cap, T_max=cfg.T).decode(xd, cfg.n_past).clone()
    b = gpu_lib.Window(d, dev_layers, cap, T_max=cfg.T, formats=[{}, {}]).decode(xd, cfg.n_past)
    assert torch.equal(a, b)


def test_mixed_window_full_shape(gpu_lib):
    """Config 3's layer shape, 4 layers, V and down projections in Q6_K (the usual mix), one token."""
    formats = [{"wv": "q6_k", "wdown": "q6_k"}] * 4
    cfg = CONFIGS["c3"].with_(n_layers=4)
    d = cfg.dims
    cap = cfg.n_past + cfg.T
    x = synth.window_input(cfg)
    dev_layers, h = [], x.astype(np.float64)
    for l in range(4):
        t = synth.layer_tensors(cfg, l, kv_cap=cap, formats=formats[l])
        dev_layers.append({k: _dev(v) for k, v in t.items()})
        h = oracle.layer(d, t, h, cfg.n_past, formats=formats[l])
        del t
    win = gpu_lib.Window(d, dev_layers, cap, T_max=cfg.T, formats=formats)
    win.workspace.fill_(0xFF)
    y = win.decode(_dev(x), cfg.n_past).cpu().numpy()
    check_hidden("config 3's shape, V and down in Q6_K", rel_err(y, h), d,
                 lambda: [synth.layer_tensors(cfg, l, kv_cap=cap, formats=formats[l]) for l in range(4)], x.astype(np.float64), cfg.n_past,
                 formats=formats, eps=EPS_FP32)


@pytest.mark.parametrize("name", ["t0", "t1", "t2"])
def test_batch_of_sequences_with_mixed_formats(gpu_lib, name):
    """One token for each of several sequences of different lengths (one empty, one full) through two layers whose
    matrices are in several formats: hidden states against the oracle (each sequence alone), appended rows."""
    formats = MIXES["all_kinds"][:2]
    cfg = TINY[name].with_(n_layers=2)
    d = cfg.dims
    lens = [0, 5, cfg.n_past, 17, 5]
    B = len(lens)
    cap = cfg.n_past + 1
    host = [synth.layer_tensors(cfg.with_(n_past=0), l, kv_cap=1, formats=formats[l]) for l in range(2)]
    dev_layers = [{k: _dev(v) for k, v in t.items()} for t in host]
    for dl in dev_layers:      # the window's own caches are not used by a batch
        dl["k_cache"] = torch.zeros((d.n_kv_heads, cap, d.head_dim), dtype=torch.float16, device="cuda")
        dl["v_cache"] = dl["k_cache"]
    caches = synth.batch_caches(cfg, 2, lens, cap)
    dev_caches = [[(_dev(k), _dev(v)) for k, v in per_layer] for per_layer in caches]
    xb = synth.batch_input(cfg, B)
    ref = oracle.window_batch(d, host, caches, xb.astype(np.float64), lens, formats=formats)     # appends to the host caches
    win = gpu_lib.Window(d, dev_layers, cap, T_max=B, formats=formats)
    win.workspace.fill_(0xFF)
    y = win.decode_batch(_dev(xb), lens, dev_caches).cpu().numpy()
    assert rel_err(y, ref) < 2e-3, rel_err(y, ref)
    for l in range(2):
        for b in range(B):
            for i in range(2):
                got = dev_caches[l][b][i][:, lens[b]].float().cpu().numpy().reshape(1, -1)
                want = caches[l][b][i][:, lens[b]].astype(np.float64).reshape(1, -1)
                assert rel_err(got, want) < 2e-3
