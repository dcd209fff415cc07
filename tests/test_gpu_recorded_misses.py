"""The window cases that randomised runs once found outside the 2e-3 hidden-state bar, kept as tests, and seeded
sweeps over random shapes with no hand-picked list: every case passes at 2e-3 or is excused by the bound that
tests/tolerance.py computes from the oracle alone (printed when used).

Recorded cases (shapes and seeds as the runs drew them):
  decode   13 tokens on an empty cache, one layer, top-2 logit gap 0.89          (missed by 3.6e-3)
  mixed    8 tokens on an empty cache, one layer, K in FP32, V in FP16, ...      (5.5e-3)
  prompt   150 tokens on an empty cache, one layer, two shapes                   (4.4e-3 and 5.7e-3)
  prompt   100 tokens behind 16 cached rows, one layer (matrix-product route 2.3e-3, decode route 1.3e-3: token 20)
In all of them a K or V element of an appended row lies within two fp32 roundings of a binary16 rounding boundary
and the softmax that reads it is nearly tied.
"""
import numpy as np
import pytest
import torch

import oracle
import tolerance
from metrics import rel_err
from tolerance import EPS_FP32, EPS_GEMM, EPS_Q4K, check_hidden
from workloads import synth
from workloads.configs import ModelDims, WindowConfig

pytestmark = pytest.mark.gpu


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _oracle_any_T(dims, host, x, n_past, formats=None):
    return oracle.window_long(dims, host, x.astype(np.float64), n_past, formats=formats)


def test_recorded_decode_window(gpu_lib):
    cfg = WindowConfig("s333", 1233, ModelDims(2048, 8, 8, 128, 1280, 1e6, rope_mode=0), 1, 13, 0)
    cap = 15
    host = [synth.layer_tensors(cfg, 0, kv_cap=cap)]
    win = gpu_lib.Window(cfg.dims, [{k: _dev(v) for k, v in host[0].items()}], cap, T_max=13)
    x = synth.window_input(cfg)
    y = win.decode(_dev(x), 0).cpu().numpy()
    err = rel_err(y, _oracle_any_T(cfg.dims, host, x, 0))
    print("recorded decode window: err", err, flush=True)
    check_hidden("recorded decode window", err, cfg.dims, host, x.astype(np.float64), 0)


def test_recorded_mixed_format_window(gpu_lib):
    fm = {"wq": "q4_k", "wk": "f32", "wv": "f16", "wo": "q5_k", "wgate": "q4_k", "wup": "f16", "wdown": "q4_k"}
    cfg = WindowConfig("m71", 1271, ModelDims(3584, 8, 8, 64, 768, 5e5, rope_mode=0), 1, 8, 0)
    cap = 9
    host = [synth.layer_tensors(cfg, 0, kv_cap=cap, formats=fm)]
    win = gpu_lib.Window(cfg.dims, [{k: _dev(v) for k, v in host[0].items()}], cap, T_max=8, formats=[fm])
    x = synth.window_input(cfg)
    y = win.decode(_dev(x), 0).cpu().numpy()
    err = rel_err(y, _oracle_any_T(cfg.dims, host, x, 0, formats=[fm]))
    print("recorded mixed-format window: err", err, flush=True)
    check_hidden("recorded mixed-format window", err, cfg.dims, host, x.astype(np.float64), 0, formats=[fm], eps=EPS_FP32)


def _route_eps(gpu_lib, small_tokens, T):
    """The accuracy class of the projections on the route a prompt call of T tokens takes."""
    return EPS_Q4K if T <= small_tokens else EPS_GEMM


@pytest.mark.parametrize("small_tokens", [0, 64])
@pytest.mark.parametrize("cid,dims,T,n_past,cap", [(533, ModelDims(512, 20, 4, 128, 768, 1e4, rope_mode=1), 150, 0, 150),
                                                   (572, ModelDims(1024, 2, 1, 128, 1280, 1e4, rope_mode=1), 150, 0, 150),
                                                   (597, ModelDims(1024, 2, 1, 128, 1280, 1e4, rope_mode=0), 100, 16, 120)])
def test_recorded_prompt_calls(gpu_lib, cid, dims, T, n_past, cap, small_tokens):
    """Prompt tokens through the prompt call (both routes) and through decode calls of 16 tokens."""
    cfg = WindowConfig("p", cid, dims, 1, T, n_past)
    host = [synth.layer_tensors(cfg, 0, kv_cap=cap)]
    x = synth.window_input(cfg)
    ref = _oracle_any_T(dims, host, x, n_past)
    xd = _dev(x)
    gpu_lib.set_prefill_small_tokens(small_tokens)
    try:
        wa = gpu_lib.Window(dims, [{k: _dev(v) for k, v in host[0].items()}], cap, T_max=16)
        yp = wa.prefill(xd, n_past).cpu().numpy()
    finally:
        gpu_lib.set_prefill_small_tokens(gpu_lib.PREFILL_SMALL_TOKENS)
    wb = gpu_lib.Window(dims, [{k: _dev(v) for k, v in host[0].items()}], cap, T_max=16)
    yd = torch.cat([wb.decode(xd[t:t + 16].contiguous(), n_past + t) for t in range(0, T, 16)]).cpu().numpy()
    ep, ed = rel_err(yp, ref), rel_err(yd, ref)
    print(f"recorded prompt case {cid}: prompt call {ep:.3e}, decode calls {ed:.3e}", flush=True)
    check_hidden(f"recorded prompt case {cid}, prompt call", ep, dims, host, x.astype(np.float64), n_past,
                 eps=_route_eps(gpu_lib, small_tokens, T))
    check_hidden(f"recorded prompt case {cid}, decode calls", ed, dims, host, x.astype(np.float64), n_past)


def _random_dims(rng, heads, groups):
    while True:
        D, Hkv, G = int(rng.choice([64, 128])), int(rng.choice(heads)), int(rng.choice(groups))
        if (Hkv * G * D) % 256 == 0:
            break
    e = int(rng.choice([256, 512, 768, 1024, 1280, 1536, 2048, 2560, 3584]))
    ffn = int(rng.choice([256, 512, 768, 1280, 1536, 2816, 3584, 4864]))
    return ModelDims(e, Hkv * G, Hkv, D, ffn, float(rng.choice([1e4, 5e5, 1e6])), rope_mode=int(rng.integers(0, 2)))


@pytest.mark.timeout(900)
def test_sweep_of_decode_windows(gpu_lib):
    """60 windows of random shape, depth 1 to 4, every token count, cache lengths around the tile boundaries."""
    rng = np.random.default_rng(20250411)
    before = len(tolerance.excused)
    for n in range(60):
        dims = _random_dims(rng, [1, 2, 4, 8], [1, 2, 3, 4, 5, 7, 8])
        T, n_past, L = int(rng.integers(1, 17)), int(rng.choice([0, 1, 17, 63, 130, 400, 1025])), int(rng.integers(1, 5))
        cfg = WindowConfig("w%d" % n, 3000 + n, dims, L, T, n_past)
        cap = n_past + T + int(rng.integers(0, 3))
        host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(L)]
        win = gpu_lib.Window(dims, [{k: _dev(v) for k, v in t.items()} for t in host], cap, T_max=T)
        win.workspace.fill_(0xFF)
        x = synth.window_input(cfg)
        print("decode window", n, dims, "L", L, "T", T, "n_past", n_past, flush=True)
        y = win.decode(_dev(x), n_past).cpu().numpy()
        err = rel_err(y, oracle.window(dims, host, x.astype(np.float64), n_past))
        check_hidden(f"decode window {n}", err, dims, host, x.astype(np.float64), n_past)
    used = len(tolerance.excused) - before
    print("decode sweep: cases excused by the computed bound:", used, "of 60", flush=True)
    assert used <= 12      # the excuse is for the rare knife-edge case, not the rule


@pytest.mark.timeout(900)
def test_sweep_of_mixed_format_windows(gpu_lib):
    """40 windows of one to three layers with a random format per matrix."""
    rng = np.random.default_rng(20250412)
    names = ["wq", "wk", "wv", "wo", "wgate", "wup", "wdown"]
    before = len(tolerance.excused)
    for n in range(40):
        dims = _random_dims(rng, [1, 2, 4, 8], [1, 2, 3, 4, 5, 7, 8])
        T, n_past, L = int(rng.integers(1, 17)), int(rng.choice([0, 1, 17, 63, 130, 400])), int(rng.integers(1, 4))
        formats = [{nm: str(rng.choice(["q4_k", "q4_k", "q4_k", "q5_k", "q6_k", "q8_0", "f16", "f32"])) for nm in names} for _ in range(L)]
        cfg = WindowConfig("m%d" % n, 3200 + n, dims, L, T, n_past)
        cap = n_past + T + 1
        host = [synth.layer_tensors(cfg, l, kv_cap=cap, formats=formats[l]) for l in range(L)]
        win = gpu_lib.Window(dims, [{k: _dev(v) for k, v in t.items()} for t in host], cap, T_max=T, formats=formats)
        win.workspace.fill_(0xFF)
        x = synth.window_input(cfg)
        print("mixed window", n, dims, "L", L, "T", T, "n_past", n_past, flush=True)
        y = win.decode(_dev(x), n_past).cpu().numpy()
        err = rel_err(y, oracle.window(dims, host, x.astype(np.float64), n_past, formats=formats))
        check_hidden(f"mixed window {n}", err, dims, host, x.astype(np.float64), n_past, formats=formats, eps=EPS_FP32)
    used = len(tolerance.excused) - before
    print("mixed sweep: cases excused by the computed bound:", used, "of 40", flush=True)
    assert used <= 8


@pytest.mark.timeout(900)
@pytest.mark.parametrize("small_tokens", [0, 64])
def test_sweep_of_prompt_calls(gpu_lib, small_tokens):
    """40 prompt calls of random shape and length (1 to 150 tokens behind 0 to 200 rows, one or two layers), on the
    matrix-product route and on the default route."""
    rng = np.random.default_rng(20250413)
    before = len(tolerance.excused)
    gpu_lib.set_prefill_small_tokens(small_tokens)
    try:
        for n in range(40):
            dims = _random_dims(rng, [1, 2, 4], [1, 2, 4, 5, 8])
            dims = ModelDims(min(dims.e, 1024), dims.n_q_heads, dims.n_kv_heads, dims.head_dim, min(dims.ffn, 1280), 1e4, rope_mode=dims.rope_mode)
            T = int(rng.choice([1, 3, 16, 17, 31, 32, 33, 47, 64, 100, 150]))
            n_past, L = int(rng.choice([0, 1, 15, 16, 40, 200])), int(rng.integers(1, 3))
            cfg = WindowConfig("p%d" % n, 3400 + n, dims, L, T, n_past)
            cap = n_past + T + int(rng.integers(0, 5))
            host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(L)]
            win = gpu_lib.Window(dims, [{k: _dev(v) for k, v in t.items()} for t in host], cap, T_max=16)
            x = synth.window_input(cfg)
            print("prompt call", n, dims, "L", L, "T", T, "n_past", n_past, flush=True)
            y = win.prefill(_dev(x), n_past).cpu().numpy()
            err = rel_err(y, _oracle_any_T(dims, host, x, n_past))
            check_hidden(f"prompt call {n} (threshold {small_tokens})", err, dims, host, x.astype(np.float64), n_past,
                         eps=_route_eps(gpu_lib, small_tokens, T))
    finally:
        gpu_lib.set_prefill_small_tokens(gpu_lib.PREFILL_SMALL_TOKENS)
    used = len(tolerance.excused) - before
    print("prompt sweep: cases excused by the computed bound:", used, "of 40", flush=True)
    assert used <= 8
