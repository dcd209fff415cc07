"""GPU parity of prompt processing (all layers of a window for T consecutive tokens in one call) against the CPU
oracle, through the C ABI.

The oracle advances at most 64 tokens a call; a prompt goes through it in such pieces, each through all layers
(the layers' caches carry what the earlier pieces appended), which is the same causal computation.
Bar: hidden states max relative error <= 2e-3 (tests/metrics.rel_err), appended cache rows within one fp16 step.
"""
import copy

import numpy as np
import pytest
import torch

import oracle
from metrics import rel_err
from tolerance import EPS_FP32, EPS_GEMM, EPS_Q4K, check_hidden
from workloads import synth
from workloads.configs import CONFIGS, TINY

pytestmark = pytest.mark.gpu

HID_TOL = 2e-3
# the accuracy class of the prompt call's matrix product, asserted on the products themselves in tests/test_gpu_gemm.py
PREFILL_EPS = EPS_GEMM


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _oracle_prompt(dims, host, x, n_past, formats=None):
    out = []
    for t0 in range(0, x.shape[0], 64):
        out.append(oracle.window(dims, host, x[t0:t0 + 64].astype(np.float64), n_past + t0, formats=formats))
    return np.concatenate(out, axis=0)


DECODE_ROUTE = 64   # a threshold that sends these tests' short prompts through the decode kernels (the default is 16)


@pytest.fixture(params=["matrix product", "decode kernels"])
def route(request, gpu_lib):
    """The prompt call's two routes: always the matrix product (threshold 0), or prompts of up to 64 tokens advanced by
    the decode kernels, 16 tokens a call (the library's default does that up to 16 tokens)."""
    gpu_lib.set_prefill_small_tokens(0 if request.param == "matrix product" else DECODE_ROUTE)
    yield request.param
    gpu_lib.set_prefill_small_tokens(gpu_lib.PREFILL_SMALL_TOKENS)


@pytest.fixture
def matrix_product_route(gpu_lib):
    gpu_lib.set_prefill_small_tokens(0)
    yield
    gpu_lib.set_prefill_small_tokens(gpu_lib.PREFILL_SMALL_TOKENS)


def _window(gpu_lib, cfg, cap, host):
    dev_layers = [{k: _dev(v) for k, v in t.items()} for t in host]
    return gpu_lib.Window(cfg.dims, dev_layers, cap, T_max=16), dev_layers


@pytest.mark.parametrize("name,T,n_past", [("t0", 50, 37), ("t1", 70, 0), ("t2", 33, 63), ("t0", 1, 5), ("t1", 16, 130), ("t0", 150, 37),
                                           ("t2", 129, 63)])
def test_prefill_vs_oracle(gpu_lib, route, name, T, n_past):
    cfg = TINY[name].with_(T=T, n_past=n_past)
    cap = n_past + T + 3
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    win, dev_layers = _window(gpu_lib, cfg, cap, host)
    x = synth.window_input(cfg)
    print("case", name, T, n_past, flush=True)
    y = win.prefill(_dev(x), n_past).cpu().numpy()
    ref = _oracle_prompt(cfg.dims, host, x, n_past)       # appends to the host caches
    check_hidden(f"prefill {name} T={T} n_past={n_past} ({route})", rel_err(y, ref), cfg.dims, host, x.astype(np.float64), n_past,
                 eps=PREFILL_EPS)
    for l in range(cfg.n_layers):
        for key in ("k_cache", "v_cache"):
            g = dev_layers[l][key].cpu().numpy().astype(np.float64)
            r = host[l][key].astype(np.float64)
            assert np.array_equal(g[:, :n_past], r[:, :n_past])
            assert np.array_equal(g[:, n_past + T:], r[:, n_past + T:])
            if l == 0:   # deeper layers' rows inherit the hidden states' error
                assert rel_err(g[:, n_past:n_past + T].reshape(1, -1), r[:, n_past:n_past + T].reshape(1, -1)) < 1e-3


def test_prefill_fills_the_cache_to_its_last_row(gpu_lib, route):
    """n_past + T == kv_cap: the last piece ends on the cache's last row; a token count with full pieces only and one
    with a rest."""
    for T, n_past in [(32, 5), (45, 0)]:
        cfg = TINY["t0"].with_(T=T, n_past=n_past)
        cap = n_past + T
        host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
        win, dev_layers = _window(gpu_lib, cfg, cap, host)
        x = synth.window_input(cfg)
        print("case", T, n_past, flush=True)
        y = win.prefill(_dev(x), n_past).cpu().numpy()
        ref = _oracle_prompt(cfg.dims, host, x, n_past)
        assert rel_err(y, ref) < HID_TOL, rel_err(y, ref)
        g = dev_layers[0]["k_cache"].cpu().numpy().astype(np.float64)
        assert rel_err(g[:, n_past:].reshape(1, -1), host[0]["k_cache"][:, n_past:].astype(np.float64).reshape(1, -1)) < 1e-3


MIXES = {
    # the usual mix of a "Q4K" model: V and down projections in Q6_K
    "q4_k_m": [{"wv": "q6_k", "wdown": "q6_k"}, {}, {"wv": "q6_k", "wdown": "q6_k"}],
    # every matrix in some other format, gate / up not both Q4_K (SwiGLU as its own launch), Q4_K matrices alone in their groups
    "all_kinds": [{"wq": "q8_0", "wk": "q5_k", "wv": "f16", "wo": "q6_k", "wgate": "q5_k", "wup": "q8_0", "wdown": "f32"},
                  {"wq": "q6_k", "wgate": "q6_k"},
                  {"wk": "q8_0", "wv": "q8_0", "wup": "f16", "wo": "f16", "wdown": "q5_k"}],
}


@pytest.mark.parametrize("mix", sorted(MIXES))
@pytest.mark.parametrize("name,T,n_past", [("t1", 37, 130), ("t2", 16, 63), ("t0", 70, 37), ("t1", 37, 9), ("t2", 100, 0)])
def test_prefill_with_mixed_formats(gpu_lib, route, mix, name, T, n_past):
    """Layers whose matrices are in several formats (Q4_K ones through the matrix product, the others 16 tokens a launch
    through the format mat-vec): hidden state and appended rows against the oracle.  (With 37 tokens behind 9 rows the
    first of these mixes has top-2 logit gaps of 0.03 to 0.1 in every layer: a case for the computed bound.)"""
    base = TINY[name]
    formats = MIXES[mix][-base.n_layers:]
    cfg = base.with_(T=T, n_past=n_past)
    cap = n_past + T + 1
    host = [synth.layer_tensors(cfg, l, kv_cap=cap, formats=formats[l]) for l in range(cfg.n_layers)]
    dev_layers = [{k: _dev(v) for k, v in t.items()} for t in host]
    win = gpu_lib.Window(cfg.dims, dev_layers, cap, T_max=16, formats=formats)
    x = synth.window_input(cfg)
    print("case", mix, name, T, n_past, flush=True)
    y = win.prefill(_dev(x), n_past).cpu().numpy()
    ref = _oracle_prompt(cfg.dims, host, x, n_past, formats)
    check_hidden(f"prefill mixed {mix} {name} T={T} n_past={n_past} ({route})", rel_err(y, ref), cfg.dims, host, x.astype(np.float64), n_past,
                 formats=formats, eps=EPS_FP32)
    g = dev_layers[0]["v_cache"].cpu().numpy().astype(np.float64)
    r = host[0]["v_cache"].astype(np.float64)
    assert rel_err(g[:, n_past:n_past + T].reshape(1, -1), r[:, n_past:n_past + T].reshape(1, -1)) < 1e-3


def test_prefill_then_decode_continues(gpu_lib, route):
    """A prompt through the prefill call, the next token through the decode call: against the oracle doing the same."""
    cfg = TINY["t1"].with_(T=40, n_past=0)
    cap = 48
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    win, _ = _window(gpu_lib, cfg, cap, host)
    x = synth.window_input(cfg)
    nxt = synth.batch_input(cfg, 1)
    win.prefill(_dev(x), 0)
    y = win.decode(_dev(nxt), 40).cpu().numpy()
    _oracle_prompt(cfg.dims, host, x, 0)
    ref = oracle.window(cfg.dims, host, nxt.astype(np.float64), 40)
    assert rel_err(y, ref) < HID_TOL, rel_err(y, ref)


def test_prefill_agrees_with_decode_calls(gpu_lib, matrix_product_route):
    """The same prompt through decode calls of 16 tokens (integer-digit mat-vec) and through one prefill call
    (binary16 matrix product): far inside the bar of each other, and prefill gives the same bits twice, in place too.
    With the threshold above its length the prompt is advanced by the decode kernels: the same bits as the decode calls."""
    cfg = TINY["t2"].with_(T=48, n_past=10)
    cap = 64
    x = synth.window_input(cfg)
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    wa, _ = _window(gpu_lib, cfg, cap, copy.deepcopy(host))
    wb, _ = _window(gpu_lib, cfg, cap, copy.deepcopy(host))
    wc, _ = _window(gpu_lib, cfg, cap, copy.deepcopy(host))
    xd = _dev(x)
    ya = torch.cat([wa.decode(xd[t:t + 16].contiguous(), 10 + t) for t in range(0, 48, 16)]).cpu().numpy()
    yb = wb.prefill(xd, 10)
    assert rel_err(yb.cpu().numpy(), ya.astype(np.float64)) < HID_TOL / 4
    xc = xd.clone()
    yc = wc.prefill(xc, 10, x_out=xc)
    assert torch.equal(yb, yc)
    gpu_lib.set_prefill_small_tokens(DECODE_ROUTE)
    wd, _ = _window(gpu_lib, cfg, cap, copy.deepcopy(host))
    assert np.array_equal(wd.prefill(xd, 10).cpu().numpy(), ya)
    gpu_lib.set_prefill_small_tokens(gpu_lib.PREFILL_SMALL_TOKENS)


@pytest.mark.parametrize("T", [80, 40])
def test_prefill_model_shape_one_layer(gpu_lib, matrix_product_route, T):
    """One 70B-shaped layer (config 3's dimensions), 80 or 40 prompt tokens behind 4000 cached rows.  At these token counts
    the Q/K/V, output and down products divide K among workgroups (6 or 8 shares), at 40 tokens the gate / up product does
    too (2 shares, SwiGLU behind the addition)."""
    cfg = CONFIGS["c3"].with_(T=T, n_past=4000, n_layers=1)
    cap = 4096
    host = [synth.layer_tensors(cfg, 0, kv_cap=cap)]
    win, _ = _window(gpu_lib, cfg, cap, host)
    x = synth.window_input(cfg)
    print(f"case c3 one layer, {T} tokens", flush=True)
    y = win.prefill(_dev(x), 4000).cpu().numpy()
    ref = _oracle_prompt(cfg.dims, host, x, 4000)
    assert rel_err(y, ref) < HID_TOL, rel_err(y, ref)


def test_prefill_at_the_largest_token_count(gpu_lib):
    """8192 prompt tokens (the call's limit) through one 8B-shaped layer, filling the cache to its last row.  The oracle
    would take hours; checked instead: the first 8176 tokens' outputs are, bit for bit, those of a call with only them
    (no result depends on how many tokens a call has), the last 16 agree with a decode call behind that shorter prompt,
    and the last appended cache rows are the same."""
    cfg = CONFIGS["c0"].with_(T=8192, n_past=0, n_layers=1)
    cap = 8192
    host = [synth.layer_tensors(cfg, 0, kv_cap=cap)]
    x = _dev(synth.window_input(cfg))
    wa, la = _window(gpu_lib, cfg, cap, host)
    wb, lb = _window(gpu_lib, cfg, cap, host)
    print("case c0 one layer, 8192 tokens", flush=True)
    ya = wa.prefill(x, 0)
    yb = wb.prefill(x[:8176].contiguous(), 0)
    yc = wb.decode(x[8176:].contiguous(), 8176)
    assert torch.isfinite(ya).all()
    assert torch.equal(ya[:8176], yb)
    # (a K or V element that rounds to the other fp16 neighbour in one of the two paths moves that token by up to ~1e-3;
    # the others agree to 1e-6)
    per_token = [rel_err(ya[8176 + t].cpu().numpy(), yc[t].cpu().numpy().astype(np.float64)) for t in range(16)]
    assert max(per_token) < HID_TOL and float(np.median(per_token)) < 1e-5, per_token
    for key in ("k_cache", "v_cache"):
        a = la[0][key][:, 8176:].float().cpu().numpy().reshape(1, -1)
        b = lb[0][key][:, 8176:].float().cpu().numpy().astype(np.float64).reshape(1, -1)
        assert rel_err(a, b) < 1e-3
        assert torch.equal(la[0][key][:, :8176], lb[0][key][:, :8176])


def test_prefill_argument_errors(gpu_lib):
    from paper_2504_08791_amd import _ffi
    import ctypes as C
    cfg = TINY["t0"]
    cap = 64
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    win, _ = _window(gpu_lib, cfg, cap, host)
    L = _ffi.lib()
    x = torch.zeros((8, cfg.dims.e), dtype=torch.float32, device="cuda")
    need = L.prima_prefill_workspace_bytes(C.byref(win.dims), cap, 8)
    assert need > 0 and L.prima_prefill_workspace_bytes(C.byref(win.dims), cap, 0) == 0
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    call = lambda **k: L.prima_layer_window_prefill(C.byref(win.dims), win._arr, k.get("L", 2), cap, k.get("n_past", 0), k.get("T", 8),
                                                    k.get("x", x.data_ptr()), x.data_ptr(), ws.data_ptr(), k.get("wsb", need), None)
    assert _ffi.STATUS[call(x=None)] == "PRIMA_E_NULL"
    assert _ffi.STATUS[call(T=0)] == "PRIMA_E_RANGE"
    assert _ffi.STATUS[call(n_past=60)] == "PRIMA_E_RANGE"
    assert _ffi.STATUS[call(L=0)] == "PRIMA_E_RANGE"
    assert _ffi.STATUS[call(wsb=need - 256)] == "PRIMA_E_WORKSPACE"
    assert _ffi.STATUS[call(x=x.data_ptr() + 4)] == "PRIMA_E_ALIGN"
    assert call() == 0
    torch.cuda.synchronize()
