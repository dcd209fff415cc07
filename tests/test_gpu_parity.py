"""GPU parity: every step of the HIP path against the CPU oracle on the same seeded inputs.

Bars: dequantisation bit-exact; hidden states / mat-vec outputs max relative error <= 2e-3;
attention outputs <= 1e-3 (error metric: tests/metrics.rel_err).
"""
import copy

import numpy as np
import pytest
import torch

import oracle
from metrics import rel_err
from tolerance import check_hidden
from q4k_pack import half_bits, pack_block
from workloads import synth
from workloads.configs import TINY, ModelDims

pytestmark = pytest.mark.gpu

HID_TOL = 2e-3
ATT_TOL = 1e-3


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _rand_q4k(rng, rows, nb):
    W = rng.integers(0, 256, size=(rows, nb, 144), dtype=np.uint8)
    dd = (1e-3 + 3e-3 * rng.random((rows * nb, 2), dtype=np.float32)).astype(np.float16)
    W.reshape(-1, 144)[:, 0:4] = dd.view(np.uint8).reshape(-1, 4)
    return W


def test_dequant_bit_exact_random(gpu_lib):
    rng = np.random.default_rng(0)
    for rows, nb in [(1, 1), (37, 3), (300, 5)]:
        W = _rand_q4k(rng, rows, nb)
        got = gpu_lib.q4k_dequant(_dev(W)).cpu().numpy()
        assert np.array_equal(got.view(np.uint32), oracle.dequant(W).view(np.uint32)), (rows, nb)


def test_dequant_bit_exact_any_half_scale(gpu_lib):
    """Arbitrary finite fp16 d / dmin, including subnormals and zero, and extreme fields."""
    rng = np.random.default_rng(1)
    W = rng.integers(0, 256, size=(64, 4, 144), dtype=np.uint8)
    flat = W.reshape(-1, 144)
    hb = rng.integers(0, 1 << 16, size=(flat.shape[0], 2)).astype(np.uint16)
    hb[(hb >> 10) & 31 == 31] &= 0x83ff           # no inf / nan
    flat[:, 0:4] = hb.view(np.uint8).reshape(-1, 4)
    flat[0] = pack_block(0, 0, [0] * 8, [0] * 8, [0] * 256)
    flat[1] = pack_block(half_bits(1.0), half_bits(0.5), [63] * 8, [63] * 8, [15] * 256)
    flat[2] = pack_block(1, 1, [63] * 8, [1] * 8, [15] * 256)      # smallest subnormal scales
    got = gpu_lib.q4k_dequant(_dev(W)).cpu().numpy()
    assert np.array_equal(got.view(np.uint32), oracle.dequant(W).view(np.uint32))


def test_dequant_empty(gpu_lib):
    W = torch.empty((0, 2, 144), dtype=torch.uint8, device="cuda")
    assert gpu_lib.q4k_dequant(W).shape == (0, 512)


@pytest.mark.parametrize("rows,nb,T", [(1, 1, 1), (7, 2, 1), (100, 5, 1), (257, 16, 1), (1030, 4, 1),
                                       (64, 3, 2), (100, 5, 4), (33, 6, 5), (96, 2, 8), (50, 3, 16), (130, 9, 3)])
def test_gemv_vs_oracle(gpu_lib, rows, nb, T):
    rng = np.random.default_rng(rows * 1000 + nb * 10 + T)
    W = _rand_q4k(rng, rows, nb)
    x = rng.standard_normal((T, nb * 256)).astype(np.float32)
    ref = oracle.gemv(W, x.astype(np.float64))
    got = gpu_lib.q4k_gemv(_dev(W), _dev(x)).cpu().numpy()
    assert rel_err(got, ref) < 1e-4, rel_err(got, ref)


def test_gemv_random_shapes(gpu_lib):
    """Shapes drawn at random (rows ragged against the 16-row tiles, odd and large numbers of super-blocks, every
    token count: one and several slabs of K, parts meeting in LDS or not, passes of up to 8 tokens), activations
    with a different scale per token: each against the oracle, and twice with identical bits."""
    rng = np.random.default_rng(2024)
    cases = []
    for _ in range(100):
        nb = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 20, 28, 32, 33, 56, 64, 100, 112, 120]))
        rows = int(rng.integers(1, max(1, min(9000, 6_000_000 // (nb * 256))) + 1))
        if rng.random() < 0.3:
            rows = max(1, rows // 16 * 16 + int(rng.choice([0, 1, 15])))
        cases.append((rows, nb, int(rng.choice([1, 1, 1, 2, 3, 4, 5, 7, 8, 9, 12, 16]))))
    cases += [(8192, 112, 1), (8192, 112, 8), (4096, 56, 4), (16, 120, 16), (1, 120, 8), (5000, 1, 16), (257, 33, 7)]
    for rows, nb, T in cases:
        W = _rand_q4k(rng, rows, nb)
        x = (rng.standard_normal((T, nb * 256)) * np.exp(3 * rng.standard_normal((T, 1)))).astype(np.float32)
        ref = oracle.gemv(W, x.astype(np.float64))
        Wd, xd = _dev(W), _dev(x)
        got = gpu_lib.q4k_gemv(Wd, xd).cpu().numpy()
        again = gpu_lib.q4k_gemv(Wd, xd).cpu().numpy()
        assert rel_err(got, ref) < 1e-4, (rows, nb, T, rel_err(got, ref))
        assert np.array_equal(got.view(np.uint32), again.view(np.uint32)), (rows, nb, T)


def test_gemv_short_last_slab_of_k(gpu_lib):
    """Many rows, K cut into slabs whose last one is much shorter than the others (25, 26, 33, 41, 57 super-blocks at 2 to
    4 tokens: slabs of 8, the last of 1 or 2): every workgroup of that slab takes many units.  (With K split further
    than the last slab's chunks these shapes once gave wrong sums: units without a chunk overran the unit queue.)"""
    rng = np.random.default_rng(99)
    for rows, nb, T in [(8000, 25, 3), (8000, 25, 2), (8000, 41, 4), (8000, 57, 2), (4000, 33, 3), (8000, 26, 4), (6000, 49, 2)]:
        print("case", rows, nb, T, flush=True)
        W = _rand_q4k(rng, rows, nb)
        x = rng.standard_normal((T, nb * 256)).astype(np.float32)
        ref = oracle.gemv(W, x.astype(np.float64))
        Wd, xd = _dev(W), _dev(x)
        got = gpu_lib.q4k_gemv(Wd, xd).cpu().numpy()
        again = gpu_lib.q4k_gemv(Wd, xd).cpu().numpy()
        assert rel_err(got, ref) < 1e-4, (rows, nb, T, rel_err(got, ref))
        assert np.array_equal(got.view(np.uint32), again.view(np.uint32)), (rows, nb, T)


def test_gemv_wide_dynamic_range(gpu_lib):
    """Activations like the SwiGLU output of the synthetic models: huge, common-mode, with outliers."""
    rng = np.random.default_rng(5)
    W = _rand_q4k(rng, 200, 8)
    for x in (1e7 * (1 + 0.01 * rng.standard_normal((2, 2048))),
              rng.standard_normal((2, 2048)) * np.exp(4 * rng.standard_normal((2, 2048))),
              np.zeros((1, 2048))):
        x = x.astype(np.float32)
        ref = oracle.gemv(W, x.astype(np.float64))
        got = gpu_lib.q4k_gemv(_dev(W), _dev(x)).cpu().numpy()
        if np.abs(ref).max() == 0:
            assert np.all(got == 0)
        else:
            assert rel_err(got, ref) < HID_TOL, rel_err(got, ref)


def test_gemv_integer_exact(gpu_lib):
    """Power-of-two scales and small integer x: every partial sum is exact in fp32, so any
    summation order must reproduce the oracle exactly."""
    rng = np.random.default_rng(3)
    rows, nb = 48, 4
    W = rng.integers(0, 256, size=(rows, nb, 144), dtype=np.uint8)
    for r in range(rows):
        for b in range(nb):
            W[r, b, 0:2] = np.frombuffer(int(half_bits(2.0 ** -(r % 3))).to_bytes(2, "little"), dtype=np.uint8)
            W[r, b, 2:4] = np.frombuffer(int(half_bits(2.0 ** -(b % 2 + 1))).to_bytes(2, "little"), dtype=np.uint8)
    x = rng.integers(-4, 5, size=(3, nb * 256)).astype(np.float32)
    ref = oracle.gemv(W, x.astype(np.float64))
    got = gpu_lib.q4k_gemv(_dev(W), _dev(x)).cpu().numpy().astype(np.float64)
    assert np.array_equal(got, ref)


def test_gemv_strided_io(gpu_lib):
    rng = np.random.default_rng(9)
    W = _rand_q4k(rng, 70, 2)
    xbig = rng.standard_normal((3, 640)).astype(np.float32)
    x = _dev(xbig)[:, :512]
    ybig = torch.full((3, 100), -7.0, device="cuda")
    import ctypes as C
    from paper_2504_08791_amd import _ffi
    ws = torch.empty(max(256, gpu_lib.gemv_workspace_bytes(70, 512, 3)), dtype=torch.uint8, device="cuda")
    Wd = _dev(W)
    rc = _ffi.lib().prima_q4k_gemv(Wd.data_ptr(), 70, 512, x.data_ptr(), 640, 3, ybig.data_ptr(), 100,
                                   ws.data_ptr(), ws.numel(), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    ref = oracle.gemv(W, xbig[:, :512].astype(np.float64))
    out = ybig.cpu().numpy()
    assert rel_err(out[:, :70], ref) < 1e-4 and np.all(out[:, 70:] == -7.0)


ATT_CASES = [  # Hq, Hkv, D, n_past, T
    (8, 2, 64, 37, 1), (10, 2, 128, 130, 4), (8, 1, 128, 0, 3), (4, 4, 64, 5, 2), (32, 8, 128, 512, 1),
    (40, 8, 128, 700, 5), (64, 8, 128, 1000, 1), (64, 8, 128, 300, 8), (8, 1, 128, 0, 1), (16, 2, 128, 2047, 16),
]


@pytest.mark.parametrize("Hq,Hkv,D,n_past,T", ATT_CASES)
def test_attention_vs_oracle(gpu_lib, Hq, Hkv, D, n_past, T):
    rng = np.random.default_rng(Hq * 7 + n_past + T)
    dims = ModelDims(Hq * D, Hq, Hkv, D, 256, 1e4)
    cap = n_past + T + 2
    K = rng.standard_normal((Hkv, cap, D)).astype(np.float16)
    V = rng.standard_normal((Hkv, cap, D)).astype(np.float16)
    K[:, n_past + T:] = np.float16(np.nan)    # rows beyond the step must never reach a result
    V[:, n_past + T:] = np.float16(np.nan)
    q = rng.standard_normal((T, Hq, D)).astype(np.float32)
    ref = oracle.attn_decode(dims, q.astype(np.float64), K, V, n_past, T)
    assert np.isfinite(ref).all()
    got = gpu_lib.attn_decode(dims, _dev(q), _dev(K), _dev(V), n_past).cpu().numpy()
    assert rel_err(got.reshape(T, -1), ref.reshape(T, -1)) < ATT_TOL


def test_attention_peaked_logits(gpu_lib):
    """Near one-hot softmax (logit spread of tens to thousands), as inside the synthetic layers."""
    rng = np.random.default_rng(77)
    Hq, Hkv, D, n_past, T = 16, 2, 128, 257, 3
    dims = ModelDims(Hq * D, Hq, Hkv, D, 256, 1e4)
    K = (rng.standard_normal((Hkv, n_past + T, D)) * 8).astype(np.float16)
    V = rng.standard_normal((Hkv, n_past + T, D)).astype(np.float16)
    q = (rng.standard_normal((T, Hq, D)) * 20).astype(np.float32)
    ref, gap = oracle.attn_decode(dims, q.astype(np.float64), K, V, n_past, T, return_gap=True)
    got = gpu_lib.attn_decode(dims, _dev(q), _dev(K), _dev(V), n_past).cpu().numpy()
    print("min top-2 logit gap", gap)
    assert rel_err(got.reshape(T, -1), ref.reshape(T, -1)) < ATT_TOL


def _window(gpu_lib, cfg, cap, layers_host):
    dev_layers = [{k: _dev(v) for k, v in t.items()} for t in layers_host]
    win = gpu_lib.Window(cfg.dims, dev_layers, cap, T_max=16)
    win.workspace.fill_(0xFF)      # NaN patterns: nothing may be read from the scratch before it is written
    return win, dev_layers


@pytest.mark.parametrize("name", ["t0", "t1", "t2"])
def test_layer_taps_vs_oracle(gpu_lib, name):
    cfg = TINY[name]
    cap = cfg.n_past + cfg.T
    host = [synth.layer_tensors(cfg, 0, kv_cap=cap)]
    win, dev_layers = _window(gpu_lib, cfg, cap, host)
    x = synth.window_input(cfg)
    ref, taps = oracle.layer(cfg.dims, host[0], x.astype(np.float64), cfg.n_past, taps=True)
    y, gt = win.decode_layer_taps(0, _dev(x), cfg.n_past)
    print(name, "oracle min top-2 gap", taps["min_gap"])
    assert rel_err(gt["q"].cpu().numpy(), taps["q"]) < HID_TOL
    assert rel_err(gt["o"].cpu().numpy(), taps["o"]) < ATT_TOL
    assert rel_err(gt["h"].cpu().numpy(), taps["h"]) < HID_TOL
    assert rel_err(gt["a"].cpu().numpy(), taps["a"]) < HID_TOL
    assert rel_err(y.cpu().numpy(), ref) < HID_TOL
    # appended fp16 rows: identical up to one fp16 ulp (rounding of values that differ in the last fp32 bits)
    for key in ("k_cache", "v_cache"):
        g = dev_layers[0][key].cpu().numpy().astype(np.float64)
        assert rel_err(g[:, cfg.n_past:cap].reshape(1, -1), host[0][key][:, cfg.n_past:cap].astype(np.float64).reshape(1, -1)) < 1e-3
        assert np.array_equal(g[:, :cfg.n_past], host[0][key][:, :cfg.n_past].astype(np.float64))


@pytest.mark.parametrize("name", ["t0", "t1", "t2"])
def test_window_vs_oracle(gpu_lib, name):
    cfg = TINY[name]
    cap = cfg.n_past + cfg.T + 3
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    win, _ = _window(gpu_lib, cfg, cap, host)
    x = synth.window_input(cfg)
    ref = oracle.window(cfg.dims, host, x.astype(np.float64), cfg.n_past)
    xd = _dev(x)
    y = win.decode(xd, cfg.n_past)
    assert rel_err(y.cpu().numpy(), ref) < HID_TOL
    # in place: x_out may alias x_in
    host2 = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    win2, _ = _window(gpu_lib, cfg, cap, host2)
    y2 = win2.decode(xd, cfg.n_past, x_out=xd)
    assert torch.equal(y2, y)


@pytest.mark.parametrize("name", ["t0", "t1", "t2"])
def test_batch_of_sequences_vs_oracle(gpu_lib, name):
    """One token for each of B sequences with their own caches and lengths (an empty one, a full one, equal
    ones): hidden states against the oracle's independent one-token steps, the appended rows, nothing else
    written, and the same bits on a second run."""
    cfg = TINY[name]
    cap = cfg.n_past + 6
    n_past = [0, cfg.n_past, cap - 1, 17, 17, 1, cfg.n_past + 3]
    B = len(n_past)
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    win, _ = _window(gpu_lib, cfg, cap, host)
    x = synth.batch_input(cfg, B)
    caches = synth.batch_caches(cfg, cfg.n_layers, n_past, cap)
    before = copy.deepcopy(caches)
    dev_caches = [[(_dev(k), _dev(v)) for k, v in per_layer] for per_layer in caches]
    ref = oracle.window_batch(cfg.dims, host, caches, x.astype(np.float64), n_past)
    y = win.decode_batch(_dev(x), n_past, dev_caches)
    assert rel_err(y.cpu().numpy(), ref) < HID_TOL
    for l in range(cfg.n_layers):
        for b in range(B):
            for got_d, want, old in zip(dev_caches[l][b], caches[l][b], before[l][b]):
                got = got_d.cpu().numpy()
                row = n_past[b]
                assert rel_err(got[:, row].astype(np.float64).reshape(1, -1), want[:, row].astype(np.float64).reshape(1, -1)) < 1e-3
                keep = np.ones(cap, dtype=bool)
                keep[row] = False
                assert np.array_equal(got[:, keep].view(np.uint16), old[:, keep].view(np.uint16))
    dev_again = [[(_dev(k), _dev(v)) for k, v in per_layer] for per_layer in before]
    y2 = win.decode_batch(_dev(x), n_past, dev_again)
    assert torch.equal(y, y2)


def test_batch_of_one_equals_single_sequence_step(gpu_lib):
    cfg = TINY["t1"]
    cap = cfg.n_past + 2
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    win, dev_layers = _window(gpu_lib, cfg, cap, host)
    x = _dev(synth.batch_input(cfg, 1))
    caches = [[(t["k_cache"].clone(), t["v_cache"].clone())] for t in dev_layers]
    yb = win.decode_batch(x, [cfg.n_past], caches)
    ys = win.decode(x, cfg.n_past)
    assert torch.equal(yb, ys)
    for t, per_layer in zip(dev_layers, caches):
        assert torch.equal(t["k_cache"], per_layer[0][0]) and torch.equal(t["v_cache"], per_layer[0][1])


@pytest.mark.parametrize("name", ["t0", "t1", "t2"])
def test_unwritten_cache_rows_may_hold_anything(gpu_lib, name):
    """Cache rows at and beyond n_past are not part of the context: filled with NaN patterns before the step, they
    must neither reach a result (one sequence: T tokens; and a batch of sequences) nor survive where the step
    appends."""
    cfg = TINY[name]
    cap = cfg.n_past + cfg.T + 20
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    x = synth.window_input(cfg)
    ref = oracle.window(cfg.dims, copy.deepcopy(host), x.astype(np.float64), cfg.n_past)
    nan16 = np.uint16(0x7E00)
    for t in host:
        for key in ("k_cache", "v_cache"):
            t[key].view(np.uint16)[:, cfg.n_past:] = nan16
    win, dev_layers = _window(gpu_lib, cfg, cap, host)
    y = win.decode(_dev(x), cfg.n_past).cpu().numpy()
    assert np.isfinite(y).all() and rel_err(y, ref) < HID_TOL
    for t in dev_layers:
        for key in ("k_cache", "v_cache"):
            rows = t[key][:, cfg.n_past:cfg.n_past + cfg.T].cpu().numpy()
            assert np.isfinite(rows.astype(np.float32)).all()
    lens = [0, cfg.n_past, 5][:max(1, min(3, cfg.T))] if cfg.T > 1 else [cfg.n_past]
    caches = synth.batch_caches(cfg, cfg.n_layers, lens, cap)
    refb = oracle.window_batch(cfg.dims, host, copy.deepcopy(caches), synth.batch_input(cfg, len(lens)).astype(np.float64), lens)
    for per_layer in caches:
        for b, (k, v) in enumerate(per_layer):
            k.view(np.uint16)[:, lens[b]:] = nan16
            v.view(np.uint16)[:, lens[b]:] = nan16
    dev_caches = [[(_dev(k), _dev(v)) for k, v in per_layer] for per_layer in caches]
    yb = win.decode_batch(_dev(synth.batch_input(cfg, len(lens))), lens, dev_caches).cpu().numpy()
    assert np.isfinite(yb).all() and rel_err(yb, refb) < HID_TOL


def test_joint_equals_sequential_on_gpu(gpu_lib):
    cfg = TINY["t1"]
    cap = cfg.n_past + cfg.T
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    wj, _ = _window(gpu_lib, cfg, cap, host)
    ws, _ = _window(gpu_lib, cfg, cap, copy.deepcopy(host))
    x = _dev(synth.window_input(cfg))
    yj = wj.decode(x, cfg.n_past).cpu().numpy()
    ys = np.stack([ws.decode(x[j:j + 1].contiguous(), cfg.n_past + j).cpu().numpy()[0] for j in range(cfg.T)])
    assert rel_err(yj, ys) < HID_TOL


def test_rewind_on_gpu(gpu_lib):
    cfg = TINY["t1"]
    d = cfg.dims
    cap = cfg.n_past + 8
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(2)]
    wa, _ = _window(gpu_lib, cfg, cap, host)
    wb, _ = _window(gpu_lib, cfg, cap, copy.deepcopy(host))
    x4 = _dev(synth.window_input(cfg))
    xb = _dev(synth.normal_f32(cfg.config_id, 1, "x_in", (2, d.e)))
    wa.decode(x4, cfg.n_past)
    ya = wa.decode(xb, cfg.n_past + 2)
    wb.decode(x4[:2].contiguous(), cfg.n_past)
    yb = wb.decode(xb, cfg.n_past + 2)
    assert torch.equal(ya, yb)


def test_rerun_is_bit_identical(gpu_lib):
    """No float atomics anywhere: the same step twice gives the same bits."""
    cfg = TINY["t2"]
    cap = cfg.n_past + cfg.T
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    win, _ = _window(gpu_lib, cfg, cap, host)
    x = _dev(synth.window_input(cfg))
    a = win.decode(x, cfg.n_past).clone()
    b = win.decode(x, cfg.n_past)
    assert torch.equal(a, b)


@pytest.mark.parametrize("name", ["t0", "t1", "t2"])
def test_profiled_step_leaves_what_a_plain_step_leaves(gpu_lib, name):
    """The measurement hook replays each kind of launch on its own; afterwards x_out and every layer's caches
    (the step's new rows included) must be bit-equal to those after prima_layer_window_decode, so that a caller
    who advances n_past after it attends over the right rows."""
    cfg = TINY[name]
    cap = cfg.n_past + cfg.T + 2
    host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
    wa, la = _window(gpu_lib, cfg, cap, host)
    wb, lb = _window(gpu_lib, cfg, cap, copy.deepcopy(host))
    x = _dev(synth.window_input(cfg))
    ya = wa.decode(x, cfg.n_past)
    yb, kinds = wb.decode_profiled(x, cfg.n_past)
    assert torch.equal(ya, yb)
    assert kinds["gate_up"][1] == cfg.n_layers
    for a, b in zip(la, lb):
        assert torch.equal(a["k_cache"], b["k_cache"]) and torch.equal(a["v_cache"], b["v_cache"])
    # the next step, which attends over the rows the profiled step appended
    x2 = _dev(synth.normal_f32(cfg.config_id, 1, "x_in", (1, cfg.dims.e)))
    assert torch.equal(wa.decode(x2, cfg.n_past + cfg.T), wb.decode(x2, cfg.n_past + cfg.T))


def test_attention_random_shapes(gpu_lib):
    """Head counts (groups of 1 to 16 queries per KV head, not only powers of two), both head sizes, context
    lengths around the tile and key-range boundaries and token counts drawn at random."""
    rng = np.random.default_rng(7)
    n = 0
    while n < 50:
        D, Hkv, G = int(rng.choice([64, 128])), int(rng.choice([1, 2, 3, 4, 8])), int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16]))
        Hq = Hkv * G
        if (Hq * D) % 256:
            continue
        T = int(rng.choice([1, 1, 2, 3, 4, 7, 8, 13, 16]))
        n_past = int(rng.choice([0, 1, 15, 16, 17, 100, 127, 128, 129, 500, 1023, 3000]))
        dims = ModelDims(Hq * D, Hq, Hkv, D, 256, 1e4)
        cap = n_past + T + int(rng.integers(0, 3))
        K = rng.standard_normal((Hkv, cap, D)).astype(np.float16)
        V = rng.standard_normal((Hkv, cap, D)).astype(np.float16)
        K[:, n_past + T:] = np.float16(np.nan)
        V[:, n_past + T:] = np.float16(np.nan)
        q = (rng.standard_normal((T, Hq, D)) * float(np.exp(rng.standard_normal()))).astype(np.float32)
        ref = oracle.attn_decode(dims, q.astype(np.float64), K, V, n_past, T)
        got = gpu_lib.attn_decode(dims, _dev(q), _dev(K), _dev(V), n_past).cpu().numpy()
        assert rel_err(got.reshape(T, -1), ref.reshape(T, -1)) < ATT_TOL, (Hq, Hkv, D, n_past, T)
        n += 1


def test_window_random_shapes(gpu_lib):
    """Small windows of random shape (widths, FFN sizes with odd numbers of tiles and super-blocks, head layouts,
    both RoPE pairings, 1 to 3 layers, every token count), as T tokens of one sequence and as a batch of T
    sequences of random lengths over the same weights."""
    from workloads.configs import WindowConfig
    rng = np.random.default_rng(11)
    n = 0
    while n < 30:
        D, Hkv, G = int(rng.choice([64, 128])), int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 3, 4, 5, 8]))
        Hq = Hkv * G
        if (Hq * D) % 256:
            continue
        e, ffn = int(rng.choice([256, 512, 768, 1024, 1280, 2048])), int(rng.choice([256, 512, 768, 1280, 1536, 2816, 3584]))
        T, n_past = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16])), int(rng.choice([0, 1, 17, 63, 130, 400]))
        dims = ModelDims(e, Hq, Hkv, D, ffn, float(rng.choice([1e4, 5e5, 1e6])), rope_mode=int(rng.integers(0, 2)))
        cfg = WindowConfig("r%d" % n, 600 + n, dims, int(rng.integers(1, 4)), T, n_past)
        cap = n_past + T + 2
        host = [synth.layer_tensors(cfg, l, kv_cap=cap) for l in range(cfg.n_layers)]
        win, _ = _window(gpu_lib, cfg, cap, host)
        x = synth.window_input(cfg)
        ref = oracle.window(dims, host, x.astype(np.float64), n_past)
        print("random window", n, dims, cfg.n_layers, T, n_past, flush=True)
        check_hidden(f"random window {n}", rel_err(win.decode(_dev(x), n_past).cpu().numpy(), ref), dims, host, x.astype(np.float64), n_past)
        lens = [int(rng.integers(0, cap)) for _ in range(T)]
        caches = synth.batch_caches(cfg, cfg.n_layers, lens, cap)
        dev_caches = [[(_dev(k), _dev(v)) for k, v in per_layer] for per_layer in caches]
        xb = synth.batch_input(cfg, T)
        refb = oracle.window_batch(dims, host, caches, xb.astype(np.float64), lens)
        assert rel_err(win.decode_batch(_dev(xb), lens, dev_caches).cpu().numpy(), refb) < HID_TOL, (cfg, lens)
        n += 1


def test_lm_head_vs_oracle(gpu_lib):
    cfg = TINY["t0"].with_(vocab=1000)
    out = synth.output_layer_tensors(cfg)
    x = synth.window_input(cfg)
    ref = oracle.lm_head(cfg.dims, out["g_final"], out["w_lm"], x.astype(np.float64))
    got = gpu_lib.lm_head(cfg.dims, _dev(out["g_final"]), _dev(out["w_lm"]), _dev(x)).cpu().numpy()
    assert rel_err(got, ref) < HID_TOL
