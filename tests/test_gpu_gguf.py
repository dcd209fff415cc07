"""GPU parity of the load-time conversion from GGUF block order (prima_repack_gguf, paper_2504_08791_amd/gguf.py).

The oracle's reading of the source bytes (oracle/interchange.py, pinned on the CPU) says what every weight is; the
library rearranges the same bytes on the device and dequantises its own layout: the two must agree bit for bit.
Then a window loaded from a (synthetic) file is advanced and compared with the oracle's window over the weights the
oracle read from the same file.  Source tensors are random bytes with finite binary16 scales of the benchmark's
range: every bit pattern is a valid block."""
import dataclasses
import os
import sys

import numpy as np
import pytest
import torch

sys.path.insert(0, os.path.dirname(__file__))
import oracle
from oracle import interchange as ix
import gguf_write
from tolerance import check_hidden, EPS_Q4K, EPS_FP32
from metrics import rel_err
from workloads.configs import TINY

pytestmark = pytest.mark.gpu

HALF_AT = {"q4_k": [(0, 144), (2, 144)], "q5_k": [(0, 176), (2, 176)], "q6_k": [(208, 210)], "q8_0": [(0, 34)]}


def source_tensor(fmt, rows, cols, seed, d_scale=1.0):
    """flat uint8: a rows x cols tensor in GGUF block order; random fields, scales uniform in [1e-3, 4e-3] * d_scale"""
    rng = np.random.default_rng(seed)
    if fmt in ("f16", "f32"):
        w = rng.standard_normal((rows, cols)).astype(np.float16 if fmt == "f16" else np.float32)
        return w.view(np.uint8).reshape(-1).copy()
    raw = rng.integers(0, 256, ix.tensor_bytes(fmt, rows, cols), dtype=np.uint8)
    for off, size in HALF_AT[fmt]:
        blk = raw.reshape(-1, size)
        h = (rng.uniform(1e-3, 4e-3, blk.shape[0]) * d_scale).astype(np.float16).view(np.uint16)
        blk[:, off] = h & 255
        blk[:, off + 1] = h >> 8
    return raw


@pytest.mark.parametrize("fmt", ["q4_k", "q5_k", "q6_k", "q8_0", "f16", "f32"])
@pytest.mark.parametrize("rows,cols", [(1, 256), (7, 768), (130, 2048)])
def test_repack_then_dequant_is_the_oracles_reading(gpu_lib, fmt, rows, cols):
    raw = source_tensor(fmt, rows, cols, seed=rows + cols)
    want = ix.dequant(fmt, raw, rows, cols)
    packed = gpu_lib.repack_gguf(fmt, torch.from_numpy(raw).cuda(), rows, cols)
    if fmt == "q4_k":
        got = gpu_lib.q4k_dequant(packed.view(rows, cols // 256, 144))
    else:
        got = gpu_lib.fmt_dequant(fmt, packed, rows, cols)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32)), (fmt, rows, cols)


def test_source_at_an_odd_address_and_overlap_refused(gpu_lib):
    from paper_2504_08791_amd import _ffi
    rows, cols = 5, 512
    raw = source_tensor("q6_k", rows, cols, seed=3)
    buf = torch.zeros(raw.size + 64, dtype=torch.uint8, device="cuda")
    buf[2:2 + raw.size] = torch.from_numpy(raw).cuda()          # 2-byte aligned only, as 210-byte blocks in a file are
    got = gpu_lib.fmt_dequant("q6_k", gpu_lib.repack_gguf("q6_k", buf[2:2 + raw.size], rows, cols), rows, cols)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), ix.dequant("q6_k", raw, rows, cols))
    n = raw.size
    big = torch.zeros(2 * n + 32, dtype=torch.uint8, device="cuda")
    rc = _ffi.lib().prima_repack_gguf(_ffi.FORMATS["q6_k"], big.data_ptr(), rows, cols, big.data_ptr() + 16, None)
    assert rc == 4                                              # overlapping buffers: refused, nothing launched
    rc = _ffi.lib().prima_repack_gguf(_ffi.FORMATS["q6_k"], big.data_ptr(), rows, cols, big.data_ptr() + (n + 15) // 16 * 16 + 8, None)
    assert rc == 3                                              # destination not 16-byte aligned


def test_mat_vec_over_a_repacked_q4k_tensor(gpu_lib):
    rows, cols, T = 200, 1024, 3
    raw = source_tensor("q4_k", rows, cols, seed=9)
    W = ix.dequant("q4_k", raw, rows, cols).astype(np.float64)
    x = np.random.default_rng(1).standard_normal((T, cols)).astype(np.float32)
    ref = x.astype(np.float64) @ W.T
    packed = gpu_lib.repack_gguf("q4_k", torch.from_numpy(raw).cuda(), rows, cols).view(rows, cols // 256, 144)
    y = gpu_lib.q4k_gemv(packed, torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    err = np.abs(y.cpu().numpy() - ref).max() / np.sqrt((ref ** 2).mean())
    assert err < 2e-6, err


@pytest.mark.parametrize("arch,mix", [("llama", {}), ("qwen2", {"attn_v": "q6_k", "ffn_down": "q6_k", "attn_output": "q5_k", "ffn_up": "q8_0"})])
def test_window_from_a_file(gpu_lib, tmp_path, arch, mix):
    from paper_2504_08791_amd import gguf
    cfg = TINY["t0"]
    d = cfg.dims
    n_layers, first, T, cap = 3, 1, 3, 8
    shapes = {"attn_q": (d.qd, d.e), "attn_k": (d.kvd, d.e), "attn_v": (d.kvd, d.e), "attn_output": (d.e, d.qd),
              "ffn_gate": (d.ffn, d.e), "ffn_up": (d.ffn, d.e), "ffn_down": (d.e, d.ffn)}
    rng = np.random.default_rng(5)
    tensors, seed = [], 100
    for l in range(n_layers):
        for name, (r, c) in shapes.items():
            fmt = mix.get(name, "q4_k")
            # the six-bit sub-scales of the K formats reach 63, signed bytes 127: scales chosen for weights of similar size
            scale = {"q4_k": 1.0, "q5_k": 0.5, "q6_k": 1.0 / 4, "q8_0": 4.0}[fmt]
            tensors.append((f"blk.{l}.{name}.weight", [c, r], fmt, source_tensor(fmt, r, c, seed, scale).tobytes()))
            seed += 1
        for name in ("attn_norm", "ffn_norm"):
            g = (1.0 + 0.1 * rng.standard_normal(d.e)).astype(np.float32)
            tensors.append((f"blk.{l}.{name}.weight", [d.e], "f32", g.tobytes()))
    meta = {"general.architecture": arch, f"{arch}.block_count": n_layers, f"{arch}.embedding_length": d.e,
            f"{arch}.attention.head_count": d.n_q_heads, f"{arch}.attention.head_count_kv": d.n_kv_heads,
            f"{arch}.feed_forward_length": d.ffn, f"{arch}.rope.freq_base": float(d.rope_theta),
            f"{arch}.attention.layer_norm_rms_epsilon": float(d.rms_eps), f"{arch}.attention.key_length": d.head_dim}
    path = str(tmp_path / "model.gguf")
    gguf_write.write(path, meta, tensors)

    field = dict(gguf.LAYER_MATRICES)
    with gguf.GGUFFile(path) as f:
        dims, layers, formats = f.load_window(first, n_layers - first, "cuda", cap)
        assert dims.rope_mode == (1 if arch == "llama" else 0)
        assert (dims.e, dims.n_q_heads, dims.n_kv_heads, dims.head_dim, dims.ffn) == (d.e, d.n_q_heads, d.n_kv_heads, d.head_dim, d.ffn)
        assert np.float32(dims.rope_theta) == np.float32(d.rope_theta) and np.float32(dims.rms_eps) == np.float32(d.rms_eps)
        od = dataclasses.replace(d, rope_mode=dims.rope_mode)       # the same dimensions, as the oracle takes them
        assert (formats is None) == (not mix)
        if mix:
            assert formats[0] == {field[k]: v for k, v in mix.items()}
        # the oracle's side: the weights as the oracle reads them from the file's bytes, kept as fp32 matrices
        host = []
        for l in range(first, n_layers):
            t = {}
            for name, (r, c) in shapes.items():
                t[field[name]] = ix.dequant(mix.get(name, "q4_k"), f.raw(f"blk.{l}.{name}.weight"), r, c).view(np.uint8).reshape(-1)
            t["g_attn"] = f.raw(f"blk.{l}.attn_norm.weight").view(np.float32).copy()
            t["g_ffn"] = f.raw(f"blk.{l}.ffn_norm.weight").view(np.float32).copy()
            t["k_cache"] = np.zeros((d.n_kv_heads, cap, d.head_dim), dtype=np.float16)
            t["v_cache"] = np.zeros((d.n_kv_heads, cap, d.head_dim), dtype=np.float16)
            host.append(t)
    x = rng.standard_normal((T, d.e)).astype(np.float32)
    win = gpu_lib.Window(dims, layers, cap, T_max=T, formats=formats)
    y = win.decode(torch.from_numpy(x).cuda(), 0)
    y2 = win.decode(torch.from_numpy(x[:1]).cuda(), T)      # one more token on top of the three cached ones
    torch.cuda.synchronize()
    all_f32 = [{k: "f32" for k in field.values()}] * len(host)
    ref = oracle.window(od, host, x.astype(np.float64), 0, formats=all_f32)
    ref2 = oracle.window(od, host, x[:1].astype(np.float64), T, formats=all_f32)
    eps = EPS_FP32 if mix else EPS_Q4K
    for got, want, xin, n_past in ((y, ref, x, 0), (y2, ref2, x[:1], T)):
        err = rel_err(got.cpu().numpy(), want)
        print("window from a file", arch, "n_past", n_past, "hidden-state max rel err", err, flush=True)
        check_hidden(f"window from a file {arch} n_past={n_past}", err, od, host, xin.astype(np.float64), n_past, formats=all_f32, eps=eps)
