"""Seeded generators for the synthetic tensors of a layer window.

Every tensor is drawn from its own Philox stream keyed by
(BASE_SEED, config_id, layer, tensor_id), so any tensor can be regenerated on
its own (one layer at a time for the large windows) and the result does not
depend on the order of generation.

A Q4_K tensor is produced as raw bytes: every 6-bit and 4-bit field of a
super-block is uniform over its whole range, so filling bytes 4..143 of each
144-byte super-block with uniform random bytes gives exactly that
distribution whatever the bit packing is; only the two fp16 values at bytes
0..3 (d, dmin uniform in [1e-3, 4e-3]) are written as numbers.  No packing or
decoding logic lives here.
"""
import numpy as np

BASE_SEED = 0x5052494D41  # fixed
QK = 256                  # weights per super-block
BLOCK_BYTES = 144

TENSOR_IDS = {
    "wq": 0, "wk": 1, "wv": 2, "wo": 3, "wgate": 4, "wup": 5, "wdown": 6,
    "g_attn": 7, "g_ffn": 8, "k_cache": 9, "v_cache": 10, "x_in": 11,
    "g_final": 12, "w_lm": 13, "q": 14, "x_in_batch": 15,
}
SEQ_CACHE_ID0 = 100  # K, V caches of sequence b of a batch: ids 100 + 2b, 101 + 2b


def _rng(config_id, layer, tensor):
    tid = TENSOR_IDS[tensor] if isinstance(tensor, str) else int(tensor)
    ss = np.random.SeedSequence([BASE_SEED, int(config_id), int(layer), tid])
    return np.random.Generator(np.random.Philox(ss))


def q4k_tensor(config_id, layer, tensor, n_rows, n_cols):
    """uint8 [n_rows, n_cols/256, 144]: row-major rows of 144-byte super-blocks."""
    assert n_cols % QK == 0
    nb = n_rows * (n_cols // QK)
    rng = _rng(config_id, layer, tensor)
    n64 = nb * BLOCK_BYTES // 8
    raw = rng.bit_generator.random_raw(n64).view(np.uint8).reshape(nb, BLOCK_BYTES)
    u = rng.random((nb, 2), dtype=np.float32)
    dd = (np.float32(1e-3) + np.float32(3e-3) * u).astype(np.float16)
    raw[:, 0:4] = dd.view(np.uint8).reshape(nb, 4)
    return raw.reshape(n_rows, n_cols // QK, BLOCK_BYTES)


FORMAT_BITS = {"q4_k": 4.5, "q5_k": 5.5, "q6_k": 6.5625, "q8_0": 8.5, "f16": 16, "f32": 32}


def fmt_tensor(config_id, layer, tensor, fmt, n_rows, n_cols):
    """Flat uint8 tensor in one of the other weight formats (planes one after the other; see the layout
    text of the format).  As for Q4_K every quant, sub-scale and sub-min field is uniform over its whole
    range, which uniform random bytes give whatever the bit placement; only the binary16 scales are written
    as numbers (at their byte positions, uniform in a range that keeps weights of the order of 0.1)."""
    assert n_cols % QK == 0
    rng = _rng(config_id, layer, tensor)
    n = n_rows * (n_cols // QK)
    if fmt == "q4_k":
        return q4k_tensor(config_id, layer, tensor, n_rows, n_cols).reshape(-1)
    if fmt in ("f16", "f32"):
        w = (0.05 * rng.standard_normal((n_rows, n_cols), dtype=np.float32))
        return w.astype(np.float16 if fmt == "f16" else np.float32).view(np.uint8).reshape(-1)
    nbytes = int(n * QK * FORMAT_BITS[fmt] / 8)
    raw = rng.bit_generator.random_raw((nbytes + 7) // 8).view(np.uint8)[:nbytes].copy()

    def scales(count, lo, hi):
        u = rng.random(count, dtype=np.float32)
        return (np.float32(lo) + np.float32(hi - lo) * u).astype(np.float16).view(np.uint8)

    if fmt == "q5_k":     # d, dmin: bytes 0..3 of every 16-byte header (first plane)
        raw[:16 * n].reshape(n, 16)[:, 0:4] = scales(2 * n, 5e-4, 2e-3).reshape(n, 4)
    elif fmt == "q6_k":   # d: the last plane, 2 bytes per super-block
        raw[208 * n:] = scales(n, 2e-5, 8e-5)
    elif fmt == "q8_0":   # d: the last plane, 2 bytes per 32 weights
        raw[n_rows * n_cols:] = scales(8 * n, 5e-4, 2e-3)
    else:
        raise KeyError(fmt)
    return raw


def normal_f32(config_id, layer, tensor, shape):
    """fp32 N(0,1)."""
    return _rng(config_id, layer, tensor).standard_normal(shape, dtype=np.float64).astype(np.float32)


def gain_f32(config_id, layer, tensor, n):
    """RMSNorm gain 1 + N(0, 0.1), fp32."""
    z = _rng(config_id, layer, tensor).standard_normal(n, dtype=np.float64)
    return (1.0 + 0.1 * z).astype(np.float32)


def kv_cache_f16(config_id, layer, tensor, n_kv_heads, kv_cap, head_dim, n_past):
    """fp16 [n_kv_heads, kv_cap, head_dim]; rows < n_past ~ N(0,1), the rest zero."""
    out = np.zeros((n_kv_heads, kv_cap, head_dim), dtype=np.float16)
    if n_past > 0:
        z = _rng(config_id, layer, tensor).standard_normal((n_kv_heads, n_past, head_dim), dtype=np.float32)
        out[:, :n_past, :] = z.astype(np.float16)
    return out


def layer_tensors(cfg, layer, kv_cap=None, formats=None):
    """All tensors of one decoder layer of window `cfg` as a dict of numpy arrays.  formats: optional dict
    tensor name -> format for matrices that are not Q4_K (those come as flat uint8, see fmt_tensor)."""
    d = cfg.dims
    cid = cfg.config_id
    cap = kv_cap if kv_cap is not None else cfg.n_past + cfg.T
    if formats:
        t = layer_tensors(cfg, layer, kv_cap)
        shapes = {"wq": (d.qd, d.e), "wk": (d.kvd, d.e), "wv": (d.kvd, d.e), "wo": (d.e, d.qd),
                  "wgate": (d.ffn, d.e), "wup": (d.ffn, d.e), "wdown": (d.e, d.ffn)}
        for name, fmt in formats.items():
            if fmt != "q4_k":
                t[name] = fmt_tensor(cid, layer, name, fmt, *shapes[name])
        return t
    return {
        "wq": q4k_tensor(cid, layer, "wq", d.qd, d.e),
        "wk": q4k_tensor(cid, layer, "wk", d.kvd, d.e),
        "wv": q4k_tensor(cid, layer, "wv", d.kvd, d.e),
        "wo": q4k_tensor(cid, layer, "wo", d.e, d.qd),
        "wgate": q4k_tensor(cid, layer, "wgate", d.ffn, d.e),
        "wup": q4k_tensor(cid, layer, "wup", d.ffn, d.e),
        "wdown": q4k_tensor(cid, layer, "wdown", d.e, d.ffn),
        "g_attn": gain_f32(cid, layer, "g_attn", d.e),
        "g_ffn": gain_f32(cid, layer, "g_ffn", d.e),
        "k_cache": kv_cache_f16(cid, layer, "k_cache", d.n_kv_heads, cap, d.head_dim, cfg.n_past),
        "v_cache": kv_cache_f16(cid, layer, "v_cache", d.n_kv_heads, cap, d.head_dim, cfg.n_past),
    }


def batch_caches(cfg, n_layers, n_past, kv_cap):
    """KV caches of a batch of independent sequences: [layer][sequence] -> (k_cache, v_cache), sequence b
    holding n_past[b] rows ~ N(0,1) (fp16 [n_kv_heads, kv_cap, head_dim], the rest zero)."""
    d = cfg.dims
    return [[(kv_cache_f16(cfg.config_id, l, SEQ_CACHE_ID0 + 2 * b, d.n_kv_heads, kv_cap, d.head_dim, n),
              kv_cache_f16(cfg.config_id, l, SEQ_CACHE_ID0 + 2 * b + 1, d.n_kv_heads, kv_cap, d.head_dim, n))
             for b, n in enumerate(n_past)] for l in range(n_layers)]


def batch_input(cfg, B):
    """x_in fp32 [B, e] ~ N(0,1): one token per sequence."""
    return normal_f32(cfg.config_id, 0, "x_in_batch", (B, cfg.dims.e))


def window_input(cfg):
    """x_in fp32 [T, e] ~ N(0,1)."""
    return normal_f32(cfg.config_id, 0, "x_in", (cfg.T, cfg.dims.e))


def output_layer_tensors(cfg):
    d = cfg.dims
    return {
        "g_final": gain_f32(cfg.config_id, 0, "g_final", d.e),
        "w_lm": q4k_tensor(cfg.config_id, 0, "w_lm", cfg.vocab, d.e),
    }
