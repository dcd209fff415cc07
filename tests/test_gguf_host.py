"""Host logic of the GGUF reader (paper_2504_08791_amd/gguf.py): directory, metadata, tensor bytes, refusals.
Files are written by tests/gguf_write.py, a writer of its own made from the same description; no GPU, no kernels."""
import os
import struct
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(__file__))
import gguf_write
from paper_2504_08791_amd import gguf

META = {"general.architecture": "llama", "llama.block_count": 2, "llama.embedding_length": 512,
        "llama.attention.head_count": 4, "llama.attention.head_count_kv": 2, "llama.feed_forward_length": 768,
        "llama.rope.freq_base": 10000.0, "llama.attention.layer_norm_rms_epsilon": 1e-5}


def _bytes(n, seed):
    return np.random.default_rng(seed).integers(0, 256, n, dtype=np.uint8).tobytes()


def test_directory_and_bytes(tmp_path):
    a, b, c = _bytes(2 * 144 * 3, 1), _bytes(512 * 4, 2), _bytes(210 * 2, 3)
    meta = dict(META)
    meta["tokenizer.ggml.tokens"] = ["tok%d" % i for i in range(100)]      # long array of strings: stepped over
    meta["tokenizer.ggml.scores"] = [float(i) for i in range(100)]         # long array of numbers: stepped over
    meta["some.list"] = [1, 2, 3]
    meta["some.u64"] = ("u64", 1 << 40)
    meta["some.flag"] = True
    p = str(tmp_path / "m.gguf")
    gguf_write.write(p, meta, [("blk.0.attn_q.weight", [512, 3], "q4_k", a), ("blk.0.attn_norm.weight", [512], "f32", b),
                               ("odd.weight", [256, 2], "q6_k", c)])
    with gguf.GGUFFile(p) as f:
        assert f.version == 3 and f.arch == "llama" and f.n_layers == 2
        assert f.meta["some.list"] == [1, 2, 3] and f.meta["some.u64"] == 1 << 40 and f.meta["some.flag"] is True
        assert f.meta["tokenizer.ggml.tokens"] == ("array", 8, 100)
        assert f.tensors["blk.0.attn_q.weight"].shape == (3, 512) and f.tensors["blk.0.attn_q.weight"].fmt == "q4_k"
        assert f.tensors["blk.0.attn_norm.weight"].shape == (1, 512)
        assert f.raw("blk.0.attn_q.weight").tobytes() == a
        assert f.raw("blk.0.attn_norm.weight").tobytes() == b
        assert f.raw("odd.weight").tobytes() == c
        assert f.data_start % 32 == 0 and f.tensors["odd.weight"].offset % 32 == 0
        d = f.dims()
        assert (d.e, d.n_q_heads, d.n_kv_heads, d.head_dim, d.ffn, d.rope_mode) == (512, 4, 2, 128, 768, 1)
        assert d.rope_theta == 10000.0 and abs(d.rms_eps - 1e-5) < 1e-12
        assert f.dims(rope_mode=0).rope_mode == 0
        with pytest.raises(gguf.GGUFError):
            f.info("missing.weight")


def test_alignment_key_and_other_architecture(tmp_path):
    meta = {"general.architecture": "qwen2", "general.alignment": 64, "qwen2.block_count": 1, "qwen2.embedding_length": 256,
            "qwen2.attention.head_count": 2, "qwen2.feed_forward_length": 512, "qwen2.rope.freq_base": 1e6,
            "qwen2.attention.layer_norm_rms_epsilon": 1e-6}
    a = _bytes(34 * 8, 5)
    p = str(tmp_path / "q.gguf")
    gguf_write.write(p, meta, [("x.weight", [256, 1], "q8_0", a)], alignment=64)
    with gguf.GGUFFile(p) as f:
        assert f.data_start % 64 == 0 and f.raw("x.weight").tobytes() == a
        d = f.dims()
        assert d.n_kv_heads == 2 and d.rope_mode == 0 and d.rope_theta == 1e6


def test_refusals(tmp_path):
    p = str(tmp_path / "bad.gguf")
    open(p, "wb").write(b"GGML" + b"\0" * 64)
    with pytest.raises(gguf.GGUFError, match="magic"):
        gguf.GGUFFile(p)
    gguf_write.write(p, META, [], version=1)
    with pytest.raises(gguf.GGUFError, match="version"):
        gguf.GGUFFile(p)
    # a tensor whose data would lie beyond the end of the file
    gguf_write.write(p, META, [("w", [256, 4], "q4_k", _bytes(144 * 4, 1))])
    raw = open(p, "rb").read()
    open(p, "wb").write(raw[:-100])
    with pytest.raises(gguf.GGUFError, match="beyond"):
        gguf.GGUFFile(p)
    # the directory itself cut short
    open(p, "wb").write(raw[:40])
    with pytest.raises(gguf.GGUFError):
        gguf.GGUFFile(p)
    # columns that are no whole number of blocks
    gguf_write.write(p, META, [("w", [100, 4], "q4_k", _bytes(144 * 4, 1))])
    with pytest.raises(gguf.GGUFError, match="blocks"):
        gguf.GGUFFile(p)
    # a tensor type the library has no layout for is only refused when asked for
    gguf_write.write(p, META, [("w", [256, 1], 10, _bytes(84, 1)), ("v", [256], "f32", _bytes(1024, 2))])
    with gguf.GGUFFile(p) as f:
        assert f.raw("v").nbytes == 1024
        with pytest.raises(gguf.GGUFError, match="not supported"):
            f.raw("w")


def test_abi_exports_repack():
    from paper_2504_08791_amd import _ffi
    L = _ffi.lib()
    assert L.prima_gguf_tensor_bytes(_ffi.FORMATS["q4_k"], 3, 512) == 3 * 2 * 144
    assert L.prima_gguf_tensor_bytes(_ffi.FORMATS["q6_k"], 3, 512) == 3 * 2 * 210
    assert L.prima_gguf_tensor_bytes(_ffi.FORMATS["q8_0"], 1, 256) == 272
    assert L.prima_gguf_tensor_bytes(_ffi.FORMATS["q5_k"], 1, 100) == 0
    for fmt in _ffi.FORMATS.values():     # same sizes as the library's own layouts
        assert L.prima_gguf_tensor_bytes(fmt, 5, 768) == L.prima_fmt_tensor_bytes(fmt, 5, 768)
    # argument checks happen before any launch: no GPU needed
    assert L.prima_repack_gguf(99, None, 1, 256, None, None) == 2
    assert L.prima_repack_gguf(0, None, 1, 100, None, None) == 2
    assert L.prima_repack_gguf(0, None, 1, 256, None, None) == 1
    assert L.prima_repack_gguf(0, None, 0, 256, None, None) == 0
