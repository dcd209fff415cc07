"""Reading a layer window out of a GGUF model file (host logic; the bit rearrangement runs on the device).

The paper's checkpoints are "Q4K" GGUF files of Llama and Qwen models (arXiv 2504.08791, Sec. 4, experimental setup);
a device of the ring loads only the layers of its window (Sec. 3.1).  This module parses the file's directory
(header, metadata, tensor table), memory-maps the tensor data, copies the tensors of the requested layers to the
GPU as they are and has `prima_repack_gguf` put them into the library's layouts there.

File structure, as read here (little endian; restated from the public description of the container, no file was at
hand, so agreement with real files is untested):
    magic "GGUF" | version u32 (2 or 3) | tensor count u64 | metadata count u64
    metadata entries:  key (string = u64 length + bytes) | value type u32 | value
        value types 0..12: u8, i8, u16, i16, u32, i32, f32, bool, string, array (element type u32, count u64,
        elements), u64, i64, f64
    tensor entries:    name (string) | number of dimensions u32 | dimensions u64 each (the first is the contiguous one:
        columns) | tensor type u32 | offset u64 from the start of the data section
    data section: starts at the next multiple of `general.alignment` (default 32) after the tensor table.
Tensor types used: 0 F32, 1 F16, 8 Q8_0, 12 Q4_K, 13 Q5_K, 14 Q6_K; a tensor of any other type is reported by name
when it is asked for.

Not covered: biases (the Qwen-2.5 files carry `attn_{q,k,v}.bias`; the window forward of this library has none, and
`load_window` refuses such a file unless told to drop them), the embedding lookup, tokenizer data.
"""
import mmap
import struct
from dataclasses import dataclass

import numpy as np

TYPE_NAMES = {0: "f32", 1: "f16", 8: "q8_0", 12: "q4_k", 13: "q5_k", 14: "q6_k"}
_BLOCK = {"f32": (1, 4), "f16": (1, 2), "q8_0": (32, 34), "q4_k": (256, 144), "q5_k": (256, 176), "q6_k": (256, 210)}
_SCALARS = {0: "<B", 1: "<b", 2: "<H", 3: "<h", 4: "<I", 5: "<i", 6: "<f", 7: "<?", 10: "<Q", 11: "<q", 12: "<d"}

# tensors of a decoder layer: name in the file -> field of a window layer
LAYER_MATRICES = {"attn_q": "wq", "attn_k": "wk", "attn_v": "wv", "attn_output": "wo",
                  "ffn_gate": "wgate", "ffn_up": "wup", "ffn_down": "wdown"}
LAYER_GAINS = {"attn_norm": "g_attn", "ffn_norm": "g_ffn"}


class GGUFError(ValueError):
    pass


@dataclass
class TensorInfo:
    name: str
    shape: tuple      # (n_rows, n_cols); a vector is (1, n)
    type_code: int
    offset: int       # from the start of the file
    nbytes: int

    @property
    def fmt(self):
        return TYPE_NAMES.get(self.type_code)


@dataclass
class Dims:
    e: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rope_theta: float
    rms_eps: float
    rope_mode: int


class _Cursor:
    def __init__(self, buf):
        self.buf, self.pos = buf, 0

    def take(self, fmt):
        n = struct.calcsize(fmt)
        if self.pos + n > len(self.buf):
            raise GGUFError("file ends inside its directory")
        v = struct.unpack_from(fmt, self.buf, self.pos)[0]
        self.pos += n
        return v

    def string(self):
        n = self.take("<Q")
        if self.pos + n > len(self.buf):
            raise GGUFError("file ends inside a string")
        s = bytes(self.buf[self.pos:self.pos + n]).decode("utf-8", errors="replace")
        self.pos += n
        return s

    def value(self, vtype):
        if vtype in _SCALARS:
            return self.take(_SCALARS[vtype])
        if vtype == 8:
            return self.string()
        if vtype == 9:
            etype, count = self.take("<I"), self.take("<Q")
            if count <= 64:
                return [self.value(etype) for _ in range(count)]
            # long arrays (tokenizer tables) are stepped over, not kept
            if etype in _SCALARS:
                size = struct.calcsize(_SCALARS[etype]) * count
                if self.pos + size > len(self.buf):
                    raise GGUFError("file ends inside an array")
                self.pos += size
            else:
                for _ in range(count):
                    self.value(etype)
            return ("array", etype, count)
        raise GGUFError(f"unknown metadata value type {vtype}")


class GGUFFile:
    """Directory of a GGUF file and memory-mapped access to its tensors."""

    def __init__(self, path):
        self.path = path
        self._f = open(path, "rb")
        self._map = mmap.mmap(self._f.fileno(), 0, access=mmap.ACCESS_READ)
        c = _Cursor(memoryview(self._map))
        if bytes(c.buf[0:4]) != b"GGUF":
            raise GGUFError("not a GGUF file (magic)")
        c.pos = 4
        self.version = c.take("<I")
        if self.version not in (2, 3):
            raise GGUFError(f"GGUF version {self.version} is not supported")
        n_tensors, n_meta = c.take("<Q"), c.take("<Q")
        self.meta = {}
        for _ in range(n_meta):
            key = c.string()
            self.meta[key] = c.value(c.take("<I"))
        entries = []
        for _ in range(n_tensors):
            name = c.string()
            nd = c.take("<I")
            if not 1 <= nd <= 4:
                raise GGUFError(f"{name}: {nd} dimensions")
            dims = [c.take("<Q") for _ in range(nd)]
            entries.append((name, dims, c.take("<I"), c.take("<Q")))
        align = int(self.meta.get("general.alignment", 32))
        if align <= 0 or align & (align - 1):
            raise GGUFError(f"general.alignment = {align}")
        self.data_start = (c.pos + align - 1) // align * align
        self.tensors = {}
        for name, dims, code, off in entries:
            n_cols = dims[0]
            n_rows = int(np.prod(dims[1:], dtype=np.int64)) if len(dims) > 1 else 1
            fmt = TYPE_NAMES.get(code)
            nbytes = -1
            if fmt is not None:
                per, size = _BLOCK[fmt]
                if n_cols % per:
                    raise GGUFError(f"{name}: {n_cols} columns are no whole number of {fmt} blocks")
                nbytes = n_rows * (n_cols // per) * size
                if self.data_start + off + nbytes > len(self._map):
                    raise GGUFError(f"{name}: data beyond the end of the file")
            self.tensors[name] = TensorInfo(name, (n_rows, n_cols), code, self.data_start + off, nbytes)

    def close(self):
        self._map.close()
        self._f.close()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # ---- metadata ----
    @property
    def arch(self):
        return self.meta.get("general.architecture", "llama")

    def _m(self, key, default=None):
        v = self.meta.get(f"{self.arch}.{key}", default)
        if v is None:
            raise GGUFError(f"metadata key {self.arch}.{key} is missing")
        return v

    @property
    def n_layers(self):
        return int(self._m("block_count"))

    def dims(self, rope_mode=None):
        """Model dimensions from the metadata.  rope_mode: 0 pairs (i, i + D/2), 1 pairs (2i, 2i + 1); by default 1 for
        architecture "llama" (whose files store Q and K rows permuted for adjacent pairs) and 0 otherwise."""
        e, hq = int(self._m("embedding_length")), int(self._m("attention.head_count"))
        hkv = int(self._m("attention.head_count_kv", hq))
        hd = int(self._m("attention.key_length", e // hq))
        if rope_mode is None:
            rope_mode = 1 if self.arch == "llama" else 0
        return Dims(e, hq, hkv, hd, int(self._m("feed_forward_length")), float(self._m("rope.freq_base", 10000.0)),
                    float(self._m("attention.layer_norm_rms_epsilon", 1e-5)), rope_mode)

    # ---- tensors ----
    def info(self, name):
        if name not in self.tensors:
            raise GGUFError(f"no tensor {name} in {self.path}")
        t = self.tensors[name]
        if t.fmt is None:
            raise GGUFError(f"{name}: tensor type {t.type_code} is not supported")
        return t

    def raw(self, name):
        """the tensor's bytes as they lie in the file (a read-only numpy view of the mapping)"""
        t = self.info(name)
        return np.frombuffer(self._map, dtype=np.uint8, count=t.nbytes, offset=t.offset)

    def load_matrix(self, name, device):
        """(format name, flat uint8 CUDA tensor in this library's layout, (rows, cols)) of a weight matrix"""
        import torch
        from . import repack_gguf
        t = self.info(name)
        rows, cols = t.shape
        if cols % 256:
            raise GGUFError(f"{name}: {cols} columns are no multiple of 256")
        staged = torch.from_numpy(self.raw(name).copy()).to(device)
        return t.fmt, repack_gguf(t.fmt, staged, rows, cols), (rows, cols)

    def load_vector(self, name, device):
        """float32 CUDA vector (norm gains; stored as F32 or F16)"""
        import torch
        t = self.info(name)
        raw = self.raw(name)
        if t.fmt == "f32":
            v = raw.view(np.float32).copy()
        elif t.fmt == "f16":
            v = raw.view(np.float16).astype(np.float32)
        else:
            raise GGUFError(f"{name}: a vector in {t.fmt}")
        return torch.from_numpy(v.reshape(-1)).to(device)

    def load_window(self, first_layer, n_layers, device, kv_cap, rope_mode=None, drop_biases=False):
        """Layers first_layer .. first_layer + n_layers - 1 on the device.

        Returns (dims, layers, formats): layers and formats as `Window(dims, layers, kv_cap, formats=formats)` takes
        them (fp16 caches of kv_cap rows allocated here, zero-filled)."""
        import torch
        d = self.dims(rope_mode)
        if first_layer < 0 or n_layers < 1 or first_layer + n_layers > self.n_layers:
            raise GGUFError(f"layers {first_layer}..{first_layer + n_layers - 1} of {self.n_layers}")
        expect = {"wq": (d.n_q_heads * d.head_dim, d.e), "wk": (d.n_kv_heads * d.head_dim, d.e), "wv": (d.n_kv_heads * d.head_dim, d.e),
                  "wo": (d.e, d.n_q_heads * d.head_dim), "wgate": (d.ffn, d.e), "wup": (d.ffn, d.e), "wdown": (d.e, d.ffn)}
        layers, formats = [], []
        for l in range(first_layer, first_layer + n_layers):
            biases = [n for n in self.tensors if n.startswith(f"blk.{l}.") and n.endswith(".bias")]
            if biases and not drop_biases:
                raise GGUFError(f"layer {l} has biases ({', '.join(sorted(biases))}); the window forward has none")
            t, f = {}, {}
            for file_name, field in LAYER_MATRICES.items():
                fmt, w, shape = self.load_matrix(f"blk.{l}.{file_name}.weight", device)
                if shape != expect[field]:
                    raise GGUFError(f"blk.{l}.{file_name}.weight is {shape[0]} x {shape[1]}, the metadata says {expect[field]}")
                t[field] = w
                if fmt != "q4_k":
                    f[field] = fmt
            for file_name, field in LAYER_GAINS.items():
                g = self.load_vector(f"blk.{l}.{file_name}.weight", device)
                if g.numel() != d.e:
                    raise GGUFError(f"blk.{l}.{file_name}.weight has {g.numel()} values, not {d.e}")
                t[field] = g
            t["k_cache"] = torch.zeros((d.n_kv_heads, kv_cap, d.head_dim), dtype=torch.float16, device=device)
            t["v_cache"] = torch.zeros((d.n_kv_heads, kv_cap, d.head_dim), dtype=torch.float16, device=device)
            layers.append(t)
            formats.append(f)
        return d, layers, (formats if any(formats) else None)

    def load_output_layer(self, device):
        """(g_final float32 [e], format name, w_lm flat uint8, vocab): the final RMSNorm's gains and the output matrix
        (`output.weight`; files that tie it to the embedding carry `token_embd.weight` only)."""
        g = self.load_vector("output_norm.weight", device)
        name = "output.weight" if "output.weight" in self.tensors else "token_embd.weight"
        fmt, w, (vocab, _) = self.load_matrix(name, device)
        return g, fmt, w, vocab
