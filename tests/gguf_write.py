"""Test-side writer of small GGUF files, written from the container's description alone (the docstring of
paper_2504_08791_amd/gguf.py); independent of the reader.  Tensors are given as ready-made bytes."""
import struct

TYPE_CODES = {"f32": 0, "f16": 1, "q8_0": 8, "q4_k": 12, "q5_k": 13, "q6_k": 14}


def _s(text):
    b = text.encode("utf-8")
    return struct.pack("<Q", len(b)) + b


def _value(v):
    """(type code, bytes) of a metadata value: str, bool, int (u32), float (f32), ("u64", n), ("f64", x), lists of one kind"""
    if isinstance(v, str):
        return 8, _s(v)
    if isinstance(v, bool):
        return 7, struct.pack("<?", v)
    if isinstance(v, int):
        return 4, struct.pack("<I", v)
    if isinstance(v, float):
        return 6, struct.pack("<f", v)
    if isinstance(v, tuple):
        kind, x = v
        code, fmt = {"u64": (10, "<Q"), "f64": (12, "<d"), "i32": (5, "<i")}[kind]
        return code, struct.pack(fmt, x)
    if isinstance(v, list):
        parts = [_value(x) for x in v]
        etype = parts[0][0] if parts else 4
        assert all(p[0] == etype for p in parts)
        return 9, struct.pack("<IQ", etype, len(parts)) + b"".join(p[1] for p in parts)
    raise TypeError(type(v))


def write(path, meta, tensors, alignment=32, version=3):
    """meta: dict key -> value; tensors: list of (name, dims with the contiguous one first, type name or code, bytes)"""
    out = bytearray(b"GGUF")
    out += struct.pack("<IQQ", version, len(tensors), len(meta))
    for k, v in meta.items():
        code, b = _value(v)
        out += _s(k) + struct.pack("<I", code) + b
    offsets, pos = [], 0
    for _, _, _, data in tensors:
        pos = (pos + alignment - 1) // alignment * alignment
        offsets.append(pos)
        pos += len(data)
    for (name, dims, typ, _), off in zip(tensors, offsets):
        out += _s(name) + struct.pack("<I", len(dims)) + b"".join(struct.pack("<Q", d) for d in dims)
        out += struct.pack("<IQ", TYPE_CODES.get(typ, typ), off)
    out += b"\0" * (-len(out) % alignment)
    start = len(out)
    for (_, _, _, data), off in zip(tensors, offsets):
        out += b"\0" * (start + off - len(out))
        out += bytes(data)
    with open(path, "wb") as f:
        f.write(out)
    return start
