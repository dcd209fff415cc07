"""Oracle-side reading of quantised tensors in the byte order of the public GGUF model files.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain numpy, one weight rule per format, no blocking.

The paper runs "Q4K" checkpoints of Llama and Qwen models distributed as GGUF files (Sec. 4, experimental
setup; the format list of App. A.3's profiler paragraph).  It prints none of the block layouts.  What is
written here restates the published block formats from their public description; nothing in this
container holds a real file or the specification, so this module is PARITY UNPINNED against real
checkpoints: its pins (tests/test_oracle_interchange.py) fix the arithmetic and the internal consistency
of the description (hand-built blocks with values known by mental arithmetic, every weight position
distinguishable, exact rationals), not the agreement with an outside file.

Block formats, as read here (t = index of a weight inside its block, bytes little endian):

  q4_k  144 bytes per 256 weights:  d (binary16) | dmin (binary16) | scales[12] | qs[128]
        six-bit sub-scales sc_j and sub-mins m_j, j = 0..7, from scales[]:
            j < 4:  sc_j = scales[j] & 63,                                  m_j = scales[j+4] & 63
            j >= 4: sc_j = (scales[j+4] & 15) | ((scales[j-4] >> 6) << 4),  m_j = (scales[j+4] >> 4) | ((scales[j] >> 6) << 4)
        quants: with c = t // 64 and l = t % 32,  q_t = qs[32c + l] & 15 when t % 64 < 32, else qs[32c + l] >> 4
        w_t = d * sc_s * q_t - dmin * m_s,  s = t // 32
  q5_k  176 bytes:  d | dmin | scales[12] (as q4_k) | qh[32] | qs[128]
        low four bits as q4_k's q_t; bit 4 of q_t = bit (2c + (t % 64 >= 32)) of qh[l];  same value rule, q_t in 0..31
  q6_k  210 bytes:  ql[128] | qh[64] | scales[16] (signed bytes) | d (binary16)
        with h = t // 128, k = (t % 128) // 32, l = t % 32:
            low four bits = ql[64h + 32(k & 1) + l] & 15 when k < 2, else ql[64h + 32(k & 1) + l] >> 4
            bits 4..5     = (qh[32h + l] >> 2k) & 3
        w_t = d * scales[t // 16] * (q_t - 32)
  q8_0  34 bytes per 32 weights:  d (binary16) | qs[32] (signed bytes);   w_t = d * qs[t]
  f16, f32: row-major numbers.

Rounding: as for the library's own layouts, every product is formed in fp32 in the order
fl(fl(fl(d * sc) * q) - fl(dmin * m)); each product is exact (11 + 6 + 5 significant bits at most).
"""
import numpy as np

BLOCK_BYTES = {"q4_k": (256, 144), "q5_k": (256, 176), "q6_k": (256, 210), "q8_0": (32, 34), "f16": (1, 2), "f32": (1, 4)}


def tensor_bytes(fmt, n_rows, n_cols):
    per, size = BLOCK_BYTES[fmt]
    assert n_cols % per == 0
    return n_rows * (n_cols // per) * size


def _half(b):
    """[..., 2] uint8 -> float32 value of the binary16 number"""
    return np.ascontiguousarray(b).view(np.float16).astype(np.float32)[..., 0]


def _scales_mins(sc12):
    """[n, 12] uint8 -> sc [n, 8], m [n, 8] (0..63)"""
    s = sc12.astype(np.int32)
    sc = np.empty(s.shape[:-1] + (8,), dtype=np.int32)
    m = np.empty_like(sc)
    for j in range(8):
        if j < 4:
            sc[..., j] = s[..., j] & 63
            m[..., j] = s[..., j + 4] & 63
        else:
            sc[..., j] = (s[..., j + 4] & 15) | ((s[..., j - 4] >> 6) << 4)
            m[..., j] = (s[..., j + 4] >> 4) | ((s[..., j] >> 6) << 4)
    return sc, m


def _low4_k(qs):
    """[n, 128] uint8 -> [n, 256] low four bits in weight order (q4_k / q5_k)"""
    q = np.empty(qs.shape[:-1] + (256,), dtype=np.int32)
    for t in range(256):
        c, l = t // 64, t % 32
        byte = qs[..., 32 * c + l].astype(np.int32)
        q[..., t] = (byte & 15) if t % 64 < 32 else (byte >> 4)
    return q


def dequant(fmt, raw, n_rows, n_cols):
    """float32 [n_rows, n_cols]: the weights of a tensor whose bytes `raw` (flat uint8) are in GGUF block order,
    rows one after the other, blocks of a row one after the other."""
    raw = np.ascontiguousarray(raw, dtype=np.uint8).reshape(-1)
    assert raw.size == tensor_bytes(fmt, n_rows, n_cols), (fmt, raw.size, n_rows, n_cols)
    if fmt == "f32":
        return raw.view(np.float32).reshape(n_rows, n_cols).copy()
    if fmt == "f16":
        return raw.view(np.float16).astype(np.float32).reshape(n_rows, n_cols)
    per, size = BLOCK_BYTES[fmt]
    blk = raw.reshape(-1, size)
    f32 = np.float32
    if fmt == "q8_0":
        d = _half(blk[:, 0:2])
        q = blk[:, 2:34].view(np.int8).astype(f32)
        w = d[:, None] * q
    elif fmt in ("q4_k", "q5_k"):
        d, dmin = _half(blk[:, 0:2]), _half(blk[:, 2:4])
        sc, m = _scales_mins(blk[:, 4:16])
        if fmt == "q4_k":
            q = _low4_k(blk[:, 16:144])
        else:
            qh, q = blk[:, 16:48].astype(np.int32), _low4_k(blk[:, 48:176])
            for t in range(256):
                c, l = t // 64, t % 32
                q[:, t] |= ((qh[:, l] >> (2 * c + (1 if t % 64 >= 32 else 0))) & 1) << 4
        s_of_t = np.arange(256) // 32
        p1 = (d[:, None] * sc.astype(f32)).astype(f32)          # fl(d * sc_s)            [n, 8]
        p3 = (dmin[:, None] * m.astype(f32)).astype(f32)        # fl(dmin * m_s)
        p2 = (p1[:, s_of_t] * q.astype(f32)).astype(f32)        # fl(fl(d sc_s) q_t)      [n, 256]
        w = (p2 - p3[:, s_of_t]).astype(f32)
    elif fmt == "q6_k":
        ql, qh = blk[:, 0:128].astype(np.int32), blk[:, 128:192].astype(np.int32)
        sc = blk[:, 192:208].view(np.int8).astype(f32)
        d = _half(blk[:, 208:210])
        q = np.empty((blk.shape[0], 256), dtype=np.int32)
        for t in range(256):
            h, k, l = t // 128, (t % 128) // 32, t % 32
            byte = ql[:, 64 * h + 32 * (k & 1) + l]
            lo = (byte & 15) if k < 2 else (byte >> 4)
            q[:, t] = lo | (((qh[:, 32 * h + l] >> (2 * k)) & 3) << 4)
        p1 = (d[:, None] * sc).astype(f32)                      # fl(d * sc_s), s = t // 16   [n, 16]
        w = (p1[:, np.arange(256) // 16] * (q - 32).astype(f32)).astype(f32)
    else:
        raise ValueError(fmt)
    return w.reshape(n_rows, n_cols)
