"""numpy front-end of the CPU oracle (oracle/prima_oracle.c).

TEST INFRASTRUCTURE ONLY: used by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module
and this module never imports the product package.

Every function takes and returns numpy arrays; hidden states are float64.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "prima_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force=False):
    """Compile the C oracle with gcc (fp contraction off, OpenMP over rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Dims(C.Structure):
    _fields_ = [("e", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn", C.c_int32),
                ("rope_theta", C.c_double), ("rms_eps", C.c_double), ("rope_mode", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_half_to_double.restype = C.c_double
        _lib.orc_half_to_double.argtypes = [C.c_uint16]
        _lib.orc_float_to_half.restype = C.c_uint16
        _lib.orc_float_to_half.argtypes = [C.c_float]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _dims(d):
    # rms_eps is the fp32 value the kernels receive, promoted
    return _Dims(d.e, d.n_q_heads, d.n_kv_heads, d.head_dim, d.ffn,
                 float(np.float32(d.rope_theta)), float(np.float32(d.rms_eps)), d.rope_mode)


def _w(W):
    W = np.ascontiguousarray(W, dtype=np.uint8)
    assert W.ndim == 3 and W.shape[2] == 144, W.shape
    return W, W.shape[0], W.shape[1] * 256


def num_threads():
    return lib().orc_num_threads()


def set_num_threads(n):
    lib().orc_set_num_threads(int(n))


def dequant(W):
    """float32 [rows, cols] dequantised weights of a Q4_K tensor uint8 [rows, cols/256, 144]."""
    W, r, c = _w(W)
    out = np.empty((r, c), dtype=np.float32)
    rc = lib().orc_q4k_dequant(_p(W), C.c_int64(r), C.c_int64(c), _p(out))
    assert rc == 0
    return out


def gemv(W, x):
    """y[t, r] = sum_c W[r, c] x[t, c]; x float64 [T, cols] -> float64 [T, rows]."""
    W, r, c = _w(W)
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    T = x.shape[0]
    assert x.shape[1] == c
    y = np.empty((T, r), dtype=np.float64)
    rc = lib().orc_q4k_gemv(_p(W), C.c_int64(r), C.c_int64(c), _p(x), C.c_int64(c), C.c_int32(T),
                            _p(y), C.c_int64(r))
    assert rc == 0
    return y


FORMATS = {"q4_k": 0, "q5_k": 1, "q6_k": 2, "q8_0": 3, "f16": 4, "f32": 5}


def fmt_tensor_bytes(fmt, n_rows, n_cols):
    lib().orc_fmt_tensor_bytes.restype = C.c_int64
    return int(lib().orc_fmt_tensor_bytes(C.c_int32(FORMATS[fmt]), C.c_int64(n_rows), C.c_int64(n_cols)))


def _wf(fmt, W, n_rows, n_cols):
    W = np.ascontiguousarray(W, dtype=np.uint8).reshape(-1)
    assert W.size == fmt_tensor_bytes(fmt, n_rows, n_cols), (fmt, W.size, n_rows, n_cols)
    return W


def fmt_dequant(fmt, W, n_rows, n_cols):
    """float32 [n_rows, n_cols]: the weights of a tensor (flat uint8) in one of FORMATS."""
    W = _wf(fmt, W, n_rows, n_cols)
    out = np.empty((n_rows, n_cols), dtype=np.float32)
    rc = lib().orc_fmt_dequant(C.c_int32(FORMATS[fmt]), _p(W), C.c_int64(n_rows), C.c_int64(n_cols), _p(out))
    assert rc == 0
    return out


def fmt_gemv(fmt, W, n_rows, n_cols, x):
    """y float64 [T, n_rows] = x [T, n_cols] times the transposed weights (fp64 accumulation)."""
    W = _wf(fmt, W, n_rows, n_cols)
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    T = x.shape[0]
    assert x.shape[1] == n_cols
    y = np.empty((T, n_rows), dtype=np.float64)
    rc = lib().orc_fmt_gemv(C.c_int32(FORMATS[fmt]), _p(W), C.c_int64(n_rows), C.c_int64(n_cols), _p(x), C.c_int64(n_cols),
                            C.c_int32(T), _p(y), C.c_int64(n_rows))
    assert rc == 0
    return y


def lm_head_fmt(dims, fmt, g_final, w_lm, vocab, x):
    """logits float64 [T, vocab]: final RMSNorm, then the output matrix in one of FORMATS."""
    W = _wf(fmt, w_lm, vocab, dims.e)
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    T = x.shape[0]
    g = np.ascontiguousarray(g_final, dtype=np.float32)
    out = np.empty((T, vocab), dtype=np.float64)
    dd = _dims(dims)
    rc = lib().orc_lm_head_fmt(C.byref(dd), C.c_int32(FORMATS[fmt]), _p(g), _p(W), C.c_int64(vocab), _p(x), C.c_int32(T), _p(out))
    assert rc == 0
    return out


def rmsnorm(x, g, eps):
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float32)
    out = np.empty_like(x)
    for j in range(x.shape[0]):
        lib().orc_rmsnorm(_p(x[j]), _p(g), C.c_int32(x.shape[1]), C.c_double(float(np.float32(eps))), _p(out[j]))
    return out


def rope(v, n_heads, head_dim, pos, theta, mode=0):
    """v float64 [n_heads * head_dim] of one token at position pos; returns the rotated copy."""
    out = np.array(v, dtype=np.float64, copy=True).reshape(-1)
    assert out.size == n_heads * head_dim
    lib().orc_rope(_p(out), C.c_int32(n_heads), C.c_int32(head_dim), C.c_int32(pos),
                   C.c_double(float(np.float32(theta))), C.c_int32(mode))
    return out


def swiglu(g, u):
    g = np.ascontiguousarray(g, dtype=np.float64)
    u = np.ascontiguousarray(u, dtype=np.float64)
    out = np.empty_like(g)
    lib().orc_swiglu(_p(g), _p(u), C.c_int64(g.size), _p(out))
    return out


def softmax(logits):
    logits = np.ascontiguousarray(logits, dtype=np.float64)
    w = np.empty_like(logits)
    lib().orc_softmax(_p(logits), C.c_int32(logits.size), _p(w))
    return w


def attn_decode(dims, q, K, V, n_past, T, return_gap=False):
    """q float64 [T, Hq, D]; K, V float16 [Hkv, cap, D] with rows < n_past + T valid."""
    q = np.ascontiguousarray(q, dtype=np.float64).reshape(T, dims.n_q_heads, dims.head_dim)
    K = np.ascontiguousarray(K, dtype=np.float16)
    V = np.ascontiguousarray(V, dtype=np.float16)
    cap = K.shape[1]
    o = np.empty_like(q)
    gap = C.c_double(0.0)
    dd = _dims(dims)
    rc = lib().orc_attn_decode(C.byref(dd), _p(q), _p(K), _p(V), C.c_int32(cap), C.c_int32(n_past),
                               C.c_int32(T), _p(o), C.byref(gap))
    assert rc == 0
    return (o, gap.value) if return_gap else o


def kv_append(dims, k, v, K, V, n_past, T):
    """Writes fp16(fp32(k)), fp16(fp32(v)) [T, Hkv*D] into K, V rows n_past..n_past+T-1 in place."""
    k = np.ascontiguousarray(k, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64)
    assert K.flags.c_contiguous and V.flags.c_contiguous and K.dtype == np.float16
    dd = _dims(dims)
    lib().orc_kv_append(C.byref(dd), _p(k), _p(v), _p(K), _p(V), C.c_int32(K.shape[1]),
                        C.c_int32(n_past), C.c_int32(T))


WEIGHTS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def layer(dims, t, x, n_past, taps=False, formats=None):
    """Advance one decoder layer by T = x.shape[0] tokens.

    t: dict of the layer's tensors (wq..wdown uint8 [r, nb, 144]; g_attn, g_ffn float32;
    k_cache, v_cache float16 [Hkv, cap, D], updated in place).  x float64 [T, e].
    formats: optional dict tensor name -> one of FORMATS for tensors kept in another format (flat uint8).
    Returns y float64 [T, e] (and a dict of taps when asked).
    """
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    T, e = x.shape
    assert e == dims.e
    K, V = t["k_cache"], t["v_cache"]
    assert K.flags.c_contiguous and V.flags.c_contiguous and K.dtype == np.float16 and V.dtype == np.float16
    ws = [np.ascontiguousarray(t[k], dtype=np.uint8) for k in WEIGHTS]
    fm = (C.c_int32 * 7)(*[FORMATS[(formats or {}).get(k, "q4_k")] for k in WEIGHTS])
    shapes = {"wq": (dims.qd, e), "wk": (dims.kvd, e), "wv": (dims.kvd, e), "wo": (e, dims.qd),
              "wgate": (dims.ffn, e), "wup": (dims.ffn, e), "wdown": (e, dims.ffn)}
    for k, w in zip(WEIGHTS, ws):
        assert w.size == fmt_tensor_bytes((formats or {}).get(k, "q4_k"), *shapes[k]), k
    ga = np.ascontiguousarray(t["g_attn"], dtype=np.float32)
    gf = np.ascontiguousarray(t["g_ffn"], dtype=np.float32)
    y = np.empty_like(x)
    tp = {}
    if taps:
        tp = {"q": np.empty((T, dims.qd)), "o": np.empty((T, dims.qd)), "h": np.empty((T, e)),
              "a": np.empty((T, dims.ffn))}
    gap = C.c_double(0.0)
    dd = _dims(dims)
    rc = lib().orc_layer_fmt(C.byref(dd), fm, *[_p(w) for w in ws], _p(ga), _p(gf), _p(K), _p(V),
                         C.c_int32(K.shape[1]), C.c_int32(n_past), C.c_int32(T), _p(x), _p(y),
                         _p(tp.get("q")), _p(tp.get("o")), _p(tp.get("h")), _p(tp.get("a")), C.byref(gap))
    assert rc == 0
    if taps:
        tp["min_gap"] = gap.value
        return y, tp
    return y


def window(dims, layers, x, n_past, formats=None):
    """Compose consecutive layers (list of tensor dicts); formats: optional list of per-layer dicts as for layer()."""
    h = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    for i, t in enumerate(layers):
        h = layer(dims, t, h, n_past, formats=formats[i] if formats else None)
    return h


def window_batch(dims, layers, caches, x, n_past, formats=None):
    """One token for each of B independent sequences (continuous batching, App. A.12): row b of x is advanced
    through the layers against sequence b's own caches, caches[l][b] = (k_cache, v_cache) with n_past[b] rows
    (updated in place), exactly as a one-token call for that sequence alone.  The layers' own caches are not used.
    formats: optional list of per-layer dicts as for layer()."""
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    y = np.empty_like(x)
    for b in range(x.shape[0]):
        h = x[b:b + 1]
        for l, t in enumerate(layers):
            tb = dict(t)
            tb["k_cache"], tb["v_cache"] = caches[l][b]
            h = layer(dims, tb, h, int(n_past[b]), formats=formats[l] if formats else None)
        y[b] = h[0]
    return y


def lm_head(dims, g_final, w_lm, x):
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    W, vocab, c = _w(w_lm)
    g = np.ascontiguousarray(g_final, dtype=np.float32)
    out = np.empty((x.shape[0], vocab), dtype=np.float64)
    dd = _dims(dims)
    rc = lib().orc_lm_head(C.byref(dd), _p(g), _p(W), C.c_int64(vocab), _p(x), C.c_int32(x.shape[0]), _p(out))
    assert rc == 0
    return out


def half_to_double(bits):
    return lib().orc_half_to_double(int(bits))


def float_to_half(f):
    return lib().orc_float_to_half(float(np.float32(f)))
