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


# ---------- conditioning of a case: how far the oracle's own output moves under perturbations of the size of one
# fp32 rounding.  Any implementation that carries fp32 intermediates (the benchmark's boundary dtype, Sec. 3.1 /
# App. A.3: FP32 hidden states) differs from this fp64 evaluation by at least such perturbations, so where they
# move the fp64 result itself by more than the tolerance, the tolerance cannot be asked of that case.  Everything
# here is computed from the oracle alone. ----------

ONE_ULP = 2.0 ** -23  # relative spacing of fp32 numbers


def rel_err(y, r):
    """The parity metric: max_i |y_i - r_i| / max(|r_i|, rms(r), 1e-30) per token vector (row), worst row."""
    y = np.atleast_2d(np.asarray(y, dtype=np.float64))
    r = np.atleast_2d(np.asarray(r, dtype=np.float64))
    y, r = y.reshape(y.shape[0], -1), r.reshape(r.shape[0], -1)
    rms = np.sqrt((r ** 2).mean(axis=1, keepdims=True))
    return float((np.abs(y - r) / np.maximum(np.abs(r), np.maximum(rms, 1e-30))).max())


def conditioning(fn, x, signs, eps=ONE_ULP):
    """max over the sign patterns s in `signs` (arrays of +-1 shaped like x) of rel_err(fn(x * (1 + eps * s)), fn(x)).
    fn: float64 array -> float64 array; it must not keep state between calls."""
    x = np.asarray(x, dtype=np.float64)
    base = fn(x)
    worst = 0.0
    for s in signs:
        s = np.asarray(s, dtype=np.float64)
        assert s.shape == x.shape and np.all(np.abs(s) == 1.0)
        worst = max(worst, rel_err(fn(x * (1.0 + eps * s)), base))
    return worst


def _fresh(layers):
    """the layers with private copies of their caches (a window call appends to them)"""
    out = []
    for t in layers:
        c = dict(t)
        c["k_cache"], c["v_cache"] = t["k_cache"].copy(), t["v_cache"].copy()
        out.append(c)
    return out


def window_long(dims, layers, x, n_past, formats=None, chunk=64):
    """window() for any number of consecutive tokens: pieces of `chunk` tokens one after the other, each seeing
    the rows the earlier ones appended (joint and sequential evaluation are the same function)."""
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    return np.concatenate([window(dims, layers, x[t0:t0 + chunk], n_past + t0, formats=formats)
                           for t0 in range(0, x.shape[0], chunk)], axis=0)


def layer_stepwise(dims, t, x, n_past, formats=None, perturb=None):
    """layer() evaluated step by step through the oracle's own operators (with perturb=None it returns exactly what
    layer() returns: a CPU test holds the two together).  perturb(name, array): called on every intermediate that an
    implementation with FP32 activations between its operators has to store (the projections' outputs q, k, v, the
    rotated q and k, the attention output o, the hidden state h after the first residual, the SwiGLU output a, the
    layer's output y); it returns the array to go on with."""
    pt = perturb if perturb is not None else (lambda name, arr: arr)
    fm = formats or {}
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    T, e = x.shape
    shapes = {"wq": (dims.qd, e), "wk": (dims.kvd, e), "wv": (dims.kvd, e), "wo": (e, dims.qd),
              "wgate": (dims.ffn, e), "wup": (dims.ffn, e), "wdown": (e, dims.ffn)}

    def product(name, act):
        return fmt_gemv(fm.get(name, "q4_k"), t[name], shapes[name][0], shapes[name][1], act)

    n1 = rmsnorm(x, t["g_attn"], dims.rms_eps)
    q, k, v = pt("q", product("wq", n1)), pt("k", product("wk", n1)), pt("v", product("wv", n1))
    for j in range(T):
        q[j] = rope(q[j], dims.n_q_heads, dims.head_dim, n_past + j, dims.rope_theta, dims.rope_mode)
        k[j] = rope(k[j], dims.n_kv_heads, dims.head_dim, n_past + j, dims.rope_theta, dims.rope_mode)
    q, k = pt("q_rot", q), pt("k_rot", k)
    kv_append(dims, k, v, t["k_cache"], t["v_cache"], n_past, T)
    o = pt("o", attn_decode(dims, q, t["k_cache"], t["v_cache"], n_past, T).reshape(T, dims.qd))
    h = pt("h", x + product("wo", o))
    n2 = rmsnorm(h, t["g_ffn"], dims.rms_eps)
    a = pt("a", swiglu(product("wgate", n2), product("wup", n2)))
    return pt("y", h + product("wdown", a))


def window_stepwise(dims, layers, x, n_past, formats=None, perturb=None, chunk=64):
    """Consecutive layers (their caches are updated in place) for any number of consecutive tokens, `chunk` tokens
    at a time, every layer through layer_stepwise()."""
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)
    out = []
    for t0 in range(0, x.shape[0], chunk):
        hcur = x[t0:t0 + chunk]
        for i, t in enumerate(layers):
            hcur = layer_stepwise(dims, t, hcur, n_past + t0, formats=formats[i] if formats else None, perturb=perturb)
        out.append(hcur)
    return np.concatenate(out, axis=0)


_APPENDED = ("k_rot", "v")  # the intermediates whose values are rounded to binary16 into the caches


def _append_ties(arr, eps):
    """Elements of `arr` (values about to be appended to an fp16 cache) that lie within eps |v| of the midpoint
    between two neighbouring binary16 numbers, i.e. whose stored value a relative perturbation of eps can change.
    Returns (mask, moved, closeness): moved = the array with those elements placed just beyond their midpoint (still
    a perturbation of at most about eps), closeness = |v - midpoint| / |v| (inf where there is no such tie)."""
    v = np.asarray(arr, dtype=np.float64)
    h = v.astype(np.float32).astype(np.float16)  # where the append rounds it to (fp64 -> fp32 -> binary16)
    hv = h.astype(np.float64)
    toward = np.where(v >= hv, np.float16(np.inf), np.float16(-np.inf)).astype(np.float16)
    other = np.nextafter(h, toward).astype(np.float64)  # the neighbour on v's side of hv
    mid = 0.5 * (hv + other)
    mag = np.maximum(np.abs(v), 1e-300)
    close = np.abs(v - mid) / mag
    mask = np.isfinite(other) & (close <= eps)
    moved = np.where(mask, mid + np.sign(mid - hv) * eps * mag * 1.000001, v)
    return mask, moved, np.where(mask, close, np.inf)


def window_conditioning(dims, layers, x, n_past, formats=None, probes=4, singles=12, seed=0, eps=ONE_ULP):
    """How far the oracle's own result for this window step moves when every FP32-stored intermediate (see
    layer_stepwise) is perturbed by a relative eps: the largest rel_err against the unperturbed result over
      - `probes` evaluations with v_i -> v_i (1 + eps s_i), random signs s_i (numpy's default generator seeded with
        (seed, probe)): the smooth sensitivity;
      - the evaluations in which appended K / V values within eps (and within eps / 2) of a binary16 rounding
        boundary are all rounded the other way, and those in which one of the `singles` closest ones alone is:
        the discontinuities that perturbations of that size reach (see _append_ties).
    The layers' caches are not modified."""
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=np.float64)

    def run(hook):
        return window_stepwise(dims, _fresh(layers), x, n_past, formats=formats, perturb=hook)

    found = []  # (closeness, site, flat index) of the ties of the unperturbed evaluation

    def record(name, arr):
        if name in _APPENDED:
            record.site += 1
            mask, _, close = _append_ties(arr, eps)
            found.extend((float(close.flat[i]), record.site, int(i)) for i in np.flatnonzero(mask))
        return arr
    record.site = -1
    base = run(record)
    worst = 0.0
    for p in range(probes):
        rng = np.random.default_rng([int(seed), p])
        worst = max(worst, rel_err(run(lambda name, arr: arr * (1.0 + eps * (rng.integers(0, 2, size=arr.shape) * 2.0 - 1.0))), base))
    for e in (eps, 0.5 * eps):
        worst = max(worst, rel_err(run(lambda name, arr: _append_ties(arr, e)[1] if name in _APPENDED else arr), base))
    for _, site, idx in sorted(found)[:singles]:
        def one(name, arr, state={"site": -1}):
            if name not in _APPENDED:
                return arr
            state["site"] += 1
            if state["site"] != site:
                return arr
            out = np.array(arr, dtype=np.float64, copy=True)
            out.flat[idx] = _append_ties(arr, eps)[1].flat[idx]
            return out
        worst = max(worst, rel_err(run(one), base))
    return worst
