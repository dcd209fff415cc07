"""MI355X decode hot path of a prima.cpp layer window: thin Python binding.

Every function marshals torch CUDA tensors (device memory and streams only) into the C ABI of
include/prima.h; all computation happens in the HIP library.  There is no CPU path.
"""
import ctypes as C

import torch

from . import _ffi
from ._ffi import Dims, Layer, PrimaError, MAX_TOK  # noqa: F401

_WEIGHTS = ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _need(t, dtype, name):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous CUDA tensor of {dtype}")
    return t


def make_dims(d):
    """ModelDims-like object (fields e, n_q_heads, n_kv_heads, head_dim, ffn, rope_theta, rms_eps, rope_mode)."""
    if isinstance(d, Dims):
        return d
    return Dims(d.e, d.n_q_heads, d.n_kv_heads, d.head_dim, d.ffn, d.rope_theta, d.rms_eps, d.rope_mode)


def abi_version():
    return _ffi.lib().prima_abi_version()


def q4k_dequant(W):
    """W uint8 [rows, cols/256, 144] -> float32 [rows, cols]."""
    _need(W, torch.uint8, "W")
    rows, nb = W.shape[0], W.shape[1]
    out = torch.empty((rows, nb * 256), dtype=torch.float32, device=W.device)
    _ffi.check(_ffi.lib().prima_q4k_dequant(_ptr(W), rows, nb * 256, _ptr(out), _stream()), "prima_q4k_dequant")
    return out


def gemv_workspace_bytes(rows, cols, T):
    return _ffi.lib().prima_gemv_workspace_bytes(rows, cols, T)


def q4k_gemv(W, x, y=None, workspace=None):
    """y[t, r] = sum_c W[r, c] x[t, c];  W uint8 [rows, cols/256, 144], x float32 [T, cols]."""
    _need(W, torch.uint8, "W")
    _need(x, torch.float32, "x")
    rows, cols = W.shape[0], W.shape[1] * 256
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, rows), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(256, gemv_workspace_bytes(rows, cols, T)), dtype=torch.uint8, device=x.device)
    _ffi.check(_ffi.lib().prima_q4k_gemv(_ptr(W), rows, cols, _ptr(x), x.stride(0), T, _ptr(y), y.stride(0),
                                         _ptr(workspace), workspace.numel(), _stream()), "prima_q4k_gemv")
    return y


def q4k_gemv_noalloc(W, x, y):
    """q4k_gemv with the library's fixed scratch (no workspace argument, nothing allocated): y must be given."""
    _need(W, torch.uint8, "W")
    _need(x, torch.float32, "x")
    if not (y.is_cuda and y.dtype == torch.float32 and y.dim() == 2 and y.stride(1) == 1):
        raise TypeError("y: need a 2-d CUDA float32 tensor with contiguous rows")
    rows, cols = W.shape[0], W.shape[1] * 256
    _ffi.check(_ffi.lib().prima_q4k_gemv_noalloc(_ptr(W), rows, cols, _ptr(x), x.stride(0), x.shape[0], _ptr(y), y.stride(0),
                                                 _stream()), "prima_q4k_gemv_noalloc")
    return y


def gemm_ksplit(T, rows, cols):
    """Into how many shares prima_q4k_gemm divides K for this shape when its workspace has room for them (1: none)."""
    return _ffi.lib().prima_gemm_ksplit(T, rows, cols)


def gemm_workspace_bytes(T, rows, cols, ksplit=True):
    """Workspace of q4k_gemm: the minimum, or (ksplit) the size with which few rows x few tokens divide K."""
    if ksplit:
        return _ffi.lib().prima_gemm_workspace_bytes_ksplit(T, rows, cols)
    return _ffi.lib().prima_gemm_workspace_bytes(T, cols)


def q4k_gemm(W, x, gain=None, eps=0.0, resid=None, y=None, workspace=None):
    """Many tokens: y[t, r] = sum_c W[r, c] a[t, c] (+ resid[t, r]), a = x or RMSNorm(x; gain, eps).
    W uint8 [rows, cols/256, 144], x float32 [T, cols] (rows may be strided)."""
    _need(W, torch.uint8, "W")
    if x.dtype != torch.float32 or not x.is_cuda or x.stride(1) != 1:
        raise ValueError("x must be a float32 CUDA tensor with contiguous rows")
    rows, cols = W.shape[0], W.shape[1] * 256
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, rows), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(256, _ffi.lib().prima_gemm_workspace_bytes_ksplit(T, rows, cols)), dtype=torch.uint8, device=x.device)
    if gain is not None:
        _need(gain, torch.float32, "gain")
    if resid is not None and (resid.dtype != torch.float32 or resid.stride(1) != 1):
        raise ValueError("resid must be float32 with contiguous rows")
    _ffi.check(_ffi.lib().prima_q4k_gemm(_ptr(W), rows, cols, _ptr(x), x.stride(0), T, _ptr(gain) if gain is not None else None,
                                         float(eps), _ptr(resid) if resid is not None else None,
                                         resid.stride(0) if resid is not None else 0, _ptr(y), y.stride(0),
                                         _ptr(workspace), workspace.numel(), _stream()), "prima_q4k_gemm")
    return y


def fmt_tensor_bytes(fmt, rows, cols):
    return _ffi.lib().prima_fmt_tensor_bytes(_ffi.FORMATS[fmt], rows, cols)


def fmt_dequant(fmt, W, rows, cols):
    """W: flat uint8 tensor in format fmt ("q5_k", "q6_k", "q8_0", "f16", "f32", "q4_k") -> float32 [rows, cols]."""
    _need(W, torch.uint8, "W")
    if W.numel() != fmt_tensor_bytes(fmt, rows, cols):
        raise ValueError(f"W holds {W.numel()} bytes, a {rows} x {cols} {fmt} tensor has {fmt_tensor_bytes(fmt, rows, cols)}")
    out = torch.empty((rows, cols), dtype=torch.float32, device=W.device)
    _ffi.check(_ffi.lib().prima_fmt_dequant(_ffi.FORMATS[fmt], _ptr(W), rows, cols, _ptr(out), _stream()), "prima_fmt_dequant")
    return out


def gguf_tensor_bytes(fmt, rows, cols):
    return _ffi.lib().prima_gguf_tensor_bytes(_ffi.FORMATS[fmt], rows, cols)


def repack_gguf(fmt, raw, rows, cols, out=None):
    """raw: flat uint8 CUDA tensor holding a rows x cols tensor in GGUF block order -> flat uint8 in this library's layout."""
    _need(raw, torch.uint8, "raw")
    if raw.numel() != gguf_tensor_bytes(fmt, rows, cols):
        raise ValueError(f"raw holds {raw.numel()} bytes, a {rows} x {cols} {fmt} tensor has {gguf_tensor_bytes(fmt, rows, cols)}")
    if out is None:
        out = torch.empty(fmt_tensor_bytes(fmt, rows, cols), dtype=torch.uint8, device=raw.device)
    _need(out, torch.uint8, "out")
    if out.numel() != fmt_tensor_bytes(fmt, rows, cols):
        raise ValueError("out has the wrong size")
    _ffi.check(_ffi.lib().prima_repack_gguf(_ffi.FORMATS[fmt], _ptr(raw), rows, cols, _ptr(out), _stream()), "prima_repack_gguf")
    return out


def fmt_gemv(fmt, W, rows, cols, x, y=None):
    """y[t, r] = sum_c W[r, c] x[t, c];  W flat uint8 in format fmt (not "q4_k"), x float32 [T, cols]."""
    _need(W, torch.uint8, "W")
    for t, name in ((x, "x"), (y, "y")):     # rows may be strided (ldx, ldy), elements of a row may not
        if t is not None and not (t.is_cuda and t.dtype == torch.float32 and t.dim() == 2 and t.stride(1) == 1):
            raise TypeError(f"{name}: need a 2-d CUDA float32 tensor with contiguous rows")
    if W.numel() != fmt_tensor_bytes(fmt, rows, cols):
        raise ValueError(f"W holds {W.numel()} bytes, a {rows} x {cols} {fmt} tensor has {fmt_tensor_bytes(fmt, rows, cols)}")
    T = x.shape[0]
    if y is None:
        y = torch.empty((T, rows), dtype=torch.float32, device=x.device)
    _ffi.check(_ffi.lib().prima_fmt_gemv(_ffi.FORMATS[fmt], _ptr(W), rows, cols, _ptr(x), x.stride(0), T, _ptr(y), y.stride(0),
                                         _stream()), "prima_fmt_gemv")
    return y


def lm_head_fmt(dims, fmt, g_final, w_lm, vocab, x, logits=None):
    """logits[t, v] = W_lm . rmsnorm(x[t]; g_final) with W_lm flat uint8 in format fmt (not "q4_k")."""
    d = make_dims(dims)
    _need(g_final, torch.float32, "g_final")
    _need(w_lm, torch.uint8, "w_lm")
    _need(x, torch.float32, "x")
    if w_lm.numel() != fmt_tensor_bytes(fmt, vocab, d.e):
        raise ValueError("w_lm has the wrong size for its format")
    T = x.shape[0]
    if logits is None:
        logits = torch.empty((T, vocab), dtype=torch.float32, device=x.device)
    _ffi.check(_ffi.lib().prima_lm_head_fmt(C.byref(d), _ffi.FORMATS[fmt], _ptr(g_final), _ptr(w_lm), vocab, _ptr(x), T,
                                            _ptr(logits), _stream()), "prima_lm_head_fmt")
    return logits


def attn_workspace_bytes(dims, kv_cap, T):
    d = make_dims(dims)
    return _ffi.lib().prima_attn_workspace_bytes(C.byref(d), kv_cap, T)


def attn_decode(dims, q, k_cache, v_cache, n_past, o=None, workspace=None):
    """q float32 [T, Hq, D]; caches float16 [Hkv, cap, D] with rows < n_past + T valid -> o like q."""
    d = make_dims(dims)
    _need(q, torch.float32, "q")
    _need(k_cache, torch.float16, "k_cache")
    _need(v_cache, torch.float16, "v_cache")
    T, cap = q.shape[0], k_cache.shape[1]
    if o is None:
        o = torch.empty_like(q)
    if workspace is None:
        workspace = torch.empty(max(256, attn_workspace_bytes(d, cap, T)), dtype=torch.uint8, device=q.device)
    _ffi.check(_ffi.lib().prima_attn_decode(C.byref(d), _ptr(q), _ptr(k_cache), _ptr(v_cache), cap, n_past, T, _ptr(o),
                                            _ptr(workspace), workspace.numel(), _stream()), "prima_attn_decode")
    return o


def workspace_bytes(dims, kv_cap, T):
    d = make_dims(dims)
    return _ffi.lib().prima_workspace_bytes(C.byref(d), kv_cap, T)


def window_plan_status(dims, kv_cap, T):
    """Host-side check (no GPU work): 0 if a window step of T tokens with these dimensions can be launched."""
    d = make_dims(dims)
    return _ffi.lib().prima_window_plan_status(C.byref(d), kv_cap, T)


def stream_read_probe(buf, sink, nt=False):
    """Measurement hook: one linear read of the uint8 tensor `buf` (discarded); `sink` any 4-byte device tensor.
    nt: with the non-temporal bit on the loads (prima_stream_read_probe_nt)."""
    fn = _ffi.lib().prima_stream_read_probe_nt if nt else _ffi.lib().prima_stream_read_probe
    _ffi.check(fn(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream()),
               "prima_stream_read_probe_nt" if nt else "prima_stream_read_probe")


PREFILL_SMALL_TOKENS = 16   # the library's default threshold (prima_set_prefill_small_tokens)


def set_prefill_small_tokens(n):
    """Prompts of up to n tokens go through the decode kernels inside Window.prefill (default 16; 0: always the matrix product)."""
    _ffi.lib().prima_set_prefill_small_tokens(int(n))


class Window:
    """A window of decoder layers resident in HBM: keeps the tensors alive, the descriptor array
    and a workspace, so that a step is a single C call."""

    def __init__(self, dims, layers, kv_cap, T_max=MAX_TOK, formats=None):
        """formats: optional list (one dict per layer) naming the format of matrices that are not Q4_K, e.g.
        {"wv": "q6_k", "wdown": "q6_k"}; such tensors are flat uint8 of fmt_tensor_bytes(...) bytes."""
        self.dims = make_dims(dims)
        self._formats = None
        if formats is not None:
            if len(formats) != len(layers):
                raise ValueError("formats needs one entry per layer")
            self._formats = (_ffi.LayerFormats * len(layers))()
            for i, f in enumerate(formats):
                for k in _WEIGHTS:
                    setattr(self._formats[i], k, _ffi.FORMATS[(f or {}).get(k, "q4_k")])
        self.layers = layers
        self.kv_cap = kv_cap
        self.T_max = T_max
        arr = (Layer * len(layers))()
        for i, t in enumerate(layers):
            for k in _WEIGHTS:
                _need(t[k], torch.uint8, k)
            _need(t["g_attn"], torch.float32, "g_attn")
            _need(t["g_ffn"], torch.float32, "g_ffn")
            _need(t["k_cache"], torch.float16, "k_cache")
            _need(t["v_cache"], torch.float16, "v_cache")
            if t["k_cache"].shape[1] != kv_cap or t["v_cache"].shape[1] != kv_cap:
                raise ValueError("kv_cap does not match the cache tensors")
            for k in _WEIGHTS + ("g_attn", "g_ffn", "k_cache", "v_cache"):
                setattr(arr[i], k, t[k].data_ptr())
        self._arr = arr
        dev = layers[0]["wq"].device
        self.workspace = torch.empty(max(256, workspace_bytes(self.dims, kv_cap, T_max)), dtype=torch.uint8, device=dev)

    def decode(self, x_in, n_past, x_out=None):
        """Advance all layers by T = x_in.shape[0] tokens; returns x_out float32 [T, e]."""
        _need(x_in, torch.float32, "x_in")
        T = x_in.shape[0]
        if x_out is None:
            x_out = torch.empty_like(x_in)
        if self._formats is not None:
            _ffi.check(_ffi.lib().prima_layer_window_decode_mixed(C.byref(self.dims), self._arr, self._formats, len(self.layers),
                                                                  self.kv_cap, n_past, T, _ptr(x_in), _ptr(x_out), _ptr(self.workspace),
                                                                  self.workspace.numel(), _stream()), "prima_layer_window_decode_mixed")
            return x_out
        _ffi.check(_ffi.lib().prima_layer_window_decode(C.byref(self.dims), self._arr, len(self.layers), self.kv_cap,
                                                        n_past, T, _ptr(x_in), _ptr(x_out), _ptr(self.workspace),
                                                        self.workspace.numel(), _stream()), "prima_layer_window_decode")
        return x_out

    def prefill(self, x_in, n_past, x_out=None):
        """Prompt processing: all layers for the T = x_in.shape[0] consecutive tokens that follow the n_past cached
        ones; returns x_out float32 [T, e].  The scratch is kept for the next call of this size."""
        _need(x_in, torch.float32, "x_in")
        T = x_in.shape[0]
        need = _ffi.lib().prima_prefill_workspace_bytes(C.byref(self.dims), self.kv_cap, T)
        if need == 0:
            raise ValueError("unsupported shape or token count")
        ws = getattr(self, "_prefill_ws", None)
        if ws is None or ws.numel() < need:
            ws = self._prefill_ws = torch.empty(need, dtype=torch.uint8, device=x_in.device)
        if x_out is None:
            x_out = torch.empty_like(x_in)
        _ffi.check(_ffi.lib().prima_layer_window_prefill_mixed(C.byref(self.dims), self._arr, self._formats, len(self.layers), self.kv_cap,
                                                               n_past, T, _ptr(x_in), _ptr(x_out), _ptr(ws), ws.numel(), _stream()),
                   "prima_layer_window_prefill")
        return x_out

    def decode_batch(self, x_in, n_past, caches, x_out=None):
        """One token for each of B = x_in.shape[0] independent sequences: n_past[b] cached rows of sequence b,
        caches[l][b] = (k_cache, v_cache) of layer l for sequence b (float16 [Hkv, kv_cap, D]); the window's own
        caches are not touched.  Returns x_out float32 [B, e]."""
        _need(x_in, torch.float32, "x_in")
        B, L = x_in.shape[0], len(self.layers)
        if len(n_past) != B or len(caches) != L or any(len(c) != B for c in caches):
            raise ValueError("n_past needs B entries and caches L x B pairs")
        for per_layer in caches:
            for k, v in per_layer:
                _need(k, torch.float16, "k_cache")
                _need(v, torch.float16, "v_cache")
                if k.shape[1] != self.kv_cap or v.shape[1] != self.kv_cap:
                    raise ValueError("kv_cap does not match the cache tensors")
        if x_out is None:
            x_out = torch.empty_like(x_in)
        np_arr = (C.c_int32 * B)(*[int(n) for n in n_past])
        k_arr = (C.c_void_p * (L * B))(*[caches[l][b][0].data_ptr() for l in range(L) for b in range(B)])
        v_arr = (C.c_void_p * (L * B))(*[caches[l][b][1].data_ptr() for l in range(L) for b in range(B)])
        _ffi.check(_ffi.lib().prima_layer_window_decode_batch_mixed(C.byref(self.dims), self._arr, self._formats, L, self.kv_cap, B,
                                                                    np_arr, k_arr, v_arr, _ptr(x_in), _ptr(x_out), _ptr(self.workspace),
                                                                    self.workspace.numel(), _stream()),
                   "prima_layer_window_decode_batch")
        return x_out

    def check(self, T=1):
        """Waits for the stream; raises if a bounded wait inside a kernel of the last step gave up."""
        _ffi.check(_ffi.lib().prima_window_check(C.byref(self.dims), self.kv_cap, T, _ptr(self.workspace),
                                                 self.workspace.numel(), _stream()), "prima_window_check")

    def decode_profiled(self, x_in, n_past, x_out=None):
        """Measurement hook: one step with an event after every launch; synchronises.
        Returns (x_out, {kind: (milliseconds, launches)})."""
        _need(x_in, torch.float32, "x_in")
        T = x_in.shape[0]
        if x_out is None:
            x_out = torch.empty_like(x_in)
        n = len(_ffi.KINDS)
        ms = (C.c_float * n)()
        cnt = (C.c_int32 * n)()
        _ffi.check(_ffi.lib().prima_layer_window_decode_profiled(
            C.byref(self.dims), self._arr, len(self.layers), self.kv_cap, n_past, T, _ptr(x_in), _ptr(x_out),
            _ptr(self.workspace), self.workspace.numel(), _stream(), ms, cnt), "prima_layer_window_decode_profiled")
        return x_out, {k: (ms[i], cnt[i]) for i, k in enumerate(_ffi.KINDS)}

    def decode_layer_taps(self, layer_index, x_in, n_past):
        """Test hook: one layer with intermediates (q, o, h, a)."""
        d = self.dims
        T = x_in.shape[0]
        dev = x_in.device
        qd = d.n_q_heads * d.head_dim
        taps = {"q": torch.empty((T, qd), dtype=torch.float32, device=dev),
                "o": torch.empty((T, qd), dtype=torch.float32, device=dev),
                "h": torch.empty((T, d.e), dtype=torch.float32, device=dev),
                "a": torch.empty((T, d.ffn), dtype=torch.float32, device=dev)}
        x_out = torch.empty_like(x_in)
        one = C.cast(C.byref(self._arr, layer_index * C.sizeof(Layer)), C.POINTER(Layer))
        _ffi.check(_ffi.lib().prima_layer_decode_taps(C.byref(d), one, self.kv_cap, n_past, T, _ptr(x_in), _ptr(x_out),
                                                      _ptr(taps["q"]), _ptr(taps["o"]), _ptr(taps["h"]), _ptr(taps["a"]),
                                                      _ptr(self.workspace), self.workspace.numel(), _stream()),
                   "prima_layer_decode_taps")
        return x_out, taps


def lm_head_workspace_bytes(dims, vocab, T):
    d = make_dims(dims)
    return _ffi.lib().prima_lm_head_workspace_bytes(C.byref(d), vocab, T)


def lm_head(dims, g_final, w_lm, x, logits=None, workspace=None):
    """logits[t, v] = W_lm . rmsnorm(x[t]; g_final)."""
    d = make_dims(dims)
    _need(g_final, torch.float32, "g_final")
    _need(w_lm, torch.uint8, "w_lm")
    _need(x, torch.float32, "x")
    T, vocab = x.shape[0], w_lm.shape[0]
    if logits is None:
        logits = torch.empty((T, vocab), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(256, lm_head_workspace_bytes(d, vocab, T)), dtype=torch.uint8, device=x.device)
    _ffi.check(_ffi.lib().prima_lm_head(C.byref(d), _ptr(g_final), _ptr(w_lm), vocab, _ptr(x), T, _ptr(logits),
                                        _ptr(workspace), workspace.numel(), _stream()), "prima_lm_head")
    return logits
