"""ctypes view of the C ABI declared in include/prima.h.  No arithmetic lives here."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libprima_hip.so")

MAX_TOK = 16
NOALLOC_SCRATCH_BYTES = 4 << 20
KINDS = ("qkv", "rope_kv", "attn", "wo", "gate_up", "down")
STATUS = {0: "PRIMA_OK", 1: "PRIMA_E_NULL", 2: "PRIMA_E_SHAPE", 3: "PRIMA_E_ALIGN", 4: "PRIMA_E_RANGE",
          5: "PRIMA_E_WORKSPACE", 6: "PRIMA_E_DEVICE"}

EXPORTS = ["prima_q4k_gemv", "prima_gemv_workspace_bytes", "prima_q4k_dequant", "prima_attn_decode",
           "prima_attn_workspace_bytes", "prima_layer_window_decode", "prima_layer_window_decode_profiled", "prima_layer_decode_taps",
           "prima_lm_head", "prima_lm_head_workspace_bytes", "prima_workspace_bytes", "prima_status_str", "prima_abi_version",
           "prima_window_check", "prima_stream_read_probe", "prima_stream_read_probe_nt", "prima_layer_window_decode_batch",
           "prima_fmt_tensor_bytes", "prima_fmt_dequant", "prima_fmt_gemv", "prima_lm_head_fmt", "prima_layer_window_decode_mixed", "prima_window_plan_status", "prima_gemv_plan_status", "prima_layer_window_decode_batch_mixed",
           "prima_q4k_gemm", "prima_gemm_workspace_bytes", "prima_gemm_workspace_bytes_ksplit", "prima_gemm_ksplit", "prima_layer_window_prefill", "prima_prefill_workspace_bytes",
           "prima_layer_window_prefill_mixed", "prima_set_prefill_small_tokens", "prima_q4k_gemv_noalloc",
           "prima_gguf_tensor_bytes", "prima_repack_gguf"]
FORMATS = {"q4_k": 0, "q5_k": 1, "q6_k": 2, "q8_0": 3, "f16": 4, "f32": 5}


class Dims(C.Structure):
    _fields_ = [("e", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("rope_mode", C.c_int32)]


class Layer(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown",
                                          "g_attn", "g_ffn", "k_cache", "v_cache")]


class LayerFormats(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("wq", "wk", "wv", "wo", "wgate", "wup", "wdown")]


class PrimaError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {STATUS.get(code, code)}")


_lib = None


def lib():
    """The HIP library.  There is no fallback: a missing build is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        dp, lp = C.POINTER(Dims), C.POINTER(Layer)
        L.prima_q4k_gemv.argtypes = [vp, i64, i64, vp, i64, i32, vp, i64, vp, sz, vp]
        L.prima_q4k_gemv_noalloc.argtypes = [vp, i64, i64, vp, i64, i32, vp, i64, vp]
        L.prima_q4k_gemv_noalloc.restype = C.c_int
        L.prima_gemv_workspace_bytes.argtypes = [i64, i64, i32]
        L.prima_gemv_workspace_bytes.restype = sz
        L.prima_q4k_dequant.argtypes = [vp, i64, i64, vp, vp]
        L.prima_q4k_gemm.argtypes = [vp, i64, i64, vp, i64, i32, vp, C.c_float, vp, i64, vp, i64, vp, sz, vp]
        L.prima_q4k_gemm.restype = C.c_int
        L.prima_gemm_workspace_bytes.argtypes = [i32, i64]
        L.prima_gemm_workspace_bytes.restype = sz
        L.prima_gemm_workspace_bytes_ksplit.argtypes = [i32, i64, i64]
        L.prima_gemm_workspace_bytes_ksplit.restype = sz
        L.prima_gemm_ksplit.argtypes = [i32, i64, i64]
        L.prima_gemm_ksplit.restype = i32
        L.prima_layer_window_prefill.argtypes = [dp, lp, i32, i32, i32, i32, vp, vp, vp, sz, vp]
        L.prima_layer_window_prefill.restype = C.c_int
        L.prima_prefill_workspace_bytes.argtypes = [dp, i32, i32]
        L.prima_layer_window_prefill_mixed.argtypes = [dp, lp, C.POINTER(LayerFormats), i32, i32, i32, i32, vp, vp, vp, sz, vp]
        L.prima_layer_window_prefill_mixed.restype = C.c_int
        L.prima_prefill_workspace_bytes.restype = sz
        L.prima_attn_decode.argtypes = [dp, vp, vp, vp, i32, i32, i32, vp, vp, sz, vp]
        L.prima_attn_workspace_bytes.argtypes = [dp, i32, i32]
        L.prima_attn_workspace_bytes.restype = sz
        L.prima_layer_window_decode.argtypes = [dp, lp, i32, i32, i32, i32, vp, vp, vp, sz, vp]
        L.prima_layer_window_decode_profiled.argtypes = [dp, lp, i32, i32, i32, i32, vp, vp, vp, sz, vp,
                                                         C.POINTER(C.c_float), C.POINTER(C.c_int32)]
        L.prima_layer_window_decode_batch.argtypes = [dp, lp, i32, i32, i32, C.POINTER(C.c_int32), C.POINTER(C.c_void_p),
                                                      C.POINTER(C.c_void_p), vp, vp, vp, sz, vp]
        L.prima_layer_window_decode_batch.restype = C.c_int
        L.prima_layer_window_decode_batch_mixed.argtypes = [dp, lp, C.POINTER(LayerFormats), i32, i32, i32, C.POINTER(C.c_int32),
                                                            C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), vp, vp, vp, sz, vp]
        L.prima_layer_window_decode_batch_mixed.restype = C.c_int
        L.prima_layer_decode_taps.argtypes = [dp, lp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.prima_lm_head.argtypes = [dp, vp, vp, i64, vp, i32, vp, vp, sz, vp]
        L.prima_lm_head_workspace_bytes.argtypes = [dp, i64, i32]
        L.prima_lm_head_workspace_bytes.restype = sz
        L.prima_fmt_tensor_bytes.argtypes = [i32, i64, i64]
        L.prima_fmt_tensor_bytes.restype = sz
        L.prima_fmt_dequant.argtypes = [i32, vp, i64, i64, vp, vp]
        L.prima_fmt_dequant.restype = C.c_int
        L.prima_fmt_gemv.argtypes = [i32, vp, i64, i64, vp, i64, i32, vp, i64, vp]
        L.prima_fmt_gemv.restype = C.c_int
        L.prima_lm_head_fmt.argtypes = [dp, i32, vp, vp, i64, vp, i32, vp, vp]
        L.prima_lm_head_fmt.restype = C.c_int
        L.prima_layer_window_decode_mixed.argtypes = [dp, lp, C.POINTER(LayerFormats), i32, i32, i32, i32, vp, vp, vp, sz, vp]
        L.prima_layer_window_decode_mixed.restype = C.c_int
        L.prima_gemv_plan_status.argtypes = [i64, i64, i32]
        L.prima_gemv_plan_status.restype = C.c_int
        L.prima_window_plan_status.argtypes = [dp, i32, i32]
        L.prima_window_plan_status.restype = C.c_int
        L.prima_workspace_bytes.argtypes = [dp, i32, i32]
        L.prima_workspace_bytes.restype = sz
        L.prima_stream_read_probe.argtypes = [vp, sz, vp, vp]
        L.prima_stream_read_probe_nt.argtypes = [vp, sz, vp, vp]
        L.prima_window_check.argtypes = [dp, i32, i32, vp, sz, vp]
        L.prima_status_str.argtypes = [C.c_int]
        L.prima_status_str.restype = C.c_char_p
        L.prima_abi_version.restype = C.c_int
        for name in ("prima_q4k_gemv", "prima_q4k_dequant", "prima_attn_decode", "prima_layer_window_decode",
                     "prima_layer_window_decode_profiled",
                     "prima_layer_decode_taps", "prima_lm_head", "prima_window_check", "prima_stream_read_probe", "prima_stream_read_probe_nt"):
            getattr(L, name).restype = C.c_int
        L.prima_gguf_tensor_bytes.argtypes = [i32, i64, i64]
        L.prima_gguf_tensor_bytes.restype = sz
        L.prima_repack_gguf.argtypes = [i32, vp, i64, i64, vp, vp]
        L.prima_repack_gguf.restype = C.c_int
        L.prima_set_prefill_small_tokens.argtypes = [i32]
        L.prima_set_prefill_small_tokens.restype = None
        _lib = L
    return _lib


def check(code, where):
    if code != 0:
        raise PrimaError(code, where)
