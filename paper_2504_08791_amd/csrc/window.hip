// C-ABI entry points: argument validation on the host, workspace carving and the per-layer
// launch sequence of a layer window (arXiv 2504.08791, Sec. 3.1: a device advances its window
// of consecutive layers and hands e FP32 values per token to its successor).
#include "common.h"

using namespace prima;

namespace {

struct WindowWs {
    size_t n, q, k, v, o, h, g, u, a, xb0, xb1, rope, attn, gemv, total;
};

bool dims_ok(const prima_dims *d)
{
    return d->e > 0 && d->e % QK == 0 && d->ffn > 0 && d->ffn % QK == 0 && d->n_kv_heads > 0 &&
           d->n_q_heads > 0 && d->n_q_heads % d->n_kv_heads == 0 && (d->head_dim == 64 || d->head_dim == 128) &&
           (static_cast<int64_t>(d->n_q_heads) * d->head_dim) % QK == 0 && (d->rope_mode == 0 || d->rope_mode == 1);
}

WindowWs carve(const prima_dims &d, int kv_cap, int T)
{
    WindowWs w{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
    const size_t qd = static_cast<size_t>(d.n_q_heads) * d.head_dim, kvd = static_cast<size_t>(d.n_kv_heads) * d.head_dim;
    const size_t f = sizeof(float);
    w.n = take(T * static_cast<size_t>(d.e) * f);
    w.q = take(T * qd * f);
    w.k = take(T * kvd * f);
    w.v = take(T * kvd * f);
    w.o = take(T * qd * f);
    w.h = take(T * static_cast<size_t>(d.e) * f);
    w.g = take(T * static_cast<size_t>(d.ffn) * f);
    w.u = take(T * static_cast<size_t>(d.ffn) * f);
    w.a = take(T * static_cast<size_t>(d.ffn) * f);
    w.xb0 = take(T * static_cast<size_t>(d.e) * f);
    w.xb1 = take(T * static_cast<size_t>(d.e) * f);
    w.rope = take(T * static_cast<size_t>(d.head_dim) * f);
    w.attn = take(attn_ws_bytes(d, kv_cap, T));
    const int64_t max_rows = 2 * static_cast<int64_t>(d.ffn) > static_cast<int64_t>(qd + 2 * kvd) ? 2 * d.ffn : qd + 2 * kvd;
    const int64_t max_cols = d.ffn > d.e ? d.ffn : d.e;
    w.gemv = take(gemv_ws_bytes(max_rows, max_cols, T));
    w.total = off;
    return w;
}

template <class P> P *at(void *ws, size_t off) { return reinterpret_cast<P *>(static_cast<char *>(ws) + off); }

GemvSeg seg(const void *W, float *y, int64_t rows, int64_t ldy, const float *resid = nullptr, int64_t ldr = 0)
{
    return GemvSeg{static_cast<const uint8_t *>(W), y, resid, rows, ldy, ldr};
}

prima_status check_layer(const prima_layer &l)
{
    const void *ptrs[] = {l.wq, l.wk, l.wv, l.wo, l.wgate, l.wup, l.wdown, l.g_attn, l.g_ffn, l.k_cache, l.v_cache};
    for (const void *p : ptrs) {
        if (!p) return PRIMA_E_NULL;
        if (!aligned(p, 16)) return PRIMA_E_ALIGN;
    }
    return PRIMA_OK;
}

// one decoder layer; x -> y (fp32 [T][e]); taps may be null
prima_status run_layer(const prima_dims &d, const prima_layer &L, int kv_cap, int n_past, int T,
                       const float *x, float *y, void *ws, const WindowWs &w, hipStream_t st,
                       float *tap_q, float *tap_o, float *tap_h, float *tap_a)
{
    const int64_t e = d.e, qd = static_cast<int64_t>(d.n_q_heads) * d.head_dim, kvd = static_cast<int64_t>(d.n_kv_heads) * d.head_dim, F = d.ffn;
    float *n = at<float>(ws, w.n), *q = at<float>(ws, w.q), *k = at<float>(ws, w.k), *v = at<float>(ws, w.v);
    float *o = at<float>(ws, w.o), *h = at<float>(ws, w.h), *g = at<float>(ws, w.g), *u = at<float>(ws, w.u), *a = at<float>(ws, w.a);
    void *gws = at<char>(ws, w.gemv);
    const size_t gws_bytes = w.total - w.gemv;
    prima_status s;
#define PRIMA_TRY(call) do { s = (call); if (s != PRIMA_OK) return s; } while (0)
    PRIMA_TRY(launch_rmsnorm(x, L.g_attn, n, T, d.e, d.rms_eps, st));
    {
        GemvArgs ga{};
        ga.seg[0] = seg(L.wq, q, qd, qd);
        ga.seg[1] = seg(L.wk, k, kvd, kvd);
        ga.seg[2] = seg(L.wv, v, kvd, kvd);
        ga.nseg = 3; ga.n_cols = e; ga.x = n; ga.ldx = e; ga.T = T;
        PRIMA_TRY(launch_gemv(ga, gws, gws_bytes, st));
    }
    PRIMA_TRY(launch_rope_kv_append(d, q, k, v, at<float>(ws, w.rope), static_cast<__half *>(L.k_cache),
                                    static_cast<__half *>(L.v_cache), kv_cap, n_past, T, st));
    if (tap_q && hipMemcpyAsync(tap_q, q, T * qd * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return PRIMA_E_DEVICE;
    PRIMA_TRY(launch_attn(d, q, static_cast<const __half *>(L.k_cache), static_cast<const __half *>(L.v_cache),
                          kv_cap, n_past, T, o, at<char>(ws, w.attn), st));
    if (tap_o && hipMemcpyAsync(tap_o, o, T * qd * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return PRIMA_E_DEVICE;
    {
        GemvArgs ga{};
        ga.seg[0] = seg(L.wo, h, e, e, x, e);
        ga.nseg = 1; ga.n_cols = qd; ga.x = o; ga.ldx = qd; ga.T = T;
        PRIMA_TRY(launch_gemv(ga, gws, gws_bytes, st));
    }
    if (tap_h && hipMemcpyAsync(tap_h, h, T * e * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return PRIMA_E_DEVICE;
    PRIMA_TRY(launch_rmsnorm(h, L.g_ffn, n, T, d.e, d.rms_eps, st));
    {
        GemvArgs ga{};
        ga.seg[0] = seg(L.wgate, g, F, F);
        ga.seg[1] = seg(L.wup, u, F, F);
        ga.nseg = 2; ga.n_cols = e; ga.x = n; ga.ldx = e; ga.T = T;
        PRIMA_TRY(launch_gemv(ga, gws, gws_bytes, st));
    }
    PRIMA_TRY(launch_swiglu(g, u, a, static_cast<int64_t>(T) * F, st));
    if (tap_a && hipMemcpyAsync(tap_a, a, T * F * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return PRIMA_E_DEVICE;
    {
        GemvArgs ga{};
        ga.seg[0] = seg(L.wdown, y, e, e, h, e);
        ga.nseg = 1; ga.n_cols = F; ga.x = a; ga.ldx = F; ga.T = T;
        PRIMA_TRY(launch_gemv(ga, gws, gws_bytes, st));
    }
#undef PRIMA_TRY
    return PRIMA_OK;
}

prima_status check_window_args(const prima_dims *d, int32_t kv_cap, int32_t n_past, int32_t T,
                               const float *x_in, float *x_out, void *ws, size_t ws_bytes)
{
    if (!d || !x_in || !x_out || !ws) return PRIMA_E_NULL;
    if (!dims_ok(d)) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK || n_past < 0 || kv_cap < 1 || static_cast<int64_t>(n_past) + T > kv_cap) return PRIMA_E_RANGE;
    if (!aligned(x_in, 16) || !aligned(x_out, 16) || !aligned(ws, 256)) return PRIMA_E_ALIGN;
    if (ws_bytes < carve(*d, kv_cap, T).total) return PRIMA_E_WORKSPACE;
    return PRIMA_OK;
}

} // namespace

extern "C" {

int prima_abi_version(void) { return PRIMA_ABI_VERSION; }

const char *prima_status_str(prima_status s)
{
    switch (s) {
    case PRIMA_OK: return "ok";
    case PRIMA_E_NULL: return "null pointer";
    case PRIMA_E_SHAPE: return "unsupported shape";
    case PRIMA_E_ALIGN: return "misaligned pointer or leading dimension";
    case PRIMA_E_RANGE: return "T, n_past or kv_cap out of range";
    case PRIMA_E_WORKSPACE: return "workspace too small";
    case PRIMA_E_DEVICE: return "kernel launch failed";
    }
    return "unknown status";
}

prima_status prima_q4k_dequant(const void *W, int64_t n_rows, int64_t n_cols, float *out, void *hip_stream)
{
    if (!W || !out) return PRIMA_E_NULL;
    if (n_rows < 0 || n_cols < 0 || n_cols % QK) return PRIMA_E_SHAPE;
    if (!aligned(W, 16) || !aligned(out, 16)) return PRIMA_E_ALIGN;
    return launch_dequant(static_cast<const uint8_t *>(W), n_rows, n_cols, out, static_cast<hipStream_t>(hip_stream));
}

size_t prima_gemv_workspace_bytes(int64_t n_rows, int64_t n_cols, int32_t T)
{
    if (n_rows < 0 || n_cols < 0 || T < 1) return 0;
    return gemv_ws_bytes(n_rows, n_cols, T);
}

prima_status prima_q4k_gemv(const void *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int32_t T,
                            float *y, int64_t ldy, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!W || !x || !y || !workspace) return PRIMA_E_NULL;
    if (n_rows < 0 || n_cols <= 0 || n_cols % QK || ldx < n_cols || ldy < n_rows) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK) return PRIMA_E_RANGE;
    if (!aligned(W, 16) || !aligned(x, 16) || !aligned(y, 4) || ldx % 4 || !aligned(workspace, 256)) return PRIMA_E_ALIGN;
    if (workspace_bytes < gemv_ws_bytes(n_rows, n_cols, T)) return PRIMA_E_WORKSPACE;
    GemvArgs ga{};
    ga.seg[0] = seg(W, y, n_rows, ldy);
    ga.nseg = 1; ga.n_cols = n_cols; ga.x = x; ga.ldx = ldx; ga.T = T;
    return launch_gemv(ga, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream));
}

size_t prima_attn_workspace_bytes(const prima_dims *d, int32_t kv_cap, int32_t T)
{
    if (!d || !dims_ok(d) || T < 1) return 0;
    return attn_ws_bytes(*d, kv_cap, T);
}

prima_status prima_attn_decode(const prima_dims *d, const float *q, const void *k_cache, const void *v_cache,
                               int32_t kv_cap, int32_t n_past, int32_t T, float *o,
                               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d || !q || !k_cache || !v_cache || !o || !workspace) return PRIMA_E_NULL;
    if (!dims_ok(d)) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK || n_past < 0 || kv_cap < 1 || static_cast<int64_t>(n_past) + T > kv_cap) return PRIMA_E_RANGE;
    if (!aligned(q, 16) || !aligned(o, 16) || !aligned(k_cache, 16) || !aligned(v_cache, 16) || !aligned(workspace, 256)) return PRIMA_E_ALIGN;
    if (workspace_bytes < attn_ws_bytes(*d, kv_cap, T)) return PRIMA_E_WORKSPACE;
    return launch_attn(*d, q, static_cast<const __half *>(k_cache), static_cast<const __half *>(v_cache), kv_cap, n_past, T, o,
                       workspace, static_cast<hipStream_t>(hip_stream));
}

size_t prima_workspace_bytes(const prima_dims *d, int32_t kv_cap, int32_t T)
{
    if (!d || !dims_ok(d) || T < 1 || T > PRIMA_MAX_TOK || kv_cap < 0) return 0;
    return carve(*d, kv_cap, T).total;
}

prima_status prima_layer_window_decode(const prima_dims *d, const prima_layer *layers, int32_t L,
                                       int32_t kv_cap, int32_t n_past, int32_t T,
                                       const float *x_in, float *x_out,
                                       void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!layers) return PRIMA_E_NULL;
    prima_status s = check_window_args(d, kv_cap, n_past, T, x_in, x_out, workspace, workspace_bytes);
    if (s != PRIMA_OK) return s;
    if (L < 1) return PRIMA_E_RANGE;
    for (int i = 0; i < L; ++i)
        if ((s = check_layer(layers[i])) != PRIMA_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const WindowWs w = carve(*d, kv_cap, T);
    s = launch_rope_table(at<float>(workspace, w.rope), T, d->head_dim, n_past, d->rope_theta, st);
    if (s != PRIMA_OK) return s;
    const float *cur = x_in;
    for (int i = 0; i < L; ++i) {
        float *dst = (i == L - 1) ? x_out : at<float>(workspace, (i & 1) ? w.xb1 : w.xb0);
        s = run_layer(*d, layers[i], kv_cap, n_past, T, cur, dst, workspace, w, st, nullptr, nullptr, nullptr, nullptr);
        if (s != PRIMA_OK) return s;
        cur = dst;
    }
    return PRIMA_OK;
}

prima_status prima_layer_decode_taps(const prima_dims *d, const prima_layer *layer,
                                     int32_t kv_cap, int32_t n_past, int32_t T,
                                     const float *x_in, float *x_out,
                                     float *tap_q, float *tap_o, float *tap_h, float *tap_a,
                                     void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!layer) return PRIMA_E_NULL;
    prima_status s = check_window_args(d, kv_cap, n_past, T, x_in, x_out, workspace, workspace_bytes);
    if (s != PRIMA_OK) return s;
    if ((s = check_layer(*layer)) != PRIMA_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const WindowWs w = carve(*d, kv_cap, T);
    s = launch_rope_table(at<float>(workspace, w.rope), T, d->head_dim, n_past, d->rope_theta, st);
    if (s != PRIMA_OK) return s;
    return run_layer(*d, *layer, kv_cap, n_past, T, x_in, x_out, workspace, w, st, tap_q, tap_o, tap_h, tap_a);
}

prima_status prima_lm_head(const prima_dims *d, const float *g_final, const void *w_lm, int64_t vocab,
                           const float *x, int32_t T, float *logits,
                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d || !g_final || !w_lm || !x || !logits || !workspace) return PRIMA_E_NULL;
    if (!dims_ok(d) || vocab < 1) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK) return PRIMA_E_RANGE;
    if (!aligned(g_final, 16) || !aligned(w_lm, 16) || !aligned(x, 16) || !aligned(logits, 4) || !aligned(workspace, 256)) return PRIMA_E_ALIGN;
    const WindowWs w = carve(*d, 0, T);
    if (workspace_bytes < w.total) return PRIMA_E_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    float *n = at<float>(workspace, w.n);
    prima_status s = launch_rmsnorm(x, g_final, n, T, d->e, d->rms_eps, st);
    if (s != PRIMA_OK) return s;
    GemvArgs ga{};
    ga.seg[0] = seg(w_lm, logits, vocab, vocab);
    ga.nseg = 1; ga.n_cols = d->e; ga.x = n; ga.ldx = d->e; ga.T = T;
    return launch_gemv(ga, at<char>(workspace, w.gemv), w.total - w.gemv, st);
}

} // extern "C"
