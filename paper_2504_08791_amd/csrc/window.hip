// C-ABI entry points: argument validation on the host, workspace carving and the per-layer
// launch sequence of a layer window (arXiv 2504.08791, Sec. 3.1: a device advances its window
// of consecutive layers and hands e FP32 values per token to its successor).
#include <algorithm>
#include <mutex>

#include "attn_common.h"

using namespace prima;

namespace {

struct WindowWs {
    size_t q, k, v, o, h, a, u, xb0, xb1, rope, attn, gemv, gemv_bytes, arrivals_bytes, sync, total;
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
    w.q = take(T * qd * f);
    w.k = take(T * kvd * f);
    w.v = take(T * kvd * f);
    w.o = take(T * qd * f);
    w.h = take(T * static_cast<size_t>(d.e) * f);
    w.a = take(T * static_cast<size_t>(d.ffn) * f);
    w.u = take(T * static_cast<size_t>(d.ffn) * f); // up projection, when gate / up are not both Q4_K
    w.xb0 = take(T * static_cast<size_t>(d.e) * f);
    w.xb1 = take(T * static_cast<size_t>(d.e) * f);
    w.rope = take(T * static_cast<size_t>(d.head_dim) * f);
    w.attn = take(attn_ws_bytes(d, kv_cap, T));
    // mat-vec scratch: sized for the largest of the layer's (and the output layer's) launches
    const int64_t rows_max = std::max<int64_t>({2 * static_cast<int64_t>(d.ffn), static_cast<int64_t>(qd + 2 * kvd), static_cast<int64_t>(d.e)});
    // (the last five: subsets of a group, launched when its other matrices are in other formats)
    const int64_t shapes[9][2] = {{static_cast<int64_t>(qd + 2 * kvd), d.e}, {d.e, static_cast<int64_t>(qd)}, {2 * static_cast<int64_t>(d.ffn), d.e}, {d.e, d.ffn},
                                  {static_cast<int64_t>(qd), d.e}, {static_cast<int64_t>(kvd), d.e}, {static_cast<int64_t>(qd + kvd), d.e},
                                  {static_cast<int64_t>(2 * kvd), d.e}, {d.ffn, d.e}};
    w.gemv_bytes = 0;
    w.arrivals_bytes = gemv_arrivals_bytes(rows_max);
    for (const auto &sh : shapes) w.gemv_bytes = std::max(w.gemv_bytes, gemv_ws_bytes(sh[0], sh[1], T)); // counters + partial sums
    w.gemv_bytes += w.arrivals_bytes; // the counter region is sized for the tallest matrix
    w.gemv = take(w.gemv_bytes);
    w.sync = take(WAIT_FLAG_BYTES);
    w.total = off;
    return w;
}

template <class P> P *at(void *ws, size_t off) { return reinterpret_cast<P *>(static_cast<char *>(ws) + off); }

GemvSeg seg(const void *W, float *y, int64_t rows, int64_t ldy, const float *resid = nullptr, int64_t ldr = 0)
{
    return GemvSeg{static_cast<const uint8_t *>(W), y, resid, rows, ldy, ldr};
}

prima_status check_layer(const prima_layer &l, bool with_caches = true)
{
    const void *ptrs[] = {l.wq, l.wk, l.wv, l.wo, l.wgate, l.wup, l.wdown, l.g_attn, l.g_ffn,
                          with_caches ? l.k_cache : l.wq, with_caches ? l.v_cache : l.wq};
    for (const void *p : ptrs) {
        if (!p) return PRIMA_E_NULL;
        if (!aligned(p, 16)) return PRIMA_E_ALIGN;
    }
    return PRIMA_OK;
}

GemvArgs gemv_args(int nseg, int64_t n_cols, const float *x, int64_t ldx, int T, int xmode = X_PLAIN,
                   const float *gain = nullptr, float eps = 0.f, int epi = EPI_ROWS)
{
    GemvArgs ga{};
    ga.nseg = nseg; ga.n_cols = n_cols; ga.x = x; ga.ldx = ldx; ga.T = T;
    ga.xmode = xmode; ga.epi = epi; ga.gain = gain; ga.eps = eps;
    return ga;
}

// the four projections of a layer as mat-vec arguments, in launch order (Q/K/V, output, gate/up, down)
void layer_gemv_args(const prima_dims &d, const prima_layer &L, int T, const float *x, float *y, void *ws, const WindowWs &w, GemvArgs ga[4])
{
    const int64_t e = d.e, qd = static_cast<int64_t>(d.n_q_heads) * d.head_dim, kvd = static_cast<int64_t>(d.n_kv_heads) * d.head_dim, F = d.ffn;
    float *q = at<float>(ws, w.q), *k = at<float>(ws, w.k), *v = at<float>(ws, w.v);
    float *o = at<float>(ws, w.o), *h = at<float>(ws, w.h), *act = at<float>(ws, w.a);
    ga[0] = gemv_args(3, e, x, e, T, X_RMSNORM, L.g_attn, d.rms_eps);
    ga[0].seg[0] = seg(L.wq, q, qd, qd);
    ga[0].seg[1] = seg(L.wk, k, kvd, kvd);
    ga[0].seg[2] = seg(L.wv, v, kvd, kvd);
    ga[1] = gemv_args(1, qd, o, qd, T);
    ga[1].seg[0] = seg(L.wo, h, e, e, x, e);
    ga[2] = gemv_args(2, e, h, e, T, X_RMSNORM, L.g_ffn, d.rms_eps, EPI_SWIGLU);
    ga[2].seg[0] = seg(L.wgate, act, F, F); // silu(gate) * up lands here
    ga[2].seg[1] = seg(L.wup, nullptr, F, F);
    ga[3] = gemv_args(1, F, act, F, T);
    ga[3].seg[0] = seg(L.wdown, y, e, e, h, e);
}

// prompts of up to this many tokens go through the decode kernels, PRIMA_MAX_TOK tokens a call (measured on config 3's shape,
// ms per layer, matrix-product route / decode route: 8 tokens 0.39 / 0.19, 16: 0.38 / 0.37, 24: 0.40 / 0.56, 32: 0.40 / 0.73,
// 64: 0.43 / 1.46, 128: 0.60 / 2.93, 256: 1.04 / 5.87).  A process-wide setting, read when a prompt call is enqueued.
int g_prefill_small_tokens = 16;

// one decoder layer; x -> y (fp32 [T][e]); taps may be null.  Five launches: Q/K/V projections
// (RMSNorm fused), attention (RoPE + KV append fused, key ranges merged by the last arriver), output projection
// (+ residual), gate/up projections (RMSNorm fused in front, SwiGLU behind), down projection (+ residual).
prima_status run_layer(const prima_dims &d, const prima_layer &L, int kv_cap, int n_past, int T,
                       const float *x, float *y, void *ws, const WindowWs &w, hipStream_t st,
                       float *tap_q, float *tap_o, float *tap_h, float *tap_a, int only = -1, const AttnSeqs *seq = nullptr,
                       const prima_layer_formats *fm = nullptr)
{
    // fm: formats of the seven matrices (null: all Q4_K).  Q4_K matrices go through the MFMA mat-vec (those of one
    // group in one launch), the others through the format mat-vec, one launch each, with the same fused RMSNorm /
    // residual; SwiGLU is a launch of its own unless gate and up are both Q4_K.
    const int f_q = fm ? fm->wq : 0, f_k = fm ? fm->wk : 0, f_v = fm ? fm->wv : 0, f_o = fm ? fm->wo : 0;
    const int f_g = fm ? fm->wgate : 0, f_u = fm ? fm->wup : 0, f_d = fm ? fm->wdown : 0;
    auto other = [&](int fmt, const void *W, int64_t rows, int64_t cols, const float *xin, const float *gain,
                     const float *resid, float *out) {
        return launch_fmt_gemv(fmt, static_cast<const uint8_t *>(W), rows, cols, xin, cols, T, gain, d.rms_eps, resid, rows, out, rows, st);
    };
    const int64_t e = d.e, qd = static_cast<int64_t>(d.n_q_heads) * d.head_dim, kvd = static_cast<int64_t>(d.n_kv_heads) * d.head_dim, F = d.ffn;
    float *q = at<float>(ws, w.q), *k = at<float>(ws, w.k), *v = at<float>(ws, w.v);
    float *o = at<float>(ws, w.o), *h = at<float>(ws, w.h), *act = at<float>(ws, w.a);
    prima_status s;
#define PRIMA_TRY(call) do { s = (call); if (s != PRIMA_OK) return s; } while (0)
#define PRIMA_WANT(k) (only < 0 || only == (k))
    if (PRIMA_WANT(PRIMA_K_QKV)) {
        GemvArgs ga = gemv_args(0, e, x, e, T, X_RMSNORM, L.g_attn, d.rms_eps);
        if (f_q == PRIMA_FMT_Q4_K) ga.seg[ga.nseg++] = seg(L.wq, q, qd, qd);
        if (f_k == PRIMA_FMT_Q4_K) ga.seg[ga.nseg++] = seg(L.wk, k, kvd, kvd);
        if (f_v == PRIMA_FMT_Q4_K) ga.seg[ga.nseg++] = seg(L.wv, v, kvd, kvd);
        if (ga.nseg) PRIMA_TRY(launch_gemv_mfma(ga, at<char>(ws, w.gemv), w.gemv_bytes, w.arrivals_bytes, st));
        if (f_q != PRIMA_FMT_Q4_K) PRIMA_TRY(other(f_q, L.wq, qd, e, x, L.g_attn, nullptr, q));
        if (f_k != PRIMA_FMT_Q4_K) PRIMA_TRY(other(f_k, L.wk, kvd, e, x, L.g_attn, nullptr, k));
        if (f_v != PRIMA_FMT_Q4_K) PRIMA_TRY(other(f_v, L.wv, kvd, e, x, L.g_attn, nullptr, v));
    }
    if (PRIMA_WANT(PRIMA_K_ATTN))
        PRIMA_TRY(launch_attn(d, q, tap_q, k, v, at<float>(ws, w.rope), static_cast<__half *>(L.k_cache),
                              static_cast<__half *>(L.v_cache), kv_cap, n_past, T, o, at<char>(ws, w.attn), st, seq));
    if (tap_o && hipMemcpyAsync(tap_o, o, T * qd * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return PRIMA_E_DEVICE;
    if (PRIMA_WANT(PRIMA_K_WO)) {
        if (f_o == PRIMA_FMT_Q4_K) {
            GemvArgs ga = gemv_args(1, qd, o, qd, T);
            ga.seg[0] = seg(L.wo, h, e, e, x, e);
            PRIMA_TRY(launch_gemv_mfma(ga, at<char>(ws, w.gemv), w.gemv_bytes, w.arrivals_bytes, st));
        } else {
            PRIMA_TRY(other(f_o, L.wo, e, qd, o, nullptr, x, h));
        }
    }
    if (tap_h && hipMemcpyAsync(tap_h, h, T * e * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return PRIMA_E_DEVICE;
    if (PRIMA_WANT(PRIMA_K_GATE_UP)) {
        if (f_g == PRIMA_FMT_Q4_K && f_u == PRIMA_FMT_Q4_K) {
            GemvArgs ga = gemv_args(2, e, h, e, T, X_RMSNORM, L.g_ffn, d.rms_eps, EPI_SWIGLU);
            ga.seg[0] = seg(L.wgate, act, F, F); // silu(gate) * up lands here
            ga.seg[1] = seg(L.wup, nullptr, F, F);
            PRIMA_TRY(launch_gemv_mfma(ga, at<char>(ws, w.gemv), w.gemv_bytes, w.arrivals_bytes, st));
        } else {
            float *up = at<float>(ws, w.u);
            const void *Wm[2] = {L.wgate, L.wup};
            float *out[2] = {act, up};
            const int fmt2[2] = {f_g, f_u};
            for (int i = 0; i < 2; ++i) {
                if (fmt2[i] == PRIMA_FMT_Q4_K) {
                    GemvArgs ga = gemv_args(1, e, h, e, T, X_RMSNORM, L.g_ffn, d.rms_eps);
                    ga.seg[0] = seg(Wm[i], out[i], F, F);
                    PRIMA_TRY(launch_gemv_mfma(ga, at<char>(ws, w.gemv), w.gemv_bytes, w.arrivals_bytes, st));
                } else {
                    PRIMA_TRY(other(fmt2[i], Wm[i], F, e, h, L.g_ffn, nullptr, out[i]));
                }
            }
            PRIMA_TRY(launch_swiglu(act, up, static_cast<int64_t>(T) * F, st));
        }
    }
    if (tap_a && hipMemcpyAsync(tap_a, act, T * F * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) return PRIMA_E_DEVICE;
    if (PRIMA_WANT(PRIMA_K_DOWN)) {
        if (f_d == PRIMA_FMT_Q4_K) {
            GemvArgs ga = gemv_args(1, F, act, F, T);
            ga.seg[0] = seg(L.wdown, y, e, e, h, e);
            PRIMA_TRY(launch_gemv_mfma(ga, at<char>(ws, w.gemv), w.gemv_bytes, w.arrivals_bytes, st));
        } else {
            PRIMA_TRY(other(f_d, L.wdown, e, F, act, nullptr, h, y));
        }
    }
#undef PRIMA_WANT
#undef PRIMA_TRY
    return PRIMA_OK;
}

// before the first layer of a step: RoPE table, the counters of the mat-vec and attention scratch zeroed (and, where
// asked, the error flag that prima_window_check reads), the attention's records set to "not written": one launch
prima_status step_init(const prima_dims &d, void *ws, const WindowWs &w, int T, int n_past, const int *positions, bool with_sync, hipStream_t st)
{
    // rows the longest sequence of the step holds after it: sets the attention's key ranges, hence the records it uses
    int n_total = n_past + T;
    if (positions) {
        n_total = 1;
        for (int t = 0; t < T; ++t) n_total = positions[t] + 1 > n_total ? positions[t] + 1 : n_total;
    }
    char *const attn = at<char>(ws, w.attn);
    void *const fp[4] = {at<char>(ws, w.gemv), attn, with_sync ? at<char>(ws, w.sync) : nullptr, attn + attn_counter_bytes(d, T)};
    const size_t fb[4] = {w.arrivals_bytes, attn_counter_bytes(d, T), WAIT_FLAG_BYTES, attn_records_bytes(d, n_total, T, positions != nullptr)};
    const unsigned fw[4] = {0u, 0u, 0u, ATTN_REC_EMPTY};
    return launch_step_init(at<float>(ws, w.rope), T, d.head_dim, n_past, d.rope_theta, positions, fp, fb, fw, st);
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

struct PrefillWs {
    size_t q, k, v, o, h, a, u, xb0, xb1, rope, attn, stat, part, part_bytes, total;
    size_t dec_base; // short prompts: the scratch of a decode call of PRIMA_MAX_TOK tokens, carved from here
    WindowWs dec;
};

// scratch of a prompt-processing call: the layer's intermediate activations for all T tokens, the RoPE table, the
// matrix product's scratch (sized for the widest matrix), and the attention scratch of one 16-token call
PrefillWs carve_prefill(const prima_dims &d, int kv_cap, int T)
{
    PrefillWs w{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off += round_up(bytes, 256); return o; };
    const size_t qd = static_cast<size_t>(d.n_q_heads) * d.head_dim, kvd = static_cast<size_t>(d.n_kv_heads) * d.head_dim;
    const size_t f = sizeof(float), t = static_cast<size_t>(T);
    w.q = take(t * qd * f);
    w.k = take(t * kvd * f);
    w.v = take(t * kvd * f);
    w.o = take(t * qd * f);
    w.h = take(t * static_cast<size_t>(d.e) * f);
    w.a = take(t * static_cast<size_t>(d.ffn) * f);
    w.u = take(t * static_cast<size_t>(d.ffn) * f); // up projection, when gate / up are not both Q4_K
    w.xb0 = take(t * static_cast<size_t>(d.e) * f);
    w.xb1 = take(t * static_cast<size_t>(d.e) * f);
    w.rope = take(t * static_cast<size_t>(d.head_dim) * f);
    w.attn = take(attn_ws_bytes(d, kv_cap, PRIMA_MAX_TOK));
    w.stat = take(gemm_ws_bytes(T, std::max<int64_t>({d.e, static_cast<int64_t>(qd), d.ffn})));
    {
        // the shares of K of the launches that divide it (few rows, few tokens): the largest of the layer's products
        const int64_t r_qkv[3] = {static_cast<int64_t>(qd), static_cast<int64_t>(kvd), static_cast<int64_t>(kvd)}, r_e[1] = {d.e}, r_f[1] = {d.ffn};
        size_t pb = gemm_part_bytes(T, r_qkv, 3, d.e);
        for (int i = 0; i < 3; ++i) pb = std::max(pb, gemm_part_bytes(T, r_qkv + i, 1, d.e)); // one by one when the formats differ
        pb = std::max({pb, gemm_part_bytes(T, r_e, 1, static_cast<int64_t>(qd)), gemm_part_bytes(T, r_e, 1, d.ffn), gemm_part_bytes(T, r_f, 1, d.e),
                       gemm_part_bytes(T, r_f, 1, d.e, true)});
        w.part_bytes = pb;
        w.part = take(pb);
    }
    w.dec = carve(d, kv_cap, PRIMA_MAX_TOK);
    w.dec_base = take(w.dec.total);
    w.total = off;
    return w;
}

// one decoder layer for T prompt tokens: the projections as matrix products over all tokens, attention for pieces of
// PRIMA_MAX_TOK tokens (each sees the rows cached before it and, causally, its own), all pieces in one launch
prima_status run_layer_prefill(const prima_dims &d, const prima_layer &L, int kv_cap, int n_past, int T,
                               const float *x, float *y, void *ws, const PrefillWs &w, hipStream_t st,
                               const prima_layer_formats *fm = nullptr)
{
    // fm: formats of the seven matrices (null: all Q4_K).  Q4_K matrices go through the matrix product; a matrix in
    // another format through the format mat-vec, PRIMA_MAX_TOK tokens a launch (there is no matrix-core kernel for those
    // formats: a model that keeps a few tensors in them pays their weight stream once per 16 tokens)
    const int f_q = fm ? fm->wq : 0, f_k = fm ? fm->wk : 0, f_v = fm ? fm->wv : 0, f_o = fm ? fm->wo : 0;
    const int f_g = fm ? fm->wgate : 0, f_u = fm ? fm->wup : 0, f_d = fm ? fm->wdown : 0;
    const int64_t e = d.e, qd = static_cast<int64_t>(d.n_q_heads) * d.head_dim, kvd = static_cast<int64_t>(d.n_kv_heads) * d.head_dim, F = d.ffn;
    float *q = at<float>(ws, w.q), *k = at<float>(ws, w.k), *v = at<float>(ws, w.v);
    float *o = at<float>(ws, w.o), *h = at<float>(ws, w.h), *act = at<float>(ws, w.a);
    void *stat = at<char>(ws, w.stat), *part = at<char>(ws, w.part);
    auto W = [](const void *p) { return static_cast<const uint8_t *>(p); };
    prima_status s;
#define PRIMA_TRY(call) do { s = (call); if (s != PRIMA_OK) return s; } while (0)
    // one projection: out = W a (+ resid), a = xin or RMSNorm(xin; gain); split_ready as for the matrix product
    auto product = [&](int fmt, const void *Wm, int64_t rows, int64_t cols, const float *xin, const float *gain, const float *resid,
                       float *out, bool split_ready) -> prima_status {
        if (fmt == PRIMA_FMT_Q4_K)
            return launch_q4k_gemm(W(Wm), rows, cols, xin, cols, T, gain, d.rms_eps, resid, rows, out, rows, stat, st, split_ready, part,
                                   w.part_bytes);
        for (int t0 = 0; t0 < T; t0 += PRIMA_MAX_TOK) {
            const int Tc = std::min<int>(PRIMA_MAX_TOK, T - t0);
            const prima_status ps = launch_fmt_gemv(fmt, W(Wm), rows, cols, xin + t0 * cols, cols, Tc, gain, d.rms_eps,
                                                    resid ? resid + t0 * rows : nullptr, rows, out + t0 * rows, rows, st);
            if (ps != PRIMA_OK) return ps;
        }
        return PRIMA_OK;
    };
    const float *g_attn = static_cast<const float *>(L.g_attn), *g_ffn = static_cast<const float *>(L.g_ffn);
    if (f_q == PRIMA_FMT_Q4_K && f_k == PRIMA_FMT_Q4_K && f_v == PRIMA_FMT_Q4_K) {
        const GemmMat qkv[3] = {{W(L.wq), q, qd, qd}, {W(L.wk), k, kvd, kvd}, {W(L.wv), v, kvd, kvd}};
        PRIMA_TRY(launch_q4k_gemm_multi(qkv, 3, false, e, x, e, T, g_attn, d.rms_eps, nullptr, 0, stat, st, false, part, w.part_bytes));
    } else {
        bool ready = false; // the first Q4_K matrix of the group splits the activations for the others
        PRIMA_TRY(product(f_q, L.wq, qd, e, x, g_attn, nullptr, q, ready));
        ready = ready || f_q == PRIMA_FMT_Q4_K;
        PRIMA_TRY(product(f_k, L.wk, kvd, e, x, g_attn, nullptr, k, ready));
        ready = ready || f_k == PRIMA_FMT_Q4_K;
        PRIMA_TRY(product(f_v, L.wv, kvd, e, x, g_attn, nullptr, v, ready));
    }
    // RoPE and the cache rows of all T tokens first; then the full pieces of PRIMA_MAX_TOK tokens in one launch and the
    // rest in a launch of the decode kind (caches complete, queries rotated)
    __half *Kc = static_cast<__half *>(L.k_cache), *Vc = static_cast<__half *>(L.v_cache);
    PRIMA_TRY(launch_rope_append(d, q, k, v, at<float>(ws, w.rope), Kc, Vc, kv_cap, n_past, T, st));
    const int n_pieces = T / PRIMA_MAX_TOK, rest = T - n_pieces * PRIMA_MAX_TOK;
    PRIMA_TRY(launch_attn_prompt(d, q, Kc, Vc, kv_cap, n_past, n_pieces, o, st));
    if (rest)
        PRIMA_TRY(launch_attn(d, q + n_pieces * PRIMA_MAX_TOK * qd, nullptr, nullptr, nullptr, nullptr, Kc, Vc, kv_cap,
                              n_past + n_pieces * PRIMA_MAX_TOK, rest, o + n_pieces * PRIMA_MAX_TOK * qd, at<char>(ws, w.attn), st));
    PRIMA_TRY(product(f_o, L.wo, e, qd, o, nullptr, x, h, false));
    if (f_g == PRIMA_FMT_Q4_K && f_u == PRIMA_FMT_Q4_K) {
        const GemmMat gate_up[2] = {{W(L.wgate), act, F, F}, {W(L.wup), nullptr, F, F}};
        PRIMA_TRY(launch_q4k_gemm_multi(gate_up, 2, true, e, h, e, T, g_ffn, d.rms_eps, nullptr, 0, stat, st, false, part, w.part_bytes));
    } else {
        float *up = at<float>(ws, w.u);
        PRIMA_TRY(product(f_g, L.wgate, F, e, h, g_ffn, nullptr, act, false));
        PRIMA_TRY(product(f_u, L.wup, F, e, h, g_ffn, nullptr, up, f_g == PRIMA_FMT_Q4_K));
        PRIMA_TRY(launch_swiglu(act, up, static_cast<int64_t>(T) * F, st));
    }
    PRIMA_TRY(product(f_d, L.wdown, e, F, act, nullptr, h, y, false));
#undef PRIMA_TRY
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
    if (n_rows < 0 || n_cols < 0 || n_cols % QK) return PRIMA_E_SHAPE;
    if (n_rows == 0 || n_cols == 0) return PRIMA_OK; // nothing to do; pointers may be null
    if (!W || !out) return PRIMA_E_NULL;
    if (!aligned(W, 16) || !aligned(out, 16)) return PRIMA_E_ALIGN;
    return launch_dequant(static_cast<const uint8_t *>(W), n_rows, n_cols, out, static_cast<hipStream_t>(hip_stream));
}

prima_status prima_stream_read_probe(const void *src, size_t bytes, void *sink, void *hip_stream)
{
    if (!src || !sink) return PRIMA_E_NULL;
    if (!aligned(src, 16) || !aligned(sink, 4)) return PRIMA_E_ALIGN;
    if (bytes < 16) return PRIMA_OK;
    return launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream), false);
}

prima_status prima_stream_read_probe_nt(const void *src, size_t bytes, void *sink, void *hip_stream)
{
    if (!src || !sink) return PRIMA_E_NULL;
    if (!aligned(src, 16) || !aligned(sink, 4)) return PRIMA_E_ALIGN;
    if (bytes < 16) return PRIMA_OK;
    return launch_stream_read(src, bytes, sink, static_cast<hipStream_t>(hip_stream), true);
}

size_t prima_gemv_workspace_bytes(int64_t n_rows, int64_t n_cols, int32_t T)
{
    if (n_rows < 0 || n_cols < 0 || T < 1) return 0;
    const size_t b = gemv_ws_bytes(n_rows, n_cols, T);
    return b < 256 ? 256 : b;
}

prima_status prima_q4k_gemv(const void *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int32_t T,
                            float *y, int64_t ldy, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!W || !x || !y || !workspace) return PRIMA_E_NULL;
    if (n_rows < 0 || n_cols <= 0 || n_cols % QK || ldx < n_cols || ldy < n_rows) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK) return PRIMA_E_RANGE;
    if (!aligned(W, 16) || !aligned(x, 16) || !aligned(y, 4) || ldx % 4 || !aligned(workspace, 256)) return PRIMA_E_ALIGN;
    if (workspace_bytes < std::max<size_t>(256, gemv_ws_bytes(n_rows, n_cols, T))) return PRIMA_E_WORKSPACE;
    if (n_rows == 0) return PRIMA_OK;
    GemvArgs ga = gemv_args(1, n_cols, x, ldx, T);
    ga.seg[0] = seg(W, y, n_rows, ldy);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    prima_status s = launch_zero_arrivals(workspace, gemv_arrivals_bytes(n_rows), st);
    if (s != PRIMA_OK) return s;
    return launch_gemv_mfma(ga, workspace, workspace_bytes, gemv_arrivals_bytes(n_rows), st);
}

} // extern "C"

// Scratch of prima_q4k_gemv_noalloc: part of the device image, one copy per GPU.  In host code the array's name is
// only a handle for hipGetSymbolAddress; kernels and fills get the device address looked up below.
static __device__ __align__(256) unsigned char scratch[PRIMA_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[NOALLOC_MAX_DEVICES]; // device address of `scratch` on each GPU, null until looked up

// the current device's copy of the array (looked up once per device, with that device current)
prima_status noalloc_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES) return PRIMA_E_DEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return PRIMA_E_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PRIMA_OK;
}
} // namespace

extern "C" {

prima_status prima_q4k_gemv_noalloc(const void *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int32_t T,
                                    float *y, int64_t ldy, void *hip_stream)
{
    if (!W || !x || !y) return PRIMA_E_NULL;
    if (n_rows < 0 || n_cols <= 0 || n_cols % QK || ldx < n_cols || ldy < n_rows) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK) return PRIMA_E_RANGE;
    if (!aligned(W, 16) || !aligned(x, 16) || !aligned(y, 4) || ldx % 4) return PRIMA_E_ALIGN;
    const size_t need = std::max<size_t>(256, gemv_ws_bytes(n_rows, n_cols, T));
    if (need > PRIMA_NOALLOC_SCRATCH_BYTES) return PRIMA_E_WORKSPACE; // beyond the fixed array: use prima_q4k_gemv
    if (n_rows == 0) return PRIMA_OK;
    void *ws = nullptr;
    prima_status s = noalloc_scratch(&ws);
    if (s != PRIMA_OK) return s;
    GemvArgs ga = gemv_args(1, n_cols, x, ldx, T);
    ga.seg[0] = seg(W, y, n_rows, ldy);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    // the array keeps what the last call left: the counters are cleared by a fill kernel (not a memset node)
    s = launch_zero_arrivals(ws, gemv_arrivals_bytes(n_rows), st);
    if (s != PRIMA_OK) return s;
    return launch_gemv_mfma(ga, ws, PRIMA_NOALLOC_SCRATCH_BYTES, gemv_arrivals_bytes(n_rows), st);
}

size_t prima_gemm_workspace_bytes(int32_t T, int64_t n_cols) { return (T < 1 || n_cols <= 0 || n_cols % QK) ? 0 : gemm_ws_bytes(T, n_cols); }

int32_t prima_gemm_ksplit(int32_t T, int64_t n_rows, int64_t n_cols)
{
    return (T < 1 || n_rows < 0 || n_cols <= 0 || n_cols % QK) ? 0 : gemm_ksplit(T, &n_rows, 1, n_cols);
}

size_t prima_gemm_workspace_bytes_ksplit(int32_t T, int64_t n_rows, int64_t n_cols)
{
    if (T < 1 || n_rows < 0 || n_cols <= 0 || n_cols % QK) return 0;
    return round_up(gemm_ws_bytes(T, n_cols), 256) + gemm_part_bytes(T, &n_rows, 1, n_cols);
}

prima_status prima_q4k_gemm(const void *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int32_t T,
                            const float *gain, float eps, const float *resid, int64_t ldr, float *y, int64_t ldy,
                            void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!W || !x || !y || !workspace) return PRIMA_E_NULL;
    if (n_rows < 0 || n_cols <= 0 || n_cols % QK || ldx < n_cols || ldy < n_rows || (resid && ldr < n_rows)) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_GEMM_MAX_TOK) return PRIMA_E_RANGE;
    if (!aligned(W, 16) || !aligned(x, 16) || !aligned(y, 4) || ldx % 4 || (gain && !aligned(gain, 16)) || (resid && !aligned(resid, 4)) ||
        !aligned(workspace, 256))
        return PRIMA_E_ALIGN;
    if (workspace_bytes < gemm_ws_bytes(T, n_cols)) return PRIMA_E_WORKSPACE;
    // what lies behind the minimum holds the shares of K, if it holds them all
    const size_t part_off = round_up(gemm_ws_bytes(T, n_cols), 256);
    void *part = workspace_bytes > part_off ? static_cast<char *>(workspace) + part_off : nullptr;
    return launch_q4k_gemm(static_cast<const uint8_t *>(W), n_rows, n_cols, x, ldx, T, gain, eps, resid, ldr, y, ldy, workspace,
                           static_cast<hipStream_t>(hip_stream), false, part, part ? workspace_bytes - part_off : 0);
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
    // the give-up flag cleared, the records this launch uses marked "not written"
    const prima_status s = launch_fill_words(workspace, attn_counter_bytes(*d, T), 0u, static_cast<char *>(workspace) + attn_counter_bytes(*d, T),
                                             attn_records_bytes(*d, n_past + T, T, false), ATTN_REC_EMPTY, static_cast<hipStream_t>(hip_stream));
    if (s != PRIMA_OK) return s;
    return launch_attn(*d, q, nullptr, nullptr, nullptr, nullptr,
                       static_cast<__half *>(const_cast<void *>(k_cache)), static_cast<__half *>(const_cast<void *>(v_cache)),
                       kv_cap, n_past, T, o, workspace, static_cast<hipStream_t>(hip_stream));
}

size_t prima_fmt_tensor_bytes(int32_t fmt, int64_t n_rows, int64_t n_cols) { return fmt_tensor_bytes(fmt, n_rows, n_cols); }

prima_status prima_fmt_dequant(int32_t fmt, const void *W, int64_t n_rows, int64_t n_cols, float *out, void *hip_stream)
{
    if (fmt == PRIMA_FMT_Q4_K) return prima_q4k_dequant(W, n_rows, n_cols, out, hip_stream);
    if (fmt < PRIMA_FMT_Q4_K || fmt > PRIMA_FMT_F32 || n_rows < 0 || n_cols < 0 || n_cols % QK) return PRIMA_E_SHAPE;
    if (n_rows == 0 || n_cols == 0) return PRIMA_OK;
    if (!W || !out) return PRIMA_E_NULL;
    if (!aligned(W, 16) || !aligned(out, 16)) return PRIMA_E_ALIGN;
    return launch_fmt_dequant(fmt, static_cast<const uint8_t *>(W), n_rows, n_cols, out, static_cast<hipStream_t>(hip_stream));
}

prima_status prima_fmt_gemv(int32_t fmt, const void *W, int64_t n_rows, int64_t n_cols,
                            const float *x, int64_t ldx, int32_t T, float *y, int64_t ldy, void *hip_stream)
{
    if (!W || !x || !y) return PRIMA_E_NULL;
    if (fmt <= PRIMA_FMT_Q4_K || fmt > PRIMA_FMT_F32) return PRIMA_E_SHAPE;
    if (n_rows < 0 || n_cols <= 0 || n_cols % QK || ldx < n_cols || ldy < n_rows) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK) return PRIMA_E_RANGE;
    if (!aligned(W, 16) || !aligned(x, 16) || !aligned(y, 4) || ldx % 4) return PRIMA_E_ALIGN;
    return launch_fmt_gemv(fmt, static_cast<const uint8_t *>(W), n_rows, n_cols, x, ldx, T, nullptr, 0.f, nullptr, 0, y, ldy,
                           static_cast<hipStream_t>(hip_stream));
}

prima_status prima_lm_head_fmt(const prima_dims *d, int32_t fmt, const float *g_final, const void *w_lm, int64_t vocab,
                               const float *x, int32_t T, float *logits, void *hip_stream)
{
    if (!d || !g_final || !w_lm || !x || !logits) return PRIMA_E_NULL;
    if (!dims_ok(d) || vocab < 1 || fmt <= PRIMA_FMT_Q4_K || fmt > PRIMA_FMT_F32) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK) return PRIMA_E_RANGE;
    if (!aligned(w_lm, 16) || !aligned(x, 16) || !aligned(g_final, 16) || !aligned(logits, 4)) return PRIMA_E_ALIGN;
    return launch_fmt_gemv(fmt, static_cast<const uint8_t *>(w_lm), vocab, d->e, x, d->e, T, g_final, d->rms_eps, nullptr, 0,
                           logits, vocab, static_cast<hipStream_t>(hip_stream));
}

prima_status prima_gemv_plan_status(int64_t n_rows, int64_t n_cols, int32_t T)
{
    if (n_rows < 0 || n_cols <= 0 || n_cols % QK) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK) return PRIMA_E_RANGE;
    if (n_rows == 0) return PRIMA_OK;
    static float dummy[4]; // addresses only: nothing is read or written
    GemvArgs ga = gemv_args(1, n_cols, dummy, n_cols, T);
    ga.seg[0] = seg(dummy, dummy, n_rows, n_rows);
    return gemv_plan_status(ga, dummy, std::max<size_t>(256, gemv_ws_bytes(n_rows, n_cols, T)), gemv_arrivals_bytes(n_rows));
}

prima_status prima_window_plan_status(const prima_dims *d, int32_t kv_cap, int32_t T)
{
    if (!d) return PRIMA_E_NULL;
    if (!dims_ok(d)) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK || kv_cap < T) return PRIMA_E_RANGE;
    const WindowWs w = carve(*d, kv_cap, T);
    const int64_t e = d->e, qd = static_cast<int64_t>(d->n_q_heads) * d->head_dim, kvd = static_cast<int64_t>(d->n_kv_heads) * d->head_dim, F = d->ffn;
    static float dummy[4];                       // addresses only: nothing is read or written
    char *const ws = reinterpret_cast<char *>(dummy);
    struct Launch { int nseg; int64_t rows[3]; int64_t cols; int xmode, epi; };
    // the launches of a layer, and those of its groups when some of their matrices are in other formats
    const Launch launches[] = {{3, {qd, kvd, kvd}, e, X_RMSNORM, EPI_ROWS}, {2, {qd, kvd, 0}, e, X_RMSNORM, EPI_ROWS},
                               {2, {kvd, kvd, 0}, e, X_RMSNORM, EPI_ROWS}, {1, {qd, 0, 0}, e, X_RMSNORM, EPI_ROWS},
                               {1, {kvd, 0, 0}, e, X_RMSNORM, EPI_ROWS}, {1, {e, 0, 0}, qd, X_PLAIN, EPI_ROWS},
                               {2, {F, F, 0}, e, X_RMSNORM, EPI_SWIGLU}, {1, {F, 0, 0}, e, X_RMSNORM, EPI_ROWS},
                               {1, {e, 0, 0}, F, X_PLAIN, EPI_ROWS}};
    for (const Launch &l : launches) {
        GemvArgs ga = gemv_args(l.nseg, l.cols, dummy, l.cols, T, l.xmode, dummy, d->rms_eps, l.epi);
        for (int i = 0; i < l.nseg; ++i) ga.seg[i] = seg(ws, dummy, l.rows[i], l.rows[i]);
        const prima_status s = gemv_plan_status(ga, ws, w.gemv_bytes, w.arrivals_bytes);
        if (s != PRIMA_OK) return s;
    }
    return PRIMA_OK;
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
    s = step_init(*d, workspace, w, T, n_past, nullptr, true, st);
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

prima_status prima_layer_window_decode_mixed(const prima_dims *d, const prima_layer *layers, const prima_layer_formats *formats,
                                             int32_t L, int32_t kv_cap, int32_t n_past, int32_t T,
                                             const float *x_in, float *x_out,
                                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!layers || !formats) return PRIMA_E_NULL;
    prima_status s = check_window_args(d, kv_cap, n_past, T, x_in, x_out, workspace, workspace_bytes);
    if (s != PRIMA_OK) return s;
    if (L < 1) return PRIMA_E_RANGE;
    for (int i = 0; i < L; ++i) {
        if ((s = check_layer(layers[i])) != PRIMA_OK) return s;
        const int32_t f[7] = {formats[i].wq, formats[i].wk, formats[i].wv, formats[i].wo, formats[i].wgate, formats[i].wup, formats[i].wdown};
        for (int32_t v : f)
            if (v < PRIMA_FMT_Q4_K || v > PRIMA_FMT_F32) return PRIMA_E_SHAPE;
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const WindowWs w = carve(*d, kv_cap, T);
    s = step_init(*d, workspace, w, T, n_past, nullptr, true, st);
    if (s != PRIMA_OK) return s;
    const float *cur = x_in;
    for (int i = 0; i < L; ++i) {
        float *dst = (i == L - 1) ? x_out : at<float>(workspace, (i & 1) ? w.xb1 : w.xb0);
        s = run_layer(*d, layers[i], kv_cap, n_past, T, cur, dst, workspace, w, st, nullptr, nullptr, nullptr, nullptr, -1, nullptr, &formats[i]);
        if (s != PRIMA_OK) return s;
        cur = dst;
    }
    return PRIMA_OK;
}

prima_status prima_layer_window_decode_batch(const prima_dims *d, const prima_layer *layers, int32_t L,
                                             int32_t kv_cap, int32_t B, const int32_t *n_past,
                                             void *const *k_caches, void *const *v_caches,
                                             const float *x_in, float *x_out,
                                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return prima_layer_window_decode_batch_mixed(d, layers, nullptr, L, kv_cap, B, n_past, k_caches, v_caches, x_in, x_out,
                                                 workspace, workspace_bytes, hip_stream);
}

prima_status prima_layer_window_decode_batch_mixed(const prima_dims *d, const prima_layer *layers, const prima_layer_formats *formats,
                                                   int32_t L, int32_t kv_cap, int32_t B, const int32_t *n_past,
                                                   void *const *k_caches, void *const *v_caches,
                                                   const float *x_in, float *x_out,
                                                   void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!layers || !n_past || !k_caches || !v_caches) return PRIMA_E_NULL;
    prima_status s = check_window_args(d, kv_cap, 0, B, x_in, x_out, workspace, workspace_bytes);
    if (s != PRIMA_OK) return s;
    if (L < 1) return PRIMA_E_RANGE;
    for (int b = 0; b < B; ++b)
        if (n_past[b] < 0 || static_cast<int64_t>(n_past[b]) + 1 > kv_cap) return PRIMA_E_RANGE;
    for (int i = 0; i < L; ++i) {
        if ((s = check_layer(layers[i], false)) != PRIMA_OK) return s;
        if (formats) {
            const int32_t f[7] = {formats[i].wq, formats[i].wk, formats[i].wv, formats[i].wo, formats[i].wgate, formats[i].wup, formats[i].wdown};
            for (int32_t v : f)
                if (v < PRIMA_FMT_Q4_K || v > PRIMA_FMT_F32) return PRIMA_E_SHAPE;
        }
        for (int b = 0; b < B; ++b) {
            const void *kc = k_caches[static_cast<size_t>(i) * B + b], *vc = v_caches[static_cast<size_t>(i) * B + b];
            if (!kc || !vc) return PRIMA_E_NULL;
            if (!aligned(kc, 16) || !aligned(vc, 16)) return PRIMA_E_ALIGN;
        }
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const WindowWs w = carve(*d, kv_cap, B);
    s = step_init(*d, workspace, w, B, 0, n_past, false, st);
    if (s != PRIMA_OK) return s;
    const float *cur = x_in;
    for (int i = 0; i < L; ++i) {
        float *dst = (i == L - 1) ? x_out : at<float>(workspace, (i & 1) ? w.xb1 : w.xb0);
        __half *kc[PRIMA_MAX_TOK], *vc[PRIMA_MAX_TOK];
        for (int b = 0; b < B; ++b) {
            kc[b] = static_cast<__half *>(k_caches[static_cast<size_t>(i) * B + b]);
            vc[b] = static_cast<__half *>(v_caches[static_cast<size_t>(i) * B + b]);
        }
        const AttnSeqs seq{n_past, kc, vc};
        s = run_layer(*d, layers[i], kv_cap, 0, B, cur, dst, workspace, w, st, nullptr, nullptr, nullptr, nullptr, -1, &seq,
                      formats ? &formats[i] : nullptr);
        if (s != PRIMA_OK) return s;
        cur = dst;
    }
    return PRIMA_OK;
}

void prima_set_prefill_small_tokens(int32_t n) { g_prefill_small_tokens = n < 0 ? 0 : n; }

size_t prima_prefill_workspace_bytes(const prima_dims *d, int32_t kv_cap, int32_t T)
{
    if (!d || !dims_ok(d) || T < 1 || T > PRIMA_PREFILL_MAX_TOK || kv_cap < 1) return 0;
    return carve_prefill(*d, kv_cap, T).total;
}

prima_status prima_layer_window_prefill(const prima_dims *d, const prima_layer *layers, int32_t L,
                                        int32_t kv_cap, int32_t n_past, int32_t T,
                                        const float *x_in, float *x_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return prima_layer_window_prefill_mixed(d, layers, nullptr, L, kv_cap, n_past, T, x_in, x_out, workspace, workspace_bytes, hip_stream);
}

prima_status prima_layer_window_prefill_mixed(const prima_dims *d, const prima_layer *layers, const prima_layer_formats *formats, int32_t L,
                                              int32_t kv_cap, int32_t n_past, int32_t T,
                                              const float *x_in, float *x_out, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d || !x_in || !x_out || !workspace || !layers) return PRIMA_E_NULL;
    if (!dims_ok(d)) return PRIMA_E_SHAPE;
    if (L < 1 || T < 1 || T > PRIMA_PREFILL_MAX_TOK || n_past < 0 || kv_cap < 1 || static_cast<int64_t>(n_past) + T > kv_cap) return PRIMA_E_RANGE;
    if (!aligned(x_in, 16) || !aligned(x_out, 16) || !aligned(workspace, 256)) return PRIMA_E_ALIGN;
    const PrefillWs w = carve_prefill(*d, kv_cap, T);
    if (workspace_bytes < w.total) return PRIMA_E_WORKSPACE;
    for (int i = 0; i < L; ++i) {
        const prima_status c = check_layer(layers[i]);
        if (c != PRIMA_OK) return c;
        if (formats) {
            const int32_t f[7] = {formats[i].wq, formats[i].wk, formats[i].wv, formats[i].wo, formats[i].wgate, formats[i].wup, formats[i].wdown};
            for (int32_t v : f)
                if (v < PRIMA_FMT_Q4_K || v > PRIMA_FMT_F32) return PRIMA_E_SHAPE;
        }
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (T <= g_prefill_small_tokens) {
        // a short prompt: a matrix-product workgroup does the work of 64 tokens whatever their number; up to one decode call's
        // worth of tokens the decode kernels are faster
        void *dws = at<char>(workspace, w.dec_base);
        for (int t0 = 0; t0 < T; t0 += PRIMA_MAX_TOK) {
            const int Tc = std::min<int>(PRIMA_MAX_TOK, T - t0);
            prima_status cs = step_init(*d, dws, w.dec, Tc, n_past + t0, nullptr, false, st);
            if (cs != PRIMA_OK) return cs;
            const float *cur = x_in + static_cast<int64_t>(t0) * d->e;
            for (int i = 0; i < L; ++i) {
                float *dst = (i == L - 1) ? x_out + static_cast<int64_t>(t0) * d->e : at<float>(dws, (i & 1) ? w.dec.xb1 : w.dec.xb0);
                cs = run_layer(*d, layers[i], kv_cap, n_past + t0, Tc, cur, dst, dws, w.dec, st, nullptr, nullptr, nullptr, nullptr, -1, nullptr,
                               formats ? &formats[i] : nullptr);
                if (cs != PRIMA_OK) return cs;
                cur = dst;
            }
        }
        return PRIMA_OK;
    }
    prima_status s = launch_rope_table(at<float>(workspace, w.rope), T, d->head_dim, n_past, d->rope_theta, st);
    if (s != PRIMA_OK) return s;
    {   // the attention launch for the last T mod 16 tokens (the only one with key ranges to merge): its records marked "not written"
        const int rest = T % PRIMA_MAX_TOK;
        char *const attn = at<char>(workspace, w.attn);
        const size_t head_bytes = attn_counter_bytes(*d, rest ? rest : 1); // the records of that launch start behind it
        s = launch_fill_words(attn, head_bytes, 0u, attn + head_bytes, rest ? attn_records_bytes(*d, n_past + T, rest, false) : 0, ATTN_REC_EMPTY, st);
        if (s != PRIMA_OK) return s;
    }
    const float *cur = x_in;
    for (int i = 0; i < L; ++i) {
        float *dst = (i == L - 1) ? x_out : at<float>(workspace, (i & 1) ? w.xb1 : w.xb0);
        s = run_layer_prefill(*d, layers[i], kv_cap, n_past, T, cur, dst, workspace, w, st, formats ? &formats[i] : nullptr);
        if (s != PRIMA_OK) return s;
        cur = dst;
    }
    return PRIMA_OK;
}

prima_status prima_window_check(const prima_dims *d, int32_t kv_cap, int32_t T, const void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d || !workspace) return PRIMA_E_NULL;
    if (!dims_ok(d) || T < 1 || T > PRIMA_MAX_TOK || kv_cap < 1) return PRIMA_E_SHAPE;
    const WindowWs w = carve(*d, kv_cap, T);
    if (workspace_bytes < w.total) return PRIMA_E_WORKSPACE;
    if (hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)) != hipSuccess) return PRIMA_E_DEVICE;
    int flag = 0, attn_flag = 0; // the flags of the mat-vec's and the attention's bounded waits
    if (hipMemcpy(&flag, static_cast<const char *>(workspace) + w.sync, sizeof(flag), hipMemcpyDeviceToHost) != hipSuccess) return PRIMA_E_DEVICE;
    if (hipMemcpy(&attn_flag, static_cast<const char *>(workspace) + w.attn, sizeof(attn_flag), hipMemcpyDeviceToHost) != hipSuccess) return PRIMA_E_DEVICE;
    return (flag | attn_flag) == 0 ? PRIMA_OK : PRIMA_E_DEVICE;
}

prima_status prima_layer_window_decode_profiled(const prima_dims *d, const prima_layer *layers, int32_t L,
                                                int32_t kv_cap, int32_t n_past, int32_t T,
                                                const float *x_in, float *x_out,
                                                void *workspace, size_t workspace_bytes, void *hip_stream,
                                                float *ms_by_kind, int32_t *launches_by_kind)
{
    if (!layers || !ms_by_kind || !launches_by_kind) return PRIMA_E_NULL;
    prima_status s = check_window_args(d, kv_cap, n_past, T, x_in, x_out, workspace, workspace_bytes);
    if (s != PRIMA_OK) return s;
    if (L < 1) return PRIMA_E_RANGE;
    for (int i = 0; i < L; ++i)
        if ((s = check_layer(layers[i])) != PRIMA_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const WindowWs w = carve(*d, kv_cap, T);
    // one ordinary step first: every intermediate buffer then holds this step's values
    auto ordinary_step = [&]() {
        prima_status os = step_init(*d, workspace, w, T, n_past, nullptr, false, st);
        const float *cur = x_in;
        for (int i = 0; i < L && os == PRIMA_OK; ++i) {
            float *dst = (i == L - 1) ? x_out : at<float>(workspace, (i & 1) ? w.xb1 : w.xb0);
            os = run_layer(*d, layers[i], kv_cap, n_past, T, cur, dst, workspace, w, st, nullptr, nullptr, nullptr, nullptr);
            cur = dst;
        }
        return os;
    };
    s = ordinary_step();
    // then each kind of launch on its own, once per layer (L different weight sets, so nothing is
    // served from a cache that the real step would not have), between two events
    hipEvent_t ev[PRIMA_N_KINDS + 1];
    int n_ev = 0;
    const int kinds[] = {PRIMA_K_QKV, PRIMA_K_ATTN, PRIMA_K_WO, PRIMA_K_GATE_UP, PRIMA_K_DOWN};
    const int n_kinds = static_cast<int>(sizeof(kinds) / sizeof(kinds[0]));
    for (int k = 0; k < PRIMA_N_KINDS; ++k) { ms_by_kind[k] = 0.f; launches_by_kind[k] = 0; }
    auto mark = [&]() {
        if (hipEventCreate(&ev[n_ev]) != hipSuccess) return false;
        ++n_ev;
        return hipEventRecord(ev[n_ev - 1], st) == hipSuccess;
    };
    if (s == PRIMA_OK && !mark()) s = PRIMA_E_DEVICE;
    float *scratch_out = at<float>(workspace, w.xb0); // the isolated down projections write here, not to x_out
    for (int ki = 0; ki < n_kinds && s == PRIMA_OK; ++ki) {
        for (int i = 0; i < L && s == PRIMA_OK; ++i)
            s = run_layer(*d, layers[i], kv_cap, n_past, T, x_in, scratch_out, workspace, w, st, nullptr, nullptr, nullptr, nullptr, kinds[ki]);
        if (s == PRIMA_OK && !mark()) s = PRIMA_E_DEVICE;
    }
    // The replayed attention launches appended rows n_past .. n_past+T-1 of every layer's caches from whatever the
    // replayed projections left in the scratch (each layer's projections of x_in, not of that layer's own input).
    // The ordinary step once more writes the right rows again (and x_out): the same bits as a plain decode call.
    if (s == PRIMA_OK) s = ordinary_step();
    if (s == PRIMA_OK && hipStreamSynchronize(st) != hipSuccess) s = PRIMA_E_DEVICE;
    for (int ki = 0; ki < n_kinds && s == PRIMA_OK; ++ki) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev[ki], ev[ki + 1]) != hipSuccess) { s = PRIMA_E_DEVICE; break; }
        ms_by_kind[kinds[ki]] = ms;
        launches_by_kind[kinds[ki]] = L;
    }
    for (int i = 0; i < n_ev; ++i) (void)hipEventDestroy(ev[i]);
    return s;
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
    s = step_init(*d, workspace, w, T, n_past, nullptr, false, st);
    if (s != PRIMA_OK) return s;
    return run_layer(*d, *layer, kv_cap, n_past, T, x_in, x_out, workspace, w, st, tap_q, tap_o, tap_h, tap_a);
}

size_t prima_lm_head_workspace_bytes(const prima_dims *d, int64_t vocab, int32_t T)
{
    if (!d || !dims_ok(d) || vocab < 1 || T < 1 || T > PRIMA_MAX_TOK) return 0;
    return std::max<size_t>(256, gemv_ws_bytes(vocab, d->e, T));
}

prima_status prima_lm_head(const prima_dims *d, const float *g_final, const void *w_lm, int64_t vocab,
                           const float *x, int32_t T, float *logits,
                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!d || !g_final || !w_lm || !x || !logits || !workspace) return PRIMA_E_NULL;
    if (!dims_ok(d) || vocab < 1) return PRIMA_E_SHAPE;
    if (T < 1 || T > PRIMA_MAX_TOK) return PRIMA_E_RANGE;
    if (!aligned(g_final, 16) || !aligned(w_lm, 16) || !aligned(x, 16) || !aligned(logits, 4) || !aligned(workspace, 256)) return PRIMA_E_ALIGN;
    if (workspace_bytes < prima_lm_head_workspace_bytes(d, vocab, T)) return PRIMA_E_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    prima_status s = launch_zero_arrivals(workspace, gemv_arrivals_bytes(vocab), st);
    if (s != PRIMA_OK) return s;
    GemvArgs ga = gemv_args(1, d->e, x, d->e, T, X_RMSNORM, g_final, d->rms_eps);
    ga.seg[0] = seg(w_lm, logits, vocab, vocab);
    return launch_gemv_mfma(ga, workspace, workspace_bytes, gemv_arrivals_bytes(vocab), st);
}

} // extern "C"
