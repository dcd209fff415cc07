/*
 * prima.h - C ABI of the MI355X (gfx950) decode hot path of a prima.cpp layer window.
 *
 * A device in the pipelined ring receives e FP32 values per token from its predecessor,
 * advances its window of consecutive decoder layers and forwards e FP32 values
 * (arXiv 2504.08791, Sec. 3.1 and App. A.3 "network communication latency").  Weights stay in
 * Q4_K and are never expanded in memory (App. A.9); the KV cache is fp16 and lives with its
 * layers, one cache per request (App. A.3 "memory access latency", App. A.10); several draft
 * tokens are verified in one batch with unchanged outputs (App. A.12).
 *
 * Conventions for every entry point
 *  - All pointers are DEVICE pointers unless a parameter says "host".  The caller owns every
 *    buffer; the library allocates and frees nothing on these paths, never synchronises the
 *    device and never changes the current device.
 *  - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = default
 *    stream).  Results are ready when that stream has drained.  The window, prompt, mat-vec, matrix-product and
 *    attention calls may be recorded into a HIP graph (stream capture) and replayed: they enqueue kernels only and
 *    clear their scratch with fill kernels; call each once outside the capture first (kernel attributes are set
 *    on a kernel's first launch).  prima_window_check and prima_layer_window_decode_profiled synchronise and may not.
 *  - Arguments are validated on the host before anything is launched; a bad argument returns
 *    a status code and launches nothing.  A fault inside a kernel surfaces at the caller's
 *    next synchronisation; PRIMA_E_DEVICE reports launch-time failures only.
 *  - Q4_K tensors: row-major by output row; a row is n_cols/256 consecutive 144-byte
 *    super-blocks; base pointer 16-byte aligned.  Super-block layout (version 1):
 *      bytes 0-1 d (binary16 LE), 2-3 dmin, 4-15 a 96-bit little-endian bit stream of sixteen
 *      6-bit fields (field i at bits [6i,6i+6): 0-7 sub-scales sc_s, 8-15 sub-mins m_s),
 *      16-143 quants (weight t in byte 16 + t/2, low nibble when t is even);
 *      w[t] = d*sc_s*q[t] - dmin*m_s with s = t/32.
 *  - T (tokens advanced jointly) must satisfy 1 <= T <= PRIMA_MAX_TOK.
 *  - Threads and devices.  One device per process: kernel attributes and the number of compute units are looked
 *    up once, for the device that is current at the first call; calls with another device current may be refused
 *    with PRIMA_E_DEVICE.  Entry points may be called from several host threads as long as no two calls that share
 *    a workspace, a cache or an output are in flight together (the library keeps no state of its own between
 *    calls, apart from the scratch of prima_q4k_gemv_noalloc and one process-wide setting,
 *    prima_set_prefill_small_tokens, which must not change while another thread enqueues a prompt call).
 */
#ifndef PRIMA_H
#define PRIMA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PRIMA_ABI_VERSION 1
#define PRIMA_MAX_TOK 16

typedef enum {
    PRIMA_OK = 0,
    PRIMA_E_NULL = 1,      /* a required pointer is NULL */
    PRIMA_E_SHAPE = 2,     /* a dimension is not supported (e.g. n_cols % 256 != 0) */
    PRIMA_E_ALIGN = 3,     /* a pointer or leading dimension is misaligned */
    PRIMA_E_RANGE = 4,     /* T, n_past or kv_cap out of range */
    PRIMA_E_WORKSPACE = 5, /* workspace too small */
    PRIMA_E_DEVICE = 6     /* a launch failed */
} prima_status;

/* Model dimensions (plain data, passed by pointer to host memory). */
typedef struct {
    int32_t e;          /* hidden size, multiple of 256 */
    int32_t n_q_heads;  /* multiple of n_kv_heads */
    int32_t n_kv_heads;
    int32_t head_dim;   /* 64 or 128 */
    int32_t ffn;        /* multiple of 256 */
    float rope_theta;
    float rms_eps;
    int32_t rope_mode;  /* 0: rotate pairs (i, i + D/2); 1: pairs (2i, 2i + 1) */
} prima_dims;

/* One decoder layer: device pointers.  Read-only except rows [n_past, n_past+T) of the caches. */
typedef struct {
    const void *wq, *wk, *wv, *wo, *wgate, *wup, *wdown; /* Q4_K */
    const float *g_attn, *g_ffn;                         /* fp32 [e] RMSNorm gains */
    void *k_cache, *v_cache;                             /* fp16 [n_kv_heads][kv_cap][head_dim] */
} prima_layer;

/*
 * Dequantised mat-vec (the seven projections of a layer; App. A.3 counts their bytes as b):
 *     y[t*ldy + r] = sum_c W[r][c] * x[t*ldx + c],  r < n_rows, t < T.
 * W: Q4_K, n_rows x n_cols, n_cols % 256 == 0.  x: fp32, ldx >= n_cols, ldx % 4 == 0.  y: fp32,
 * ldy >= n_rows; y must not overlap x.
 * workspace: scratch of at least prima_gemv_workspace_bytes(n_rows, n_cols, T) bytes, 256-byte aligned.
 */
prima_status prima_q4k_gemv(const void *W, int64_t n_rows, int64_t n_cols,
                            const float *x, int64_t ldx, int32_t T,
                            float *y, int64_t ldy,
                            void *workspace, size_t workspace_bytes, void *hip_stream);
size_t prima_gemv_workspace_bytes(int64_t n_rows, int64_t n_cols, int32_t T);

/*
 * prima_q4k_gemv for callers that cannot allocate or pass scratch: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same bits as prima_q4k_gemv, but
 * the scratch (arrival counters and the partial sums of the slabs of K) is a fixed array of
 * PRIMA_NOALLOC_SCRATCH_BYTES in the library's device image instead of a caller buffer; each GPU the library
 * runs on holds its own copy until the process ends.  A shape whose scratch (prima_gemv_workspace_bytes) exceeds
 * that size returns PRIMA_E_WORKSPACE and launches nothing.  The call allocates and frees nothing (the array's
 * device address is looked up once per device, on the first call made with that device current).  Every call on
 * a GPU shares that GPU's array: the counters are cleared by a small fill kernel at the start of each call, and
 * calls that overlap on one GPU (two streams, two threads) race; calls on one stream are safe.
 */
#define PRIMA_NOALLOC_SCRATCH_BYTES (4u << 20)
prima_status prima_q4k_gemv_noalloc(const void *W, int64_t n_rows, int64_t n_cols,
                                    const float *x, int64_t ldx, int32_t T,
                                    float *y, int64_t ldy, void *hip_stream);

/*
 * Measurement hook: reads `bytes` (rounded down to 16) of device memory at `src` once, linearly, with
 * 128-bit loads from about 8 workgroups per compute unit, and discards them; `sink` is 4 bytes of device
 * memory that is (practically never) written.  Timed by the caller it states what a plain read of HBM
 * reaches on this device, the practical ceiling beside the nominal peak (App. A.3's device-loading
 * throughput).  src 16-byte aligned.
 */
prima_status prima_stream_read_probe(const void *src, size_t bytes, void *sink, void *hip_stream);
/*
 * The same read with the non-temporal bit on every load (the lines are marked to leave the caches first), which is how
 * the one-token mat-vec requests its weights: bytes that a launch reads once.  On an MI355X this reaches about 7.1 TB/s
 * where the plain read reaches 6.4.  Same arguments and errors.
 */
prima_status prima_stream_read_probe_nt(const void *src, size_t bytes, void *sink, void *hip_stream);

/*
 * Test hook: out[r*n_cols + c] = fp32 value of weight (r, c).  The value is the fp32 number
 * nearest to the exact d*sc*q - dmin*m (both products are exact in fp32); results are
 * bit-exact by contract.
 */
prima_status prima_q4k_dequant(const void *W, int64_t n_rows, int64_t n_cols, float *out,
                               void *hip_stream);

/*
 * GQA decode attention over an fp16 KV cache (App. A.3: 2(h_k e_k + h_v e_v) n_kv bytes read per
 * layer per step):
 *     o[t][h][:] = sum_{p <= n_past+t} softmax_p( q[t][h] . K[h/G][p] / sqrt(D) ) V[h/G][p],
 *     G = n_q_heads / n_kv_heads.
 * q, o: fp32 [T][n_q_heads][head_dim].  k_cache, v_cache: fp16 [n_kv_heads][kv_cap][head_dim];
 * rows 0 .. n_past+T-1 must be valid (the T new rows already appended).  n_past >= 0,
 * n_past + T <= kv_cap.  workspace >= prima_attn_workspace_bytes(d, kv_cap, T).
 */
prima_status prima_attn_decode(const prima_dims *d, const float *q,
                               const void *k_cache, const void *v_cache,
                               int32_t kv_cap, int32_t n_past, int32_t T, float *o,
                               void *workspace, size_t workspace_bytes, void *hip_stream);
size_t prima_attn_workspace_bytes(const prima_dims *d, int32_t kv_cap, int32_t T);

/*
 * Advance a window of L consecutive decoder layers by T tokens (Sec. 3.1, Def. 1: the layer
 * window; App. A.12: T > 1 is speculative verification with a causal mask among the T tokens).
 * Per layer: RMSNorm, Q/K/V projections, RoPE at positions n_past+t, append fp16 K/V rows
 * n_past..n_past+T-1 (2(h_k e_k + h_v e_v) bytes per token), attention over rows 0..n_past+t,
 * output projection + residual, RMSNorm, SwiGLU feed-forward + residual.
 * layers: HOST array of L descriptors.  x_in, x_out: fp32 [T][e]; x_out may alias x_in.
 * The library keeps no position state: the caller advances n_past (by fewer than T after a
 * rejection; stale rows are overwritten by the next step, never read).
 * workspace >= prima_workspace_bytes(d, kv_cap, T), 256-byte aligned.
 */
prima_status prima_layer_window_decode(const prima_dims *d, const prima_layer *layers, int32_t L,
                                       int32_t kv_cap, int32_t n_past, int32_t T,
                                       const float *x_in, float *x_out,
                                       void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * One step of a batch of B independent sequences through the window: sequence b contributes one token
 * (x_in[b], fp32 [B][e]) that continues its own cached context of n_past[b] rows (continuous batching of
 * requests on a layer window, App. A.12).  The mat-vecs stream the weights once for up to 8 tokens, as for T
 * tokens of one sequence; attention, RoPE (position n_past[b]) and the KV append run per sequence.
 *   n_past    HOST array of B lengths, 0 <= n_past[b] < kv_cap; they may differ.
 *   k_caches  HOST array of L*B DEVICE pointers: entry [l*B + b] is the fp16 K cache [n_kv_heads][kv_cap][head_dim]
 *   v_caches  of layer l for sequence b (same layout as prima_layer.k_cache / v_cache, which this call ignores;
 *             they may be null).  Row n_past[b] of every cache of sequence b is written.
 *   B         1 <= B <= PRIMA_MAX_TOK; workspace as for prima_workspace_bytes(d, kv_cap, B).
 * The pointer arrays and n_past are read before the call returns.  Errors as for prima_layer_window_decode.
 */
prima_status prima_layer_window_decode_batch(const prima_dims *d, const prima_layer *layers, int32_t L,
                                             int32_t kv_cap, int32_t B, const int32_t *n_past,
                                             void *const *k_caches, void *const *v_caches,
                                             const float *x_in, float *x_out,
                                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Some kernels of a window step wait, inside the launch, for records that other workgroups of the same launch write
 * (the workgroup that merges the key ranges of the attention, the one that adds the slabs of a long mat-vec).  These
 * waits are bounded; one that gives up (it never should) raises a flag in the workspace and the step's results are
 * invalid.  prima_window_check() waits for `hip_stream` (it SYNCHRONISES) and returns PRIMA_E_DEVICE if a wait of the
 * last window call on this workspace gave up, else PRIMA_OK.
 */
prima_status prima_window_check(const prima_dims *d, int32_t kv_cap, int32_t T,
                                const void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Measurement hook.  Runs one ordinary window step, then replays each kind of launch on its own,
 * once per layer (L different weight sets), bracketed by two HIP events on `hip_stream`, and
 * returns per kind the elapsed time of its L back-to-back launches.  SYNCHRONISES the stream before
 * returning and creates/destroys events (host-side allocation), so it is not for the serving
 * path.  The replayed launches overwrite the step's new cache rows with other values, so the call
 * ends with a second ordinary step: x_out and rows n_past .. n_past+T-1 of every cache are then
 * bit-equal to what prima_layer_window_decode leaves.  ms_by_kind and launches_by_kind are HOST
 * arrays of PRIMA_N_KINDS entries (milliseconds for all launches of the kind; number of launches).
 */
enum {
    PRIMA_K_QKV = 0,     /* Q/K/V projections with fused RMSNorm */
    PRIMA_K_ROPE_KV = 1, /* unused: RoPE + fp16 KV append run inside the attention kernel */
    PRIMA_K_ATTN = 2,    /* attention: partial (with RoPE + KV append) and merge */
    PRIMA_K_WO = 3,      /* output projection + residual */
    PRIMA_K_GATE_UP = 4, /* gate/up projections with fused RMSNorm */
    PRIMA_K_DOWN = 5,    /* down projection with fused SwiGLU + residual */
    PRIMA_N_KINDS = 6
};
prima_status prima_layer_window_decode_profiled(const prima_dims *d, const prima_layer *layers, int32_t L,
                                                int32_t kv_cap, int32_t n_past, int32_t T,
                                                const float *x_in, float *x_out,
                                                void *workspace, size_t workspace_bytes, void *hip_stream,
                                                float *ms_by_kind, int32_t *launches_by_kind);

/*
 * Test hook: one layer as above, additionally copying intermediates to caller buffers (each may be
 * NULL): tap_q [T][n_q_heads*head_dim] rotated queries, tap_o same shape attention output,
 * tap_h [T][e] hidden state after the attention residual, tap_a [T][ffn] SwiGLU output.
 */
prima_status prima_layer_decode_taps(const prima_dims *d, const prima_layer *layer,
                                     int32_t kv_cap, int32_t n_past, int32_t T,
                                     const float *x_in, float *x_out,
                                     float *tap_q, float *tap_o, float *tap_h, float *tap_a,
                                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Output layer (App. A.3: b_o bytes): logits[t][v] = W_lm . rmsnorm(x[t]; g_final).
 * w_lm: Q4_K [vocab][e].  x: fp32 [T][e].  logits: fp32 [T][vocab].
 * workspace >= prima_lm_head_workspace_bytes(d, vocab, T), 256-byte aligned.
 */
prima_status prima_lm_head(const prima_dims *d, const float *g_final, const void *w_lm, int64_t vocab,
                           const float *x, int32_t T, float *logits,
                           void *workspace, size_t workspace_bytes, void *hip_stream);

size_t prima_lm_head_workspace_bytes(const prima_dims *d, int64_t vocab, int32_t T);

/*
 * The other weight formats of the format set (Sec. 4 / App. A.3, the profiler paragraph: a "Q4K" model
 * keeps some tensors in Q5_K, Q6_K, Q8_0, FP16 or FP32).  The paper names the formats and gives no layout;
 * field sizes and value rules are the formats' own, the placement is this library's (version 1): every
 * field of a tensor is a plane of its own, planes follow one another without padding, blocks inside a
 * plane are in row-major order (row r, block b -> r * n_cols / block + b).  n = n_rows * n_cols / 256.
 * The quant bits of Q5_K and Q6_K are placed word by word: a super-block's bits of one kind are consecutive
 * 32-bit little-endian words, and weight t (0..255 inside its super-block) always sits in byte t%4 of its word
 * (byte j of a word = the byte at offset 4*word + j of the super-block's share of the plane):
 *     low 4 bits  (Q5_K, Q6_K): word t/8  (128 bytes per super-block); the low nibble of byte t%4 when t%8 < 4,
 *                               the high nibble when t%8 >= 4;
 *     bits 4..5   (Q6_K):       word t/16 (64 bytes); bits 2g and 2g+1 of byte t%4, g = (t%16)/4;
 *     bit 4       (Q5_K):       word t/32 (32 bytes); bit g of byte t%4, g = (t%32)/4.
 *   Q5_K  [n][16]: d, dmin (binary16, little endian), then sixteen 6-bit fields sc_0..7, m_0..7 as a
 *         96-bit little-endian stream (bytes 0..15 of a Q4_K super-block) | [n][128]: the low 4 bits |
 *         [n][32]: bit 4.   q = low + 16 * bit4 in 0..31;  w = d sc_s q - dmin m_s, s = t/32.
 *   Q6_K  [n][128]: the low 4 bits | [n][64]: bits 4..5 | [n][16]: signed bytes sc_s, s = t/16 |
 *         [n]: d (binary16, little endian).   q = low + 16 * bits45 in 0..63;  w = d sc_s (q - 32).
 *   Q8_0  [n_rows*n_cols]: one signed byte per weight | [n_rows*n_cols/32]: d (binary16) per 32 weights.
 *         w = d q.
 *   F16, F32: row-major numbers.
 * Every product above is exact in fp32, so a dequantised weight is the fp32 number nearest to the exact
 * value; prima_fmt_dequant is bit-exact by contract.
 */
typedef enum prima_format {
    PRIMA_FMT_Q4_K = 0, /* 144-byte super-blocks (see prima_layer); has entry points of its own */
    PRIMA_FMT_Q5_K = 1,
    PRIMA_FMT_Q6_K = 2,
    PRIMA_FMT_Q8_0 = 3,
    PRIMA_FMT_F16 = 4,
    PRIMA_FMT_F32 = 5
} prima_format;

/* Bytes of an n_rows x n_cols tensor in format fmt (n_cols % 256 == 0); 0 for bad arguments. */
size_t prima_fmt_tensor_bytes(int32_t fmt, int64_t n_rows, int64_t n_cols);

/* Test hook: out[r*n_cols + c] = fp32 value of weight (r, c); any format.  W, out: device, 16-byte aligned. */
prima_status prima_fmt_dequant(int32_t fmt, const void *W, int64_t n_rows, int64_t n_cols, float *out, void *hip_stream);

/*
 * Mat-vec in formats Q5_K .. F32 (PRIMA_FMT_Q4_K: PRIMA_E_SHAPE, use prima_q4k_gemv):
 *     y[t*ldy + r] = sum_c W[r][c] * x[t*ldx + c],  r < n_rows, t < T,  1 <= T <= PRIMA_MAX_TOK.
 * W: device, 16-byte aligned, prima_fmt_tensor_bytes(fmt, n_rows, n_cols) bytes.  x: fp32, 16-byte aligned,
 * ldx >= n_cols, ldx % 4 == 0.  y: fp32, ldy >= n_rows, must not overlap x.  No scratch.  Results do not
 * depend on the launch (fixed order of additions).
 */
prima_status prima_fmt_gemv(int32_t fmt, const void *W, int64_t n_rows, int64_t n_cols,
                            const float *x, int64_t ldx, int32_t T, float *y, int64_t ldy, void *hip_stream);

/* Output layer with w_lm in formats Q5_K .. F32 (commonly Q6_K in a "Q4K" model): as prima_lm_head, no scratch. */
prima_status prima_lm_head_fmt(const prima_dims *d, int32_t fmt, const float *g_final, const void *w_lm, int64_t vocab,
                               const float *x, int32_t T, float *logits, void *hip_stream);

/*
 * Tensors as they lie in a GGUF model file -> this library's layouts, on the device, once at load time.  The paper's
 * checkpoints are "Q4K" GGUF files of Llama and Qwen models (Sec. 4, experimental setup; App. A.3, the format list).
 * Field meanings and values do not change, only the placement of the bits; F16 and F32 are copied.
 * Source block order, as read here (little endian; t = index of a weight in its block; restated from the public
 * description of the formats: no file or specification was at hand, so agreement with real files is untested):
 *   Q4_K 144 B / 256 weights: d | dmin (binary16) | scales[12] | qs[128].
 *        j < 4: sc_j = scales[j] & 63, m_j = scales[j+4] & 63;  j >= 4: sc_j = (scales[j+4] & 15) | (scales[j-4] >> 6) << 4,
 *        m_j = (scales[j+4] >> 4) | (scales[j] >> 6) << 4.  q_t = low (t % 64 < 32) or high nibble of qs[32 (t/64) + t % 32].
 *   Q5_K 176 B: d | dmin | scales[12] | qh[32] | qs[128]; low bits as Q4_K, bit 4 of q_t = bit 2 (t/64) + (t % 64 >= 32) of qh[t % 32].
 *   Q6_K 210 B: ql[128] | qh[64] | scales[16] (signed) | d.  h = t/128, k = (t % 128)/32, l = t % 32: low bits = low (k < 2)
 *        or high nibble of ql[64h + 32 (k & 1) + l]; bits 4..5 = (qh[32h + l] >> 2k) & 3; sub-scale scales[t/16].
 *   Q8_0 34 B / 32 weights: d | qs[32] (signed).
 * Rows one after the other, a row's blocks one after the other.  src: device, prima_gguf_tensor_bytes(fmt, ..) bytes,
 * any alignment.  dst: device, 16-byte aligned, prima_fmt_tensor_bytes(fmt, ..) bytes (the same number), must not
 * overlap src (PRIMA_E_RANGE).  n_cols % 256 == 0.  One launch on hip_stream; no scratch.
 */
size_t prima_gguf_tensor_bytes(int32_t fmt, int64_t n_rows, int64_t n_cols);
prima_status prima_repack_gguf(int32_t fmt, const void *src, int64_t n_rows, int64_t n_cols, void *dst, void *hip_stream);

/*
 * Window forward for a model that keeps some matrices in other formats (the "Q4K" models of Sec. 4 / App. A.3:
 * mostly Q4_K, some tensors Q5_K / Q6_K / Q8_0 / FP16 / FP32).  As prima_layer_window_decode, with formats[i]
 * naming the prima_format of each of layer i's seven matrices (the pointers of prima_layer then point at
 * tensors in those formats).  Same results as if every matrix were dequantised to fp32 and multiplied
 * (within the tolerance of prima_layer_window_decode).  Q4_K matrices run as in prima_layer_window_decode,
 * the others through the mat-vec of prima_fmt_gemv with the same fused RMSNorm and residual.
 * Errors as prima_layer_window_decode; a format code outside prima_format: PRIMA_E_SHAPE.
 */
typedef struct {
    int32_t wq, wk, wv, wo, wgate, wup, wdown; /* prima_format */
} prima_layer_formats;

prima_status prima_layer_window_decode_mixed(const prima_dims *d, const prima_layer *layers, const prima_layer_formats *formats,
                                             int32_t L, int32_t kv_cap, int32_t n_past, int32_t T,
                                             const float *x_in, float *x_out,
                                             void *workspace, size_t workspace_bytes, void *hip_stream);

/* prima_layer_window_decode_batch for layers whose matrices are in several formats (formats as above; NULL: all Q4_K). */
prima_status prima_layer_window_decode_batch_mixed(const prima_dims *d, const prima_layer *layers, const prima_layer_formats *formats,
                                                   int32_t L, int32_t kv_cap, int32_t B, const int32_t *n_past,
                                                   void *const *k_caches, void *const *v_caches,
                                                   const float *x_in, float *x_out,
                                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Host-side check, no GPU work: PRIMA_OK if every mat-vec launch of a window step of T tokens with these
 * dimensions (including the launches used when some matrices are in other formats) finds a launch plan and
 * fits the scratch of prima_workspace_bytes(d, kv_cap, T); otherwise the status such a step would return.
 */
prima_status prima_window_plan_status(const prima_dims *d, int32_t kv_cap, int32_t T);
/*
 * Q4_K matrix product for many tokens (prompt processing; the paper reports the time to the first token next to
 * the time per output token, Sec. 4.1): for t < T, r < n_rows
 *     y[t*ldy + r] = sum_c W[r][c] * a[t][c]  (+ resid[t*ldr + r]),
 *     a[t] = x[t] when gain is null, else RMSNorm(x[t]; gain, eps) (App. A.3's layer, pre-normalised projections).
 * 1 <= T <= PRIMA_GEMM_MAX_TOK.  W: Q4_K layout v1, device, 16-byte aligned.  x: fp32 [T][ldx], 16-byte aligned,
 * ldx >= n_cols, ldx % 4 == 0.  gain: fp32 [n_cols], 16-byte aligned, or null.  resid: fp32 [T][ldr] or null (may be y).
 * y: fp32 [T][ldy], ldy >= n_rows, must not overlap x.  workspace: device, 256-byte aligned, at least
 * prima_gemm_workspace_bytes(T, n_cols) bytes (per-token scales and the activations laid out for the matrix cores,
 * about 4.25 bytes per activation; contents need not be kept).  The activations enter the matrix cores as the sum of
 * two binary16 numbers (22 bits after a per-token power-of-two scale), products and sums are fp32; the same arguments
 * always give the same bits.  All pointers device; asynchronous on hip_stream.
 *
 * Few rows and few tokens (an output projection against a prompt of a hundred tokens) give fewer workgroups than the
 * device has compute units.  With a workspace of prima_gemm_workspace_bytes_ksplit(T, n_rows, n_cols) bytes the call
 * then divides K among prima_gemm_ksplit(T, n_rows, n_cols) workgroups per block of rows and tokens, each leaving its
 * sums behind the first prima_gemm_workspace_bytes(T, n_cols) bytes (rounded up to 256), and a second launch adds them
 * in a fixed order (and the residual).  prima_gemm_ksplit returns 1 where K is not divided (the two sizes are then
 * equal up to that rounding) and 0 for arguments the product would refuse; with less than the larger size the call
 * does not divide K.
 */
#define PRIMA_GEMM_MAX_TOK 65536
prima_status prima_q4k_gemm(const void *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int32_t T,
                            const float *gain, float eps, const float *resid, int64_t ldr, float *y, int64_t ldy,
                            void *workspace, size_t workspace_bytes, void *hip_stream);
size_t prima_gemm_workspace_bytes(int32_t T, int64_t n_cols);
size_t prima_gemm_workspace_bytes_ksplit(int32_t T, int64_t n_rows, int64_t n_cols);
int32_t prima_gemm_ksplit(int32_t T, int64_t n_rows, int64_t n_cols);

/*
 * Prompt processing: all L layers of the window for T consecutive tokens of one sequence that has n_past rows
 * cached (the paper's time to the first token, Sec. 4.1, is this call over the prompt, window by window).  The same
 * arithmetic as prima_layer_window_decode per token, with the projections as matrix products over all tokens
 * (prima_q4k_gemm) and attention in pieces of PRIMA_MAX_TOK tokens, each over the rows cached before it and,
 * causally, its own; the K / V rows of all T tokens are appended to the layers' caches.  Every matrix Q4_K (see
 * prima_layer_window_prefill_mixed for the other formats).
 * 1 <= T <= PRIMA_PREFILL_MAX_TOK, n_past + T <= kv_cap, L >= 1.  x_in, x_out: fp32 [T][e], device, 16-byte
 * aligned (x_out may be x_in).  workspace: device, 256-byte aligned, prima_prefill_workspace_bytes(d, kv_cap, T)
 * bytes, contents need not be kept.  Asynchronous on hip_stream; nothing is allocated.  Errors as for the decode call
 * (PRIMA_E_NULL, _SHAPE, _RANGE, _ALIGN, _WORKSPACE before anything is enqueued; PRIMA_E_DEVICE for a failed launch).
 */
#define PRIMA_PREFILL_MAX_TOK 8192
prima_status prima_layer_window_prefill(const prima_dims *d, const prima_layer *layers, int32_t L,
                                        int32_t kv_cap, int32_t n_past, int32_t T,
                                        const float *x_in, float *x_out,
                                        void *workspace, size_t workspace_bytes, void *hip_stream);
/* The same with every matrix in a format of its own (formats[l], as for prima_layer_window_decode_mixed; null: all
 * Q4_K).  Q4_K matrices go through the matrix product; a matrix in another format is multiplied PRIMA_MAX_TOK tokens a
 * launch by the format mat-vec, so its bytes are read once per 16 prompt tokens.  Same scratch size. */
prima_status prima_layer_window_prefill_mixed(const prima_dims *d, const prima_layer *layers, const prima_layer_formats *formats,
                                              int32_t L, int32_t kv_cap, int32_t n_past, int32_t T,
                                              const float *x_in, float *x_out,
                                              void *workspace, size_t workspace_bytes, void *hip_stream);
size_t prima_prefill_workspace_bytes(const prima_dims *d, int32_t kv_cap, int32_t T);
/* Prompts of up to n tokens are advanced by the decode kernels, PRIMA_MAX_TOK tokens at a time, inside the prompt call
 * (default 16, one decode call: from 17 tokens on the matrix product is faster).  0: always the matrix product (tests).  Process-wide; not to be changed while a call is being enqueued. */
void prima_set_prefill_small_tokens(int32_t n);

/* The same for one prima_q4k_gemv call with the scratch of prima_gemv_workspace_bytes(n_rows, n_cols, T). */
prima_status prima_gemv_plan_status(int64_t n_rows, int64_t n_cols, int32_t T);

/* Bytes of scratch the window calls need for up to T tokens and kv_cap cache rows. */
size_t prima_workspace_bytes(const prima_dims *d, int32_t kv_cap, int32_t T);

const char *prima_status_str(prima_status s);
int prima_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PRIMA_H */
