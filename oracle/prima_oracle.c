/*
 * CPU oracle for the per-token decode forward over a layer window of a
 * Q4_K-quantised Llama/Qwen-style model.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is the plain definition of
 * what the decode path computes, evaluated slowly: scalar Q4_K decoding, every
 * intermediate in fp64, loops in the order of the definition, OpenMP over
 * output rows only.  It shares no code with the HIP library and neither side
 * includes, links or calls the other.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may use it.
 *
 * What the paper fixes (arXiv 2504.08791): weights stay in Q4_K and are never
 * expanded to 16/32-bit in memory (Sec. 4 / App. A.9, memory footprint); the KV
 * cache is fp16 with 2(h_k e_k + h_v e_v) bytes appended per layer per token and
 * 2(h_k e_k + h_v e_v) n_kv bytes read per layer per step (App. A.3, memory
 * access latency); a window receives and returns e FP32 values per token
 * (App. A.3, communication latency); speculative verification evaluates several
 * tokens in one batch without changing outputs (App. A.12).  The paper names the
 * model families (Llama, Qwen) but writes none of the layer formulas; each
 * function below states the standard definition it evaluates.
 *
 * The other weight formats the paper lists (Q5_K, Q6_K, Q8_0, FP16, FP32) are
 * decoded further down; their pins are in tests/test_oracle_formats.py.
 *
 * Pins (tests/test_oracle_*.py): hand-built super-blocks with values known by
 * mental arithmetic, exact rational evaluation of the dequantisation rule,
 * brute-force dense products, library fp64 matmul / softmax, invariants of
 * softmax / RMSNorm / RoPE, joint-equals-sequential for T > 1, KV rewind.
 * Unpinned against any external artefact (free choices with no outside truth
 * here): the byte layout of a super-block, the placement of the fields of the
 * other formats, the RoPE pairing default, bias-free projections.  These are
 * "parity unpinned" with respect to real checkpoints.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define QK 256
#define BLOCK_BYTES 144

typedef struct {
    int32_t e, n_q_heads, n_kv_heads, head_dim, ffn;
    double rope_theta, rms_eps;
    int32_t rope_mode; /* 0: pairs (i, i+D/2); 1: pairs (2i, 2i+1) */
} orc_dims;

/* ---------- IEEE binary16 <-> wider types (no hardware half used) ---------- */

static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1, ex = (h >> 10) & 31, man = h & 1023;
    double v;
    if (ex == 0) v = ldexp((double)man, -24);
    else if (ex == 31) v = man ? NAN : INFINITY;
    else v = ldexp(1.0 + (double)man / 1024.0, ex - 15);
    return sign ? -v : v;
}

/* round-to-nearest-even of an fp32 value to binary16 */
static uint16_t float_to_half_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t a = u & 0x7fffffffu;
    if (a >= 0x7f800000u) return (uint16_t)(sign | 0x7c00u | ((a > 0x7f800000u) ? 0x200u : 0));
    double v = fabs((double)f);
    if (v >= 65520.0) return (uint16_t)(sign | 0x7c00u);           /* rounds to inf */
    if (v < ldexp(1.0, -25)) return (uint16_t)sign;                /* below half of the smallest subnormal */
    int ex;
    frexp(v, &ex);                                                  /* v = m * 2^ex, m in [0.5,1) */
    int e16 = ex - 1;                                               /* v = 1.xxx * 2^e16 */
    if (e16 < -14) e16 = -14;                                       /* subnormal range: fixed quantum 2^-24 */
    double q = ldexp(v, 10 - e16);                                  /* in units of the target ulp */
    double r = nearbyint(q);                                        /* default rounding mode: nearest even */
    uint32_t bits;
    if (e16 == -14 && r < 1024.0) bits = (uint32_t)r;               /* subnormal */
    else {
        if (r >= 2048.0) { r *= 0.5; e16 += 1; }
        bits = ((uint32_t)(e16 + 15) << 10) + ((uint32_t)r - 1024u);
    }
    return (uint16_t)(sign | bits);
}

/* ---------- Q4_K super-block decoding ----------
 * Semantics (as in config 0 of workloads/configs.py): 256 weights per super-block; fp16 d and dmin;
 * eight 6-bit sub-scales sc_s and eight 6-bit sub-mins m_s; 256 4-bit quants;
 *     w = d * sc_s * q - dmin * m_s,   s = index / 32.
 * Byte layout of the 144 bytes (this repository's layout, version 1):
 *     0..1   d     (binary16, little endian)
 *     2..3   dmin  (binary16, little endian)
 *     4..15  a 96-bit little-endian bit stream of sixteen 6-bit fields; field i
 *            occupies stream bits [6i, 6i+6); fields 0..7 are sc_0..7, 8..15 are m_0..7
 *     16..143 quants: weight t is in byte 16 + t/2, low nibble when t is even.
 * Rounding: w32 = fl32( fl32(fl32(d*sc)*q) - fl32(dmin*m) ); the two products
 * are exact in fp32 (11+6+4 and 11+6 significant bits), so this is the fp32
 * number nearest to the exact rational value.
 */
static unsigned field6(const uint8_t *blk, int i)
{
    unsigned v = 0;
    for (int b = 0; b < 6; ++b) {
        int bit = 6 * i + b;
        v |= (unsigned)((blk[4 + (bit >> 3)] >> (bit & 7)) & 1u) << b;
    }
    return v;
}

static void decode_block(const uint8_t *blk, float *w /* [256] */)
{
    float d = (float)half_to_double((uint16_t)(blk[0] | (blk[1] << 8)));
    float dmin = (float)half_to_double((uint16_t)(blk[2] | (blk[3] << 8)));
    for (int s = 0; s < 8; ++s) {
        float sc = (float)field6(blk, s);
        float m = (float)field6(blk, 8 + s);
        for (int t = 32 * s; t < 32 * s + 32; ++t) {
            uint8_t byte = blk[16 + t / 2];
            float q = (float)((t & 1) ? (byte >> 4) : (byte & 15));
            volatile float p1 = d * sc;
            volatile float p2 = p1 * q;
            volatile float p3 = dmin * m;
            w[t] = p2 - p3;
        }
    }
}

/* out[r][c] = dequantised weight, fp32 */
int orc_q4k_dequant(const uint8_t *W, int64_t n_rows, int64_t n_cols, float *out)
{
    if (n_cols % QK) return 1;
    int64_t nb = n_cols / QK;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r)
        for (int64_t b = 0; b < nb; ++b)
            decode_block(W + (r * nb + b) * BLOCK_BYTES, out + r * n_cols + b * QK);
    return 0;
}

/* y[t][r] = sum_c w32[r][c] * x[t][c], fp64 accumulation, ascending c */
int orc_q4k_gemv(const uint8_t *W, int64_t n_rows, int64_t n_cols,
                 const double *x, int64_t ldx, int32_t T, double *y, int64_t ldy)
{
    if (n_cols % QK) return 1;
    int64_t nb = n_cols / QK;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        float w[QK];
        double acc[64];
        for (int t = 0; t < T; ++t) acc[t] = 0.0;
        for (int64_t b = 0; b < nb; ++b) {
            decode_block(W + (r * nb + b) * BLOCK_BYTES, w);
            for (int t = 0; t < T; ++t) {
                const double *xt = x + (int64_t)t * ldx + b * QK;
                double a = acc[t];
                for (int c = 0; c < QK; ++c) a += (double)w[c] * xt[c];
                acc[t] = a;
            }
        }
        for (int t = 0; t < T; ++t) y[(int64_t)t * ldy + r] = acc[t];
    }
    return 0;
}

/* ---------- the other weight formats of the set Q (Sec. 4 / App. A.3, the profiler's list of formats:
 * Q4_K, Q5_K, Q6_K, Q8_0, FP16, FP32) ----------
 * The paper names the formats and gives no layout.  Field sizes and the value rule are those the names
 * stand for; the placement of the fields is this repository's (version 1): each field of a tensor is a
 * plane of its own, the planes follow one another without padding, and inside a plane blocks are in
 * row-major order (row r, block b -> index r * (n_cols / block) + b).  n = number of 256-weight
 * super-blocks of the tensor.
 *
 * The quant bits of Q5_K and Q6_K are placed word by word (32-bit words, byte t%4 of its word holds bits
 * of weight t), so that four weights come out of a word with one mask:
 *   low 4 bits: one word per 8 weights; byte t%4 of word t/8 holds weight t in its low nibble when
 *     t%8 < 4, in its high nibble otherwise;
 *   bits 4..5 (Q6_K): one word per 16 weights; bits 2g, 2g+1 of byte t%4 of word t/16, g = (t%16)/4;
 *   bit 4 (Q5_K): one word per 32 weights; bit g of byte t%4 of word t/32, g = (t%32)/4.
 *
 *   Q5_K (5.5 bits per weight): plane 1, 16 bytes per super-block: d, dmin (binary16) and the sixteen
 *     6-bit fields exactly as bytes 0..15 of a Q4_K super-block; plane 2 at byte 16 n, 128 bytes per
 *     super-block: the low 4 bits; plane 3 at byte 144 n, 32 bytes per super-block: bit 4.
 *     w = d * sc_s * q - dmin * m_s, q in 0..31, s = t / 32.
 *   Q6_K (6.5625 bits): plane 1, 128 bytes per super-block: the low 4 bits; plane 2 at 128 n, 64
 *     bytes: bits 4..5; plane 3 at 192 n, 16 signed bytes: sc_s for s = t / 16; plane 4 at 208 n:
 *     d (binary16).   w = d * sc_s * (q - 32), q in 0..63.
 *   Q8_0 (8.5 bits): plane 1: one signed byte per weight; plane 2 at n_rows * n_cols: d (binary16) per
 *     32 weights.  w = d * q.
 *   FP16, FP32: row-major numbers.
 * Rounding: every product above is exact in fp32 (at most 11 + 7 + 5 significant bits), so w32 is the
 * fp32 number nearest to the exact value in each format.
 */
enum { FMT_Q4_K = 0, FMT_Q5_K = 1, FMT_Q6_K = 2, FMT_Q8_0 = 3, FMT_F16 = 4, FMT_F32 = 5 };

static float half_at(const uint8_t *p) { return (float)half_to_double((uint16_t)(p[0] | (p[1] << 8))); }

/* low 4 bits of weight t of a super-block whose nibble plane starts at nib */
static int low4(const uint8_t *nib, int t)
{
    uint8_t byte = nib[(t / 8) * 4 + t % 4];
    return (t % 8 < 4) ? (byte & 15) : (byte >> 4);
}

int64_t orc_fmt_tensor_bytes(int32_t fmt, int64_t n_rows, int64_t n_cols)
{
    if (n_rows < 0 || n_cols < 0 || n_cols % QK) return -1;
    int64_t n = n_rows * (n_cols / QK);
    switch (fmt) {
    case FMT_Q4_K: return n * 144;
    case FMT_Q5_K: return n * 176;
    case FMT_Q6_K: return n * 210;
    case FMT_Q8_0: return n * 272;
    case FMT_F16: return n * 512;
    case FMT_F32: return n * 1024;
    }
    return -1;
}

/* the dequantised weights of row r, fp32 */
static void decode_row(int32_t fmt, const uint8_t *W, int64_t n_rows, int64_t n_cols, int64_t r, float *w)
{
    int64_t nb = n_cols / QK, n = n_rows * nb;
    for (int64_t b = 0; b < nb; ++b) {
        int64_t blk = r * nb + b;
        float *o = w + b * QK;
        if (fmt == FMT_Q4_K) {
            decode_block(W + blk * BLOCK_BYTES, o);
        } else if (fmt == FMT_Q5_K) {
            const uint8_t *hdr = W + blk * 16, *qs = W + 16 * n + blk * 128, *qh = W + 144 * n + blk * 32;
            float d = half_at(hdr), dmin = half_at(hdr + 2);
            for (int t = 0; t < QK; ++t) {
                int s = t / 32;
                float sc = (float)field6(hdr, s), m = (float)field6(hdr, 8 + s); /* field6 skips the 4 bytes of d, dmin */
                int lo = low4(qs, t);
                int hi = (qh[(t / 32) * 4 + t % 4] >> ((t % 32) / 4)) & 1;
                volatile float p1 = d * sc;
                volatile float p2 = p1 * (float)(lo | (hi << 4));
                volatile float p3 = dmin * m;
                o[t] = p2 - p3;
            }
        } else if (fmt == FMT_Q6_K) {
            const uint8_t *ql = W + blk * 128, *qh = W + 128 * n + blk * 64;
            const int8_t *sc = (const int8_t *)(W + 192 * n + blk * 16);
            float d = half_at(W + 208 * n + blk * 2);
            for (int t = 0; t < QK; ++t) {
                int lo = low4(ql, t);
                int hi = (qh[(t / 16) * 4 + t % 4] >> (2 * ((t % 16) / 4))) & 3;
                volatile float p1 = d * (float)sc[t / 16];
                o[t] = p1 * (float)((lo | (hi << 4)) - 32);
            }
        } else if (fmt == FMT_Q8_0) {
            const int8_t *q = (const int8_t *)W + blk * QK;
            const uint8_t *dp = W + n_rows * n_cols + blk * 16; /* 8 scales of 2 bytes per 256 weights */
            for (int t = 0; t < QK; ++t) o[t] = half_at(dp + 2 * (t / 32)) * (float)q[t];
        } else if (fmt == FMT_F16) {
            for (int t = 0; t < QK; ++t) o[t] = half_at(W + (blk * QK + t) * 2);
        } else {
            memcpy(o, W + blk * QK * 4, QK * 4);
        }
    }
}

int orc_fmt_dequant(int32_t fmt, const uint8_t *W, int64_t n_rows, int64_t n_cols, float *out)
{
    if (orc_fmt_tensor_bytes(fmt, n_rows, n_cols) < 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) decode_row(fmt, W, n_rows, n_cols, r, out + r * n_cols);
    return 0;
}

/* y[t][r] = sum_c w32[r][c] * x[t][c], fp64 accumulation, ascending c */
int orc_fmt_gemv(int32_t fmt, const uint8_t *W, int64_t n_rows, int64_t n_cols,
                 const double *x, int64_t ldx, int32_t T, double *y, int64_t ldy)
{
    if (orc_fmt_tensor_bytes(fmt, n_rows, n_cols) < 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        float *w = malloc(sizeof(float) * (size_t)(n_cols ? n_cols : 1));
        decode_row(fmt, W, n_rows, n_cols, r, w);
        for (int t = 0; t < T; ++t) {
            const double *xt = x + (int64_t)t * ldx;
            double a = 0.0;
            for (int64_t c = 0; c < n_cols; ++c) a += (double)w[c] * xt[c];
            y[(int64_t)t * ldy + r] = a;
        }
        free(w);
    }
    return 0;
}

/* RMSNorm: out_i = x_i * g_i / sqrt(mean(x^2) + eps) (eps inside the root, gain after) */
void orc_rmsnorm(const double *x, const float *g, int32_t n, double eps, double *out)
{
    double ss = 0.0;
    for (int i = 0; i < n; ++i) ss += x[i] * x[i];
    double inv = 1.0 / sqrt(ss / (double)n + eps);
    for (int i = 0; i < n; ++i) out[i] = x[i] * inv * (double)g[i];
}

/* RoPE on one token's heads, in place: pair index i < D/2 is rotated by pos * theta^(-2i/D) */
void orc_rope(double *v, int32_t n_heads, int32_t D, int32_t pos, double theta, int32_t mode)
{
    int half = D / 2;
    for (int h = 0; h < n_heads; ++h) {
        double *p = v + (int64_t)h * D;
        for (int i = 0; i < half; ++i) {
            double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)D);
            double c = cos(ang), s = sin(ang);
            int ia = mode ? 2 * i : i, ib = mode ? 2 * i + 1 : i + half;
            double a = p[ia], b = p[ib];
            p[ia] = a * c - b * s;
            p[ib] = a * s + b * c;
        }
    }
}

/* silu(g) * u, silu(z) = z / (1 + exp(-z)) */
void orc_swiglu(const double *g, const double *u, int64_t n, double *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = g[i] / (1.0 + exp(-g[i])) * u[i];
}

/* GQA decode attention.
 * q [T][Hq][D] fp64; K, V fp16 [Hkv][kv_cap][D]; token j attends to cache rows 0..n_past+j
 * (rows n_past..n_past+T-1 must already hold the new tokens); query head h reads KV head
 * h / (Hq/Hkv).  o [T][Hq][D].  min_gap (optional) receives the smallest difference between
 * the two largest logits over all (j,h) that see at least two keys.
 */
int orc_attn_decode(const orc_dims *d, const double *q, const uint16_t *K, const uint16_t *V,
                    int32_t kv_cap, int32_t n_past, int32_t T, double *o, double *min_gap)
{
    int Hq = d->n_q_heads, Hkv = d->n_kv_heads, D = d->head_dim;
    if (Hq % Hkv || n_past + T > kv_cap) return 1;
    int grp = Hq / Hkv;
    double scale = 1.0 / sqrt((double)D);
    double gap_all = INFINITY;
#pragma omp parallel for collapse(2) schedule(static) reduction(min : gap_all)
    for (int j = 0; j < T; ++j)
        for (int h = 0; h < Hq; ++h) {
            int n = n_past + j + 1;
            const uint16_t *Kh = K + (int64_t)(h / grp) * kv_cap * D;
            const uint16_t *Vh = V + (int64_t)(h / grp) * kv_cap * D;
            const double *qh = q + ((int64_t)j * Hq + h) * D;
            double *s = (double *)malloc(sizeof(double) * (size_t)n);
            double mx = -INFINITY, mx2 = -INFINITY;
            for (int p = 0; p < n; ++p) {
                double a = 0.0;
                for (int i = 0; i < D; ++i) a += qh[i] * half_to_double(Kh[(int64_t)p * D + i]);
                a *= scale;
                s[p] = a;
                if (a > mx) { mx2 = mx; mx = a; } else if (a > mx2) mx2 = a;
            }
            if (n >= 2 && mx - mx2 < gap_all) gap_all = mx - mx2;
            double den = 0.0;
            for (int p = 0; p < n; ++p) { s[p] = exp(s[p] - mx); den += s[p]; }
            double *oh = o + ((int64_t)j * Hq + h) * D;
            for (int i = 0; i < D; ++i) oh[i] = 0.0;
            for (int p = 0; p < n; ++p) {
                double w = s[p] / den;
                for (int i = 0; i < D; ++i) oh[i] += w * half_to_double(Vh[(int64_t)p * D + i]);
            }
            free(s);
        }
    if (min_gap) *min_gap = gap_all;
    return 0;
}

/* softmax weights of one (token, head) for the invariants test: w[p], p = 0..n-1 */
void orc_softmax(const double *logits, int32_t n, double *w)
{
    double mx = -INFINITY, den = 0.0;
    for (int p = 0; p < n; ++p) if (logits[p] > mx) mx = logits[p];
    for (int p = 0; p < n; ++p) { w[p] = exp(logits[p] - mx); den += w[p]; }
    for (int p = 0; p < n; ++p) w[p] /= den;
}

/* append the T new tokens' k (already rotated) and v to the fp16 cache at rows n_past..n_past+T-1:
 * each value is the hidden fp64 value rounded to fp32 and then to binary16, both nearest-even
 * (the kernel stores from fp32, so the storing decision is taken in that precision). */
void orc_kv_append(const orc_dims *d, const double *k, const double *v, uint16_t *K, uint16_t *V,
                   int32_t kv_cap, int32_t n_past, int32_t T)
{
    int Hkv = d->n_kv_heads, D = d->head_dim;
    for (int j = 0; j < T; ++j)
        for (int h = 0; h < Hkv; ++h)
            for (int i = 0; i < D; ++i) {
                int64_t dst = ((int64_t)h * kv_cap + n_past + j) * D + i;
                int64_t src = ((int64_t)j * Hkv + h) * D + i;
                K[dst] = float_to_half_rne((float)k[src]);
                V[dst] = float_to_half_rne((float)v[src]);
            }
}

/* One pre-norm decoder layer advanced by T tokens (standard Llama/Qwen topology, no biases):
 *   n1 = rmsnorm(x; g_attn); q,k,v = Wq n1, Wk n1, Wv n1; rope(q), rope(k) at pos = n_past + j;
 *   cache rows n_past+j <- fp16(k), fp16(v); a = attention over the cache; h = x + Wo a;
 *   n2 = rmsnorm(h; g_ffn); y = h + Wdown( silu(Wgate n2) * (Wup n2) ).
 * x_in, x_out: fp64 [T][e] (may alias).  Optional taps (may be NULL): tap_q [T][qd] rotated
 * queries, tap_o [T][qd] attention output, tap_h [T][e] post-attention hidden state,
 * tap_a [T][ffn] SwiGLU output.
 */
/* a projection in the format of its tensor (0: Q4_K, the decoder above) */
static int gemv_any(int32_t fmt, const uint8_t *W, int64_t n_rows, int64_t n_cols,
                    const double *x, int64_t ldx, int32_t T, double *y, int64_t ldy)
{
    if (fmt == FMT_Q4_K) return orc_q4k_gemv(W, n_rows, n_cols, x, ldx, T, y, ldy);
    return orc_fmt_gemv(fmt, W, n_rows, n_cols, x, ldx, T, y, ldy);
}

/* fmts: the formats of wq, wk, wv, wo, wgate, wup, wdown (a "Q4K" model keeps some tensors in other formats,
 * Sec. 4 / App. A.3); the layer's arithmetic does not depend on them */
int orc_layer_fmt(const orc_dims *d, const int32_t *fmts,
              const uint8_t *wq, const uint8_t *wk, const uint8_t *wv, const uint8_t *wo,
              const uint8_t *wgate, const uint8_t *wup, const uint8_t *wdown,
              const float *g_attn, const float *g_ffn,
              uint16_t *k_cache, uint16_t *v_cache, int32_t kv_cap, int32_t n_past, int32_t T,
              const double *x_in, double *x_out,
              double *tap_q, double *tap_o, double *tap_h, double *tap_a, double *min_gap)
{
    int e = d->e, D = d->head_dim, F = d->ffn;
    int64_t qd = (int64_t)d->n_q_heads * D, kvd = (int64_t)d->n_kv_heads * D;
    if (n_past + T > kv_cap || T < 1 || T > 64) return 1;
    double *n1 = malloc(sizeof(double) * T * e), *q = malloc(sizeof(double) * T * qd);
    double *k = malloc(sizeof(double) * T * kvd), *v = malloc(sizeof(double) * T * kvd);
    double *a = malloc(sizeof(double) * T * qd), *h = malloc(sizeof(double) * T * e);
    double *g = malloc(sizeof(double) * T * F), *u = malloc(sizeof(double) * T * F);
    double *dn = malloc(sizeof(double) * T * e);
    int rc = 0;
    for (int j = 0; j < T; ++j) orc_rmsnorm(x_in + (int64_t)j * e, g_attn, e, d->rms_eps, n1 + (int64_t)j * e);
    rc |= gemv_any(fmts[0], wq, qd, e, n1, e, T, q, qd);
    rc |= gemv_any(fmts[1], wk, kvd, e, n1, e, T, k, kvd);
    rc |= gemv_any(fmts[2], wv, kvd, e, n1, e, T, v, kvd);
    for (int j = 0; j < T; ++j) {
        orc_rope(q + j * qd, d->n_q_heads, D, n_past + j, d->rope_theta, d->rope_mode);
        orc_rope(k + j * kvd, d->n_kv_heads, D, n_past + j, d->rope_theta, d->rope_mode);
    }
    orc_kv_append(d, k, v, k_cache, v_cache, kv_cap, n_past, T);
    rc |= orc_attn_decode(d, q, k_cache, v_cache, kv_cap, n_past, T, a, min_gap);
    if (tap_q) memcpy(tap_q, q, sizeof(double) * T * qd);
    if (tap_o) memcpy(tap_o, a, sizeof(double) * T * qd);
    rc |= gemv_any(fmts[3], wo, e, qd, a, qd, T, h, e);
    for (int64_t i = 0; i < (int64_t)T * e; ++i) h[i] += x_in[i];
    if (tap_h) memcpy(tap_h, h, sizeof(double) * T * e);
    for (int j = 0; j < T; ++j) orc_rmsnorm(h + (int64_t)j * e, g_ffn, e, d->rms_eps, n1 + (int64_t)j * e);
    rc |= gemv_any(fmts[4], wgate, F, e, n1, e, T, g, F);
    rc |= gemv_any(fmts[5], wup, F, e, n1, e, T, u, F);
    orc_swiglu(g, u, (int64_t)T * F, g);
    if (tap_a) memcpy(tap_a, g, sizeof(double) * T * F);
    rc |= gemv_any(fmts[6], wdown, e, F, g, F, T, dn, e);
    for (int64_t i = 0; i < (int64_t)T * e; ++i) x_out[i] = h[i] + dn[i];
    free(n1); free(q); free(k); free(v); free(a); free(h); free(g); free(u); free(dn);
    return rc;
}

int orc_layer(const orc_dims *d,
              const uint8_t *wq, const uint8_t *wk, const uint8_t *wv, const uint8_t *wo,
              const uint8_t *wgate, const uint8_t *wup, const uint8_t *wdown,
              const float *g_attn, const float *g_ffn,
              uint16_t *k_cache, uint16_t *v_cache, int32_t kv_cap, int32_t n_past, int32_t T,
              const double *x_in, double *x_out,
              double *tap_q, double *tap_o, double *tap_h, double *tap_a, double *min_gap)
{
    const int32_t all_q4k[7] = {0, 0, 0, 0, 0, 0, 0};
    return orc_layer_fmt(d, all_q4k, wq, wk, wv, wo, wgate, wup, wdown, g_attn, g_ffn, k_cache, v_cache, kv_cap, n_past, T,
                         x_in, x_out, tap_q, tap_o, tap_h, tap_a, min_gap);
}

/* output layer: logits[t][v] = W_lm . rmsnorm(x_t; g_final) */
int orc_lm_head(const orc_dims *d, const float *g_final, const uint8_t *w_lm, int64_t vocab,
                const double *x, int32_t T, double *logits)
{
    int e = d->e;
    double *n = malloc(sizeof(double) * T * e);
    for (int j = 0; j < T; ++j) orc_rmsnorm(x + (int64_t)j * e, g_final, e, d->rms_eps, n + (int64_t)j * e);
    int rc = orc_q4k_gemv(w_lm, vocab, e, n, e, T, logits, vocab);
    free(n);
    return rc;
}

/* the same with the output matrix in any format of the set */
int orc_lm_head_fmt(const orc_dims *d, int32_t fmt, const float *g_final, const uint8_t *w_lm, int64_t vocab,
                    const double *x, int32_t T, double *logits)
{
    int e = d->e;
    double *n = malloc(sizeof(double) * T * e);
    for (int j = 0; j < T; ++j) orc_rmsnorm(x + (int64_t)j * e, g_final, e, d->rms_eps, n + (int64_t)j * e);
    int rc = orc_fmt_gemv(fmt, w_lm, vocab, e, n, e, T, logits, vocab);
    free(n);
    return rc;
}

uint16_t orc_float_to_half(float f) { return float_to_half_rne(f); }
double orc_half_to_double(uint16_t h) { return half_to_double(h); }

#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
void orc_set_num_threads(int n) { omp_set_num_threads(n); }
#else
int orc_num_threads(void) { return 1; }
void orc_set_num_threads(int n) { (void)n; }
#endif
