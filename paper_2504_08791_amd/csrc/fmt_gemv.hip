// Mat-vec and dequantisation for the other weight formats of the paper's format set (Sec. 4 / App. A.3, the
// profiler's list: Q5_K, Q6_K, Q8_0, FP16, FP32; Q4_K has the MFMA kernel of q4k_gemv_mfma.hip).
//
// Layout (version 1, this repository's): every field of a tensor is a plane of its own, the planes follow one
// another without padding, blocks inside a plane are in row-major order; n = rows * cols / 256 super-blocks.
// Quant bits of Q5_K / Q6_K sit in 32-bit words, weight t always in byte t%4 of its word:
//   low 4 bits: word t/8, low nibble when t%8 < 4, else high nibble;
//   bits 4..5 (Q6_K): word t/16, bits 2g, 2g+1, g = (t%16)/4;    bit 4 (Q5_K): word t/32, bit g = (t%32)/4.
// so that four weights come out of a word as the four bytes of  (low >> 0|4) & 0x0F0F0F0F | (high << s) & mask.
//   Q5_K  [n][16] d, dmin (binary16) + sixteen 6-bit fields (sc_0..7, m_0..7: a 96-bit little-endian stream) |
//         [n][128] low 4 bits | [n][32] bit 4;     w = d sc_s q - dmin m_s, s = t/32
//   Q6_K  [n][128] low 4 bits | [n][64] bits 4..5 | [n][16] int8 sc_s, s = t/16 | [n] binary16 d;
//         w = d sc_s (q - 32)
//   Q8_0  [rows*cols] int8 | [rows*cols/32] binary16 d;  w = d q
//   FP16, FP32: row-major numbers.
// With the fields in planes every lane's load is aligned to its size and a wave's loads are contiguous,
// whatever the block size (210 and 34 bytes per block otherwise); the bytes per weight are the formats' own.
//
// Mat-vec design: HBM-bound streaming with fp32 vector arithmetic (no matrix cores: one to eight tokens leave
// them nothing to contract).  One workgroup of 16 waves per compute unit keeps the activations in LDS (up to
// 128 KB: all of K for one token up to K = 32768; otherwise K is walked in chunks and y accumulates chunk by
// chunk), with the RMSNorm gain already applied: read from L2 by every wave they cost as much bandwidth as
// the weights (measured: every quantised format stuck at the same 4.6 T weights/s, FP16 alone reached the
// HBM rate).  A wave owns its rows outright: R rows (4; with few rows 1 at one or two tokens and 2 at three or
// four, for balance; always 2 from five tokens on, for registers) times U = 4/R pieces of 1024 weights per
// step, a lane taking 16 consecutive weights of a piece: one 4..16-byte load per
// field, four loads in flight per lane.  The 16 weights of a lane lie in one sub-block of every format, so a
// lane needs one scale per piece and adds  scale * (sum q x) - offset * (sum x): one multiply-add per weight
// and token plus the unpacking, which the tokens share.  Lanes are summed by row rotations and permlane swaps;
// nothing is summed across waves, so results do not depend on the launch.  RMSNorm in front (optional): 1/rms
// multiplies the finished sums; every workgroup computes the mean squares itself.  Residual behind (optional).
#include <hip/hip_fp16.h>

#include <atomic>

#include "common.h"

namespace prima {
namespace {

constexpr int FG_THREADS = 1024;
constexpr int FG_WAVES = FG_THREADS / 64;
constexpr int FG_V = 16;                 // weights per lane in one piece
constexpr int FG_PIECE = 64 * FG_V;      // weights per wave in one piece
constexpr int FG_MAX_T = 8;              // tokens per pass over the weights
constexpr int FG_X_BYTES = 128 * 1024;   // LDS for the activations
constexpr int FG_CUS = 256;
constexpr int FG_TAIL_BYTES = (FG_MAX_T + FG_MAX_T * FG_WAVES) * 4; // 1/rms per token and the waves' partial mean squares

struct FmtArgs {
    const uint8_t *W;
    int64_t n_rows, n_cols;
    const float *x;
    int64_t ldx;
    const float *gain; // null: plain activations
    float eps;
    const float *resid; // null: none
    int64_t ldr;
    float *y;
    int64_t ldy;
    int T;
    int kc; // weights per chunk of K (a multiple of FG_PIECE)
};

__device__ __forceinline__ float half_bits_to_float(unsigned h) { return __half2float(__ushort_as_half(static_cast<unsigned short>(h))); }

// Sub-scale and sub-min of sub-block s (0..7) from a Q5_K header: fields s and 8 + s of the 96-bit stream in
// words 1..3, i.e. stream bits 6s.. (inside words 1, 2) and 48 + 6s.. (inside words 2, 3): one 64-bit shift each
__device__ __forceinline__ void q5k_scale_min(const uint4 &hdr, int s, unsigned &sc, unsigned &m)
{
    const uint64_t lo = hdr.y | (static_cast<uint64_t>(hdr.z) << 32); // stream bits 0..63
    const uint64_t hi = hdr.z | (static_cast<uint64_t>(hdr.w) << 32); // stream bits 32..95
    sc = static_cast<unsigned>(lo >> (6 * s)) & 63u;
    m = static_cast<unsigned>(hi >> (16 + 6 * s)) & 63u;
}

// The bytes of the 16 weights of (row, k0..k0+15) as loaded (Raw), and as fp32 numbers q[16] with
// w = scale * q - offset (Piece; FP16 / FP32: scale 1; Q6_K: q is the stored 0..63 and offset = 32 scale).
template <int FMT> struct Raw;
template <> struct Raw<PRIMA_FMT_Q8_0> { uint4 q; unsigned short d; };
template <> struct Raw<PRIMA_FMT_Q6_K> { uint2 lo; unsigned hi; signed char sc; unsigned short d; };
template <> struct Raw<PRIMA_FMT_Q5_K> { uint4 hdr; uint2 lo; unsigned hi; int s, half; };
template <> struct Raw<PRIMA_FMT_F16> { uint4 a, b; };
template <> struct Raw<PRIMA_FMT_F32> { float4 v[4]; };

struct Piece {
    float q[FG_V];
    float scale, offset;
};

// a weight field, read once in a launch: non-temporal load (the line is marked to leave the caches first)
typedef unsigned nt_v4u __attribute__((ext_vector_type(4)));
typedef unsigned nt_v2u __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 nt_load16(const void *p)
{
    const nt_v4u v = __builtin_nontemporal_load(static_cast<const nt_v4u *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 nt_load8(const void *p)
{
    const nt_v2u v = __builtin_nontemporal_load(static_cast<const nt_v2u *>(p));
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ unsigned nt_load4(const void *p) { return __builtin_nontemporal_load(static_cast<const unsigned *>(p)); }

template <int FMT>
__device__ __forceinline__ void load_raw(const uint8_t *__restrict__ W, int64_t n_rows, int64_t n_cols, int64_t row, int64_t k0, Raw<FMT> &r)
{
    const int64_t nb = n_cols >> 8, n = n_rows * nb;
    const int64_t blk = row * nb + (k0 >> 8);
    const int t0 = static_cast<int>(k0 & 255);
    if constexpr (FMT == PRIMA_FMT_Q8_0) {
        r.q = nt_load16(W + row * n_cols + k0);
        r.d = *reinterpret_cast<const unsigned short *>(W + n_rows * n_cols + ((row * n_cols + k0) >> 5) * 2);
    } else if constexpr (FMT == PRIMA_FMT_Q6_K) {
        r.lo = nt_load8(W + blk * 128 + (t0 >> 1));
        r.hi = nt_load4(W + 128 * n + blk * 64 + (t0 >> 2));
        r.sc = *reinterpret_cast<const signed char *>(W + 192 * n + blk * 16 + (t0 >> 4));
        r.d = *reinterpret_cast<const unsigned short *>(W + 208 * n + blk * 2);
    } else if constexpr (FMT == PRIMA_FMT_Q5_K) {
        r.hdr = *reinterpret_cast<const uint4 *>(W + blk * 16);
        r.lo = nt_load8(W + 16 * n + blk * 128 + (t0 >> 1));
        r.hi = nt_load4(W + 144 * n + blk * 32 + (t0 >> 5) * 4); // one word per 32 weights: shared by two lanes
        r.s = t0 >> 5;
        r.half = (t0 >> 4) & 1;
    } else if constexpr (FMT == PRIMA_FMT_F16) {
        r.a = nt_load16(W + (row * n_cols + k0) * 2);
        r.b = nt_load16(W + (row * n_cols + k0) * 2 + 16);
    } else {
        static_assert(FMT == PRIMA_FMT_F32, "format");
        const float4 *src = reinterpret_cast<const float4 *>(W + (row * n_cols + k0) * 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) r.v[i] = src[i];
    }
}

__device__ __forceinline__ void bytes_to_floats(unsigned b, float *dst)
{
    dst[0] = static_cast<float>(b & 0xFFu);
    dst[1] = static_cast<float>((b >> 8) & 0xFFu);
    dst[2] = static_cast<float>((b >> 16) & 0xFFu);
    dst[3] = static_cast<float>(b >> 24);
}

template <int FMT>
__device__ __forceinline__ void decode(const Raw<FMT> &r, Piece &p)
{
    p.offset = 0.f;
    p.scale = 1.f;
    if constexpr (FMT == PRIMA_FMT_Q8_0) {
        const unsigned wv[4] = {r.q.x, r.q.y, r.q.z, r.q.w};
#pragma unroll
        for (int i = 0; i < 16; ++i) p.q[i] = static_cast<float>(static_cast<int>(wv[i >> 2] << (24 - 8 * (i & 3))) >> 24);
        p.scale = half_bits_to_float(r.d);
    } else if constexpr (FMT == PRIMA_FMT_Q6_K) {
        // weights 4g..4g+3 are the bytes of (low word g/2 >> 4(g%2)) & 0x0F0F0F0F | (high word >> 2g << 4) & 0x30303030
        const unsigned h = r.hi;
        bytes_to_floats((r.lo.x & 0x0F0F0F0Fu) | ((h << 4) & 0x30303030u), p.q);
        bytes_to_floats(((r.lo.x >> 4) & 0x0F0F0F0Fu) | ((h << 2) & 0x30303030u), p.q + 4);
        bytes_to_floats((r.lo.y & 0x0F0F0F0Fu) | (h & 0x30303030u), p.q + 8);
        bytes_to_floats(((r.lo.y >> 4) & 0x0F0F0F0Fu) | ((h >> 2) & 0x30303030u), p.q + 12);
        p.scale = half_bits_to_float(r.d) * static_cast<float>(r.sc); // exact: 11 + 7 bits
        p.offset = 32.f * p.scale;                                    // exact
    } else if constexpr (FMT == PRIMA_FMT_Q5_K) {
        const unsigned h = r.half ? r.hi >> 4 : r.hi; // bits g = 0..3 of every byte: this lane's four groups of four
        bytes_to_floats((r.lo.x & 0x0F0F0F0Fu) | ((h << 4) & 0x10101010u), p.q);
        bytes_to_floats(((r.lo.x >> 4) & 0x0F0F0F0Fu) | ((h << 3) & 0x10101010u), p.q + 4);
        bytes_to_floats((r.lo.y & 0x0F0F0F0Fu) | ((h << 2) & 0x10101010u), p.q + 8);
        bytes_to_floats(((r.lo.y >> 4) & 0x0F0F0F0Fu) | ((h << 1) & 0x10101010u), p.q + 12);
        unsigned sc, m;
        q5k_scale_min(r.hdr, r.s, sc, m);
        p.scale = half_bits_to_float(r.hdr.x & 0xFFFFu) * static_cast<float>(sc); // exact
        p.offset = half_bits_to_float(r.hdr.x >> 16) * static_cast<float>(m);    // exact
    } else if constexpr (FMT == PRIMA_FMT_F16) {
        const unsigned wv[8] = {r.a.x, r.a.y, r.a.z, r.a.w, r.b.x, r.b.y, r.b.z, r.b.w};
#pragma unroll
        for (int i = 0; i < 16; ++i) p.q[i] = half_bits_to_float((wv[i >> 1] >> (16 * (i & 1))) & 0xFFFFu);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            p.q[4 * i] = r.v[i].x; p.q[4 * i + 1] = r.v[i].y; p.q[4 * i + 2] = r.v[i].z; p.q[4 * i + 3] = r.v[i].w;
        }
    }
}

// out[r][c] = w, fp32, one thread per 16 weights.  Rounding: the products are exact in fp32 (Q6_K: d sc q with
// q up to 63 has 11 + 7 + 6 significant bits, 32 d sc is exact), the one subtraction of Q5_K / Q6_K rounds once
// (with or without contraction into a multiply-add: the same number), to the fp32 nearest to the exact weight.
template <int FMT>
__global__ void __launch_bounds__(256) fmt_dequant_kernel(const uint8_t *__restrict__ W, int64_t n_rows, int64_t n_cols, float *__restrict__ out)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t per_row = n_cols / FG_V;
    if (idx >= n_rows * per_row) return;
    const int64_t row = idx / per_row, k0 = (idx - row * per_row) * FG_V;
    Raw<FMT> raw;
    load_raw<FMT>(W, n_rows, n_cols, row, k0, raw);
    Piece p;
    decode<FMT>(raw, p);
    float4 *dst = reinterpret_cast<float4 *>(out + row * n_cols + k0);
    // (Q6_K: the difference first, so that a zero weight keeps the sign of d sc times zero)
    auto value = [&](float q) __attribute__((always_inline)) {
        if constexpr (FMT == PRIMA_FMT_Q6_K) return p.scale * (q - 32.f);
        else return p.scale * q - p.offset;
    };
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float4 v;
        v.x = value(p.q[4 * i]);
        v.y = value(p.q[4 * i + 1]);
        v.z = value(p.q[4 * i + 2]);
        v.w = value(p.q[4 * i + 3]);
        dst[i] = v;
    }
}

// LDS: the activations of a chunk, [TT][kc] floats with the gain applied, each piece of 1024 stored as [4][64]
// float4 (a lane's i-th float4 at [i][lane]: a wave's reads are contiguous), then 1/rms [TT] and [TT][16] partial sums.
template <int FMT, int TT, int R>
__global__ void __launch_bounds__(FG_THREADS) fmt_gemv_kernel(FmtArgs a)
{
    // pieces in flight per lane (8 for the quantised formats, whose pieces are only 11..18 bytes per lane, measured
    // the same or slower)
    constexpr int NP = 4;
    constexpr int U = NP / R; // pieces of a row per step
    extern __shared__ __align__(16) float l_mem[];
    const int kc = a.kc;
    float4 *const l_x4 = reinterpret_cast<float4 *>(l_mem);
    float *const l_inv = l_mem + static_cast<size_t>(TT) * kc;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t K = a.n_cols;
    const float *__restrict__ x = a.x;
    const float *__restrict__ gain = a.gain;

    // 1/rms of every token (RMSNorm in front): all threads read, waves are summed in wave order
    if (gain) {
        float *const l_red = l_inv + TT; // [TT][FG_WAVES]
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            float ss = 0.f;
            for (int64_t k = static_cast<int64_t>(threadIdx.x) * 4; k < K; k += FG_THREADS * 4) {
                const float4 v = *reinterpret_cast<const float4 *>(x + t * a.ldx + k);
                ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
            }
            ss = wave_sum(ss);
            if (lane == 0) l_red[t * FG_WAVES + wave] = ss;
        }
        __syncthreads();
        if (threadIdx.x < TT) {
            float ss = 0.f;
            for (int w = 0; w < FG_WAVES; ++w) ss += l_red[threadIdx.x * FG_WAVES + w];
            l_inv[threadIdx.x] = 1.0f / sqrtf(ss / static_cast<float>(K) + a.eps);
        }
    } else if (threadIdx.x < TT) {
        l_inv[threadIdx.x] = 1.f;
    }

    const int64_t n_tasks = (a.n_rows + R - 1) / R;
    for (int64_t c0 = 0; c0 < K; c0 += kc) {
        const int len = static_cast<int>(K - c0 < kc ? K - c0 : kc); // a multiple of 256
        __syncthreads(); // the previous chunk has been used
        for (int f = threadIdx.x; f < TT * (len >> 2); f += FG_THREADS) {
            const int t = f / (len >> 2), f4 = f - t * (len >> 2); // float4 f4 of token t of this chunk
            float4 v = *reinterpret_cast<const float4 *>(x + t * a.ldx + c0 + 4 * f4);
            if (gain) {
                const float4 g = *reinterpret_cast<const float4 *>(gain + c0 + 4 * f4);
                v.x *= g.x; v.y *= g.y; v.z *= g.z; v.w *= g.w;
            }
            const int piece = f4 >> 8, in_piece = f4 & 255;
            l_x4[t * (kc >> 2) + piece * 256 + (in_piece & 3) * 64 + (in_piece >> 2)] = v;
        }
        __syncthreads();

        for (int64_t task = static_cast<int64_t>(blockIdx.x) * FG_WAVES + wave; task < n_tasks; task += static_cast<int64_t>(gridDim.x) * FG_WAVES) {
            const int64_t row0 = task * R;
            int64_t rows[R];
#pragma unroll
            for (int r = 0; r < R; ++r) rows[r] = row0 + r < a.n_rows ? row0 + r : a.n_rows - 1; // past the end: a valid row, not stored
            float acc[R][TT];
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int t = 0; t < TT; ++t) acc[r][t] = 0.f;

            // one step: U pieces of each of the R rows: all loads requested, then decoded and used piece by piece
            auto load_step = [&](Raw<FMT> (&raw)[U][R], int kk) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int kq = kk + u * FG_PIECE < len ? kk + u * FG_PIECE : kk; // past the end: this lane's first piece again, not used
#pragma unroll
                    for (int r = 0; r < R; ++r) load_raw<FMT>(a.W, a.n_rows, K, rows[r], c0 + kq, raw[u][r]);
                }
            };
            auto use_step = [&](const Raw<FMT> (&raw)[U][R], int kk) __attribute__((always_inline)) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (kk + u * FG_PIECE < len) {
                        const float4 *xp = l_x4 + ((kk + u * FG_PIECE) >> 10) * 256 + lane;
                        Piece p[R];
#pragma unroll
                        for (int r = 0; r < R; ++r) decode<FMT>(raw[u][r], p[r]);
#pragma unroll
                        for (int t = 0; t < TT; ++t) {
                            float xv[FG_V];
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float4 v = xp[t * (kc >> 2) + i * 64];
                                xv[4 * i] = v.x; xv[4 * i + 1] = v.y; xv[4 * i + 2] = v.z; xv[4 * i + 3] = v.w;
                            }
                            float sx = 0.f;
                            if constexpr (FMT == PRIMA_FMT_Q5_K || FMT == PRIMA_FMT_Q6_K) {
#pragma unroll
                                for (int i = 0; i < FG_V; ++i) sx += xv[i];
                            }
#pragma unroll
                            for (int r = 0; r < R; ++r) {
                                float s = 0.f;
#pragma unroll
                                for (int i = 0; i < FG_V; ++i) s = fmaf(p[r].q[i], xv[i], s);
                                if constexpr (FMT == PRIMA_FMT_Q5_K || FMT == PRIMA_FMT_Q6_K) acc[r][t] += p[r].scale * s - p[r].offset * sx;
                                else if constexpr (FMT == PRIMA_FMT_F16 || FMT == PRIMA_FMT_F32) acc[r][t] += s;
                                else acc[r][t] = fmaf(p[r].scale, s, acc[r][t]);
                            }
                        }
                    }
                }
            };
            constexpr int STEP = U * FG_PIECE;
            int kk = lane * FG_V;
            // (Requesting the next step's weights before this step's arithmetic, with a second set of registers, was
            // measured: no gain at one token, spills beyond; the other waves of the SIMD already cover the wait.
            // Two workgroups per compute unit at one token (64 registers a lane, 8 waves per SIMD): 10-30 % slower.)
            for (; kk < len; kk += STEP) {
                Raw<FMT> raw[U][R];
                load_step(raw, kk);
                use_step(raw, kk);
            }

            // lanes; the first chunk writes y (with the residual), the others add to it (same lane, in chunk order)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    float v = wave_sum(acc[r][t]) * l_inv[t];
                    const int64_t row = row0 + r;
                    if (lane == 0 && row < a.n_rows) {
                        float *dst = a.y + t * a.ldy + row;
                        if (c0 == 0) {
                            if (a.resid) v += a.resid[t * a.ldr + row];
                        } else {
                            v += *dst;
                        }
                        *dst = v;
                    }
                }
        }
    }
}

template <int FMT, int TT, int R>
prima_status launch_ttr(const FmtArgs &a, size_t lds, hipStream_t st)
{
    static std::atomic<bool> attr_set{false}; // set twice by two threads at worst: the attribute call is idempotent
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(fmt_gemv_kernel<FMT, TT, R>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                FG_X_BYTES + FG_TAIL_BYTES) != hipSuccess)
            return PRIMA_E_DEVICE;
        attr_set = true;
    }
    const int64_t n_tasks = (a.n_rows + R - 1) / R;
    const int64_t wgs = (n_tasks + FG_WAVES - 1) / FG_WAVES;
    const int grid = static_cast<int>(wgs < FG_CUS ? wgs : FG_CUS); // one workgroup per compute unit
    hipLaunchKernelGGL((fmt_gemv_kernel<FMT, TT, R>), dim3(grid), dim3(FG_THREADS), lds, st, a);
    return last_launch_status();
}

template <int FMT, int TT>
prima_status launch_tt(FmtArgs a, hipStream_t st)
{
    // weights per chunk: what fits the LDS budget for TT tokens, in whole pieces; not more than K needs
    int kc = FG_X_BYTES / (4 * TT) / FG_PIECE * FG_PIECE;
    const int64_t k_pieces = (a.n_cols + FG_PIECE - 1) / FG_PIECE * FG_PIECE;
    if (k_pieces < kc) kc = static_cast<int>(k_pieces);
    a.kc = kc;
    const size_t lds = static_cast<size_t>(TT) * kc * 4 + FG_TAIL_BYTES;
    // Rows per wave.  4 share one read of the activations from LDS; fewer when there are so few rows that the
    // waves of the device would not have two groups each (they finish together then): 1 row and four pieces of it
    // at a time for one or two tokens, 2 rows for three and four (with 1 their LDS reads would take longer than
    // the arithmetic).  Five and more tokens: 2 rows always (the sums and decoded weights of 4 rows do not fit
    // the 128 registers of a lane).
    const bool few_rows = a.n_rows < int64_t{2} * 4 * FG_CUS * FG_WAVES;
    if constexpr (TT <= 2) return few_rows ? launch_ttr<FMT, TT, 1>(a, lds, st) : launch_ttr<FMT, TT, 4>(a, lds, st);
    else if constexpr (TT <= 4) return few_rows ? launch_ttr<FMT, TT, 2>(a, lds, st) : launch_ttr<FMT, TT, 4>(a, lds, st);
    else return launch_ttr<FMT, TT, 2>(a, lds, st);
}

template <int FMT>
prima_status launch_fmt(FmtArgs a, hipStream_t st)
{
    const float *x = a.x, *resid = a.resid;
    float *y = a.y;
    const int T = a.T;
    for (int t0 = 0; t0 < T; t0 += FG_MAX_T) {
        const int Tp = T - t0 < FG_MAX_T ? T - t0 : FG_MAX_T;
        a.x = x + t0 * a.ldx;
        a.resid = resid ? resid + t0 * a.ldr : nullptr;
        a.y = y + t0 * a.ldy;
        a.T = Tp;
        prima_status s;
        switch (Tp) {
        case 1: s = launch_tt<FMT, 1>(a, st); break;
        case 2: s = launch_tt<FMT, 2>(a, st); break;
        case 3: s = launch_tt<FMT, 3>(a, st); break;
        case 4: s = launch_tt<FMT, 4>(a, st); break;
        case 5: s = launch_tt<FMT, 5>(a, st); break;
        case 6: s = launch_tt<FMT, 6>(a, st); break;
        case 7: s = launch_tt<FMT, 7>(a, st); break;
        default: s = launch_tt<FMT, 8>(a, st); break;
        }
        if (s != PRIMA_OK) return s;
    }
    return PRIMA_OK;
}

} // namespace

size_t fmt_tensor_bytes(int fmt, int64_t n_rows, int64_t n_cols)
{
    if (n_rows < 0 || n_cols < 0 || n_cols % QK) return 0;
    const size_t n = static_cast<size_t>(n_rows) * static_cast<size_t>(n_cols / QK);
    switch (fmt) {
    case PRIMA_FMT_Q4_K: return n * 144;
    case PRIMA_FMT_Q5_K: return n * 176;
    case PRIMA_FMT_Q6_K: return n * 210;
    case PRIMA_FMT_Q8_0: return n * 272;
    case PRIMA_FMT_F16: return n * 512;
    case PRIMA_FMT_F32: return n * 1024;
    }
    return 0;
}

prima_status launch_fmt_dequant(int fmt, const uint8_t *W, int64_t n_rows, int64_t n_cols, float *out, hipStream_t st)
{
    const int64_t n_threads = n_rows * (n_cols / FG_V);
    if (n_threads == 0) return PRIMA_OK;
    if ((n_threads + 255) / 256 >= (int64_t{1} << 31)) return PRIMA_E_SHAPE;
    const dim3 grid(static_cast<unsigned>((n_threads + 255) / 256));
    switch (fmt) {
    case PRIMA_FMT_Q5_K: hipLaunchKernelGGL((fmt_dequant_kernel<PRIMA_FMT_Q5_K>), grid, dim3(256), 0, st, W, n_rows, n_cols, out); break;
    case PRIMA_FMT_Q6_K: hipLaunchKernelGGL((fmt_dequant_kernel<PRIMA_FMT_Q6_K>), grid, dim3(256), 0, st, W, n_rows, n_cols, out); break;
    case PRIMA_FMT_Q8_0: hipLaunchKernelGGL((fmt_dequant_kernel<PRIMA_FMT_Q8_0>), grid, dim3(256), 0, st, W, n_rows, n_cols, out); break;
    case PRIMA_FMT_F16: hipLaunchKernelGGL((fmt_dequant_kernel<PRIMA_FMT_F16>), grid, dim3(256), 0, st, W, n_rows, n_cols, out); break;
    case PRIMA_FMT_F32: hipLaunchKernelGGL((fmt_dequant_kernel<PRIMA_FMT_F32>), grid, dim3(256), 0, st, W, n_rows, n_cols, out); break;
    default: return PRIMA_E_SHAPE;
    }
    return last_launch_status();
}

prima_status launch_fmt_gemv(int fmt, const uint8_t *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int T,
                             const float *gain, float eps, const float *resid, int64_t ldr, float *y, int64_t ldy, hipStream_t st)
{
    if (n_rows == 0) return PRIMA_OK;
    FmtArgs a{W, n_rows, n_cols, x, ldx, gain, eps, resid, ldr, y, ldy, T, 0};
    switch (fmt) {
    case PRIMA_FMT_Q5_K: return launch_fmt<PRIMA_FMT_Q5_K>(a, st);
    case PRIMA_FMT_Q6_K: return launch_fmt<PRIMA_FMT_Q6_K>(a, st);
    case PRIMA_FMT_Q8_0: return launch_fmt<PRIMA_FMT_Q8_0>(a, st);
    case PRIMA_FMT_F16: return launch_fmt<PRIMA_FMT_F16>(a, st);
    case PRIMA_FMT_F32: return launch_fmt<PRIMA_FMT_F32>(a, st);
    default: return PRIMA_E_SHAPE;
    }
}

} // namespace prima
