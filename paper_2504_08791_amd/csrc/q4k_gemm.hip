// Q4_K matrix product for many tokens (prompt processing: the paper reports the time to the first token next to
// the time per output token, Sec. 4.1 / Table 2; the same projections as in decode, App. A.3, for T tokens at once).
//
//     y[t][r] = sum_c W[r][c] * a[t][c],   a = x (or RMSNorm(x; gain)),   + resid[t][r] (optional)
//
// With tens to hundreds of tokens the product is a real contraction and belongs on the matrix cores; the decode
// kernel (tokens as int8 digits, sub-scales applied to every MFMA result) spends four multiply-adds per MFMA and
// token group and stops scaling at 8 tokens.  Here:
//   * the B operand is the weight tile itself: per sub-block of 32 weights the integers sc_s * q (at most 945:
//     exact in binary16), built once per workgroup pass and used for every token of the pass;
//   * the A operand is the activations as two binary16 numbers hi + lo (22 bits), scaled per token by a power
//     of two so that |a| < 4096; products of two binary16 numbers are exact in fp32, the MFMA adds in fp32;
//   * one accumulator per super-block (256 weights, 8 MFMA steps x 2), then  y += d * acc - dmin * sum_s m_s * xs_s
//     with xs_s the sub-block sums of the scaled activations (fp32, from the staging pass).
// Workgroup: 8 waves = 128 rows (16 per wave) x 32 tokens (two 16-token tiles); the activations of a super-block
// are staged once per workgroup into LDS in the A-operand order, the weights go from global memory straight into
// registers (each wave reads only its own 16 rows).  A first kernel gives every token its scale: 2^p (times 1/rms).
#include <hip/hip_fp16.h>

#include "common.h"

namespace prima {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int GM_THREADS = 512;
constexpr int GM_WAVES = GM_THREADS / 64;
constexpr int GM_ROWS = 16 * GM_WAVES; // rows per workgroup
constexpr int GM_TM = 32;              // tokens per workgroup
constexpr int GM_TT = GM_TM / 16;      // 16-token tiles

struct GemmArgs {
    const uint8_t *W;
    int64_t n_rows, n_cols;
    const float *x;
    int64_t ldx;
    const float *gain;  // null: plain activations
    const float2 *stat; // per token: (2^p [* 1/rms], 2^-p)
    const float *resid; // null: none
    int64_t ldr;
    float *y;
    int64_t ldy;
    int T;
};

// per token: 1/rms (RMSNorm in front) and the power of two that brings max |a| below 4096
__global__ void __launch_bounds__(256) gemm_token_scale_kernel(const float *__restrict__ x, int64_t ldx, int64_t K, const float *__restrict__ gain,
                                                               float eps, float2 *__restrict__ stat)
{
    __shared__ float red[2][4];
    const int t = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float ss = 0.f, amax = 0.f;
    for (int64_t k = static_cast<int64_t>(threadIdx.x) * 4; k < K; k += 1024) {
        const float4 v = *reinterpret_cast<const float4 *>(x + t * ldx + k);
        float4 g = make_float4(1.f, 1.f, 1.f, 1.f);
        if (gain) g = *reinterpret_cast<const float4 *>(gain + k);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
        amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v.x * g.x), fabsf(v.y * g.y))), fmaxf(fabsf(v.z * g.z), fabsf(v.w * g.w)));
    }
    ss = wave_sum(ss);
    amax = wave_max(amax);
    if (lane == 0) { red[0][wave] = ss; red[1][wave] = amax; }
    __syncthreads();
    if (threadIdx.x == 0) {
        ss = ((red[0][0] + red[0][1]) + red[0][2]) + red[0][3];
        amax = fmaxf(fmaxf(red[1][0], red[1][1]), fmaxf(red[1][2], red[1][3]));
        const float inv_rms = gain ? 1.0f / sqrtf(ss / static_cast<float>(K) + eps) : 1.f;
        amax *= inv_rms;
        int ex = 0;
        if (amax > 0.f) frexpf(amax, &ex); // amax < 2^ex
        int p = 12 - ex;
        p = p > 100 ? 100 : (p < -100 ? -100 : p);
        stat[t] = make_float2(ldexpf(inv_rms, p), ldexpf(1.0f, -p));
    }
}

struct GemmLds {
    half8 hi[GM_TT][8][64]; // A operand: [token tile][sub-block][lane = token % 16 + 16 * (k / 8)]
    half8 lo[GM_TT][8][64];
    float xs[GM_TM][8];     // sub-block sums of the scaled activations
};

__global__ void __launch_bounds__(GM_THREADS) q4k_gemm_kernel(GemmArgs a)
{
    __shared__ GemmLds lds;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 15, g = lane >> 4;
    const int64_t nb = a.n_cols >> 8;
    const int t0 = blockIdx.y * GM_TM;
    const int64_t row = min<int64_t>(static_cast<int64_t>(blockIdx.x) * GM_ROWS + wave * 16 + n, a.n_rows - 1); // past the end: a valid row, not stored
    const uint8_t *wrow = a.W + row * nb * 144;

    // staging: thread -> (token, 16 consecutive columns of the super-block)
    const int s_tok = threadIdx.x >> 4, s_c0 = (threadIdx.x & 15) * 16;
    const int s_t = min(t0 + s_tok, a.T - 1); // past the last token: a valid token, not stored
    const float2 s_stat = a.stat[s_t];
    const int s_s8 = s_c0 >> 5, s_g0 = (s_c0 & 31) >> 3; // sub-block and first of the two 8-column groups

    v4f yacc[GM_TT];
#pragma unroll
    for (int tt = 0; tt < GM_TT; ++tt) yacc[tt] = {0.f, 0.f, 0.f, 0.f};

    for (int64_t b = 0; b < nb; ++b) {
        // this wave's weights of the super-block: header and the 8 columns 8g.. of every sub-block (requested before
        // the barrier, used after it)
        const uint4 hdr = *reinterpret_cast<const uint4 *>(wrow + b * 144);
        uint32_t qw[8];
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) qw[s8] = *reinterpret_cast<const uint32_t *>(wrow + b * 144 + 16 + 16 * s8 + 4 * g);

        __syncthreads(); // the previous super-block's activations have been used
        {
            const float *xp = a.x + s_t * a.ldx + b * 256 + s_c0;
            float v[16];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 q = *reinterpret_cast<const float4 *>(xp + 4 * i);
                v[4 * i] = q.x; v[4 * i + 1] = q.y; v[4 * i + 2] = q.z; v[4 * i + 3] = q.w;
            }
            if (a.gain) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float4 q = *reinterpret_cast<const float4 *>(a.gain + b * 256 + s_c0 + 4 * i);
                    v[4 * i] *= q.x; v[4 * i + 1] *= q.y; v[4 * i + 2] *= q.z; v[4 * i + 3] *= q.w;
                }
            }
            float sum = 0.f;
            half8 h[2], l[2];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float sv = v[i] * s_stat.x;
                // the product as an opaque fp32 number: left visible, the compiler formed the stored hi from the rounded
                // product and the hi that lo is taken against from the exact one (fused multiply-convert); the two differ
                // now and then by one binary16 step, which lo then does not make up for
                asm volatile("" : "+v"(sv));
                const _Float16 hh = static_cast<_Float16>(sv);
                const _Float16 ll = static_cast<_Float16>(sv - static_cast<float>(hh));
                h[i >> 3][i & 7] = hh;
                l[i >> 3][i & 7] = ll;
                sum += static_cast<float>(hh) + static_cast<float>(ll); // what the MFMAs will see
            }
            const int tt = s_tok >> 4, m = s_tok & 15;
            lds.hi[tt][s_s8][m + 16 * s_g0] = h[0];
            lds.hi[tt][s_s8][m + 16 * (s_g0 + 1)] = h[1];
            lds.lo[tt][s_s8][m + 16 * s_g0] = l[0];
            lds.lo[tt][s_s8][m + 16 * (s_g0 + 1)] = l[1];
            sum += __shfl_xor(sum, 1, 64); // the two threads of a sub-block are neighbours
            if ((threadIdx.x & 1) == 0) lds.xs[s_tok][s_s8] = sum;
        }
        __syncthreads();

        // B operand: sc_s * q as binary16 (exact), lane (row n, columns 8g .. 8g+7 of sub-block s)
        const float d = hdr_d(hdr), dmin = hdr_dmin(hdr);
        half8 B[8];
        float mf[8];
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) {
            const float sc = static_cast<float>(hdr_field(hdr, s8));
            mf[s8] = static_cast<float>(hdr_field(hdr, 8 + s8));
            const uint32_t w = qw[s8];
#pragma unroll
            for (int e = 0; e < 8; ++e) B[s8][e] = static_cast<_Float16>(static_cast<float>((w >> (4 * e)) & 15u) * sc);
        }
#pragma unroll
        for (int tt = 0; tt < GM_TT; ++tt) {
            v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s8 = 0; s8 < 8; ++s8) {
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(lds.hi[tt][s8][lane], B[s8], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(lds.lo[tt][s8][lane], B[s8], acc, 0, 0, 0);
            }
            // this lane: row n, tokens 4g .. 4g+3 of the tile
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 xa = *reinterpret_cast<const float4 *>(&lds.xs[tt * 16 + 4 * g + i][0]);
                const float4 xb = *reinterpret_cast<const float4 *>(&lds.xs[tt * 16 + 4 * g + i][4]);
                float ms = mf[0] * xa.x;
                ms = fmaf(mf[1], xa.y, ms); ms = fmaf(mf[2], xa.z, ms); ms = fmaf(mf[3], xa.w, ms);
                ms = fmaf(mf[4], xb.x, ms); ms = fmaf(mf[5], xb.y, ms); ms = fmaf(mf[6], xb.z, ms); ms = fmaf(mf[7], xb.w, ms);
                yacc[tt][i] += d * acc[i] - dmin * ms;
            }
        }
    }

    const int64_t out_row = static_cast<int64_t>(blockIdx.x) * GM_ROWS + wave * 16 + n;
    if (out_row < a.n_rows) {
#pragma unroll
        for (int tt = 0; tt < GM_TT; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = t0 + tt * 16 + 4 * g + i;
                if (t < a.T) {
                    float v = yacc[tt][i] * a.stat[t].y;
                    if (a.resid) v += a.resid[t * a.ldr + out_row];
                    a.y[t * a.ldy + out_row] = v;
                }
            }
    }
}

} // namespace

size_t gemm_ws_bytes(int T) { return round_up(static_cast<size_t>(T) * sizeof(float2), 256); }

prima_status launch_q4k_gemm(const uint8_t *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int T,
                             const float *gain, float eps, const float *resid, int64_t ldr, float *y, int64_t ldy,
                             void *ws, hipStream_t st, bool scales_ready)
{
    if (n_rows == 0 || T == 0) return PRIMA_OK;
    const int64_t row_blocks = (n_rows + GM_ROWS - 1) / GM_ROWS;
    if (row_blocks >= (int64_t{1} << 31) || (T + GM_TM - 1) / GM_TM > 65535) return PRIMA_E_SHAPE;
    float2 *stat = static_cast<float2 *>(ws);
    // scales_ready: ws holds the scales of these very activations (the call before this one had the same x, gain, eps)
    if (!scales_ready) hipLaunchKernelGGL(gemm_token_scale_kernel, dim3(T), dim3(256), 0, st, x, ldx, n_cols, gain, eps, stat);
    GemmArgs a{W, n_rows, n_cols, x, ldx, gain, stat, resid, ldr, y, ldy, T};
    hipLaunchKernelGGL(q4k_gemm_kernel, dim3(static_cast<unsigned>(row_blocks), static_cast<unsigned>((T + GM_TM - 1) / GM_TM)), dim3(GM_THREADS), 0, st, a);
    return last_launch_status();
}

} // namespace prima
