// Q4_K matrix product for many tokens (prompt processing: the paper reports the time to the first token next to
// the time per output token, Sec. 4.1 / Table 2; the same projections as in decode, App. A.3, for T tokens at once).
//
//     y[t][r] = sum_c W[r][c] * a[t][c],   a = x (or RMSNorm(x; gain)),   + resid[t][r] (optional)
//
// With tens to thousands of tokens the product is a real contraction and belongs on the matrix cores; the decode
// kernel (tokens as int8 digits, sub-scales applied to every MFMA result) spends four multiply-adds per MFMA and
// token group and stops scaling at 8 tokens.  Here:
//   * the B operand is the weight tile itself: per sub-block of 32 weights the integers sc_s * q (at most 945:
//     exact in binary16), built in registers once per super-block and used for every token of the workgroup;
//   * the A operand is the activations as two binary16 numbers hi + lo (22 bits), scaled per token by a power
//     of two so that |a| < 1024; products of two binary16 numbers are exact in fp32, the MFMA adds in fp32;
//   * one accumulator per super-block (256 weights, 8 MFMA steps x 2); the min term sum_s m_s * xs_s (xs_s: the
//     sub-block sums of the scaled activations, again as hi + lo) is one more MFMA step with the m_s as B operand;
//     then  y += d * acc - dmin * acc_m  in fp32.
// Three kernels.  (1) per token: 1/rms (RMSNorm in front) and the power of two.  (2) the activations, split and
// laid out in A-operand order per (16-token tile, super-block): 17 slabs of 1 KiB (8 sub-blocks x (hi, lo), and
// the sums), so that the product kernel moves them into LDS with 16-byte global->LDS loads and no arithmetic; the
// split is done once, not once per row block.  (3) the product: a workgroup of 8 waves owns 256 rows x 128 tokens,
// a wave 32 rows (two B tiles in registers: every A tile read from LDS feeds two MFMAs).  Per super-block the B
// tiles are built once and used for the workgroup's 128 tokens, which pass through LDS in two halves of four token
// tiles (68 KiB each, two buffers): while one half is multiplied the other arrives.  The weights go from global
// memory straight into registers, one super-block ahead.  Workgroups are numbered so that those running on one XCD
// (one L2) at a time are a patch of 8 row blocks x 4 token blocks.  A launch whose workgroups would still fit the
// compute units in one round with 64 tokens each runs only the first half of that loop per workgroup.  Up to three
// matrices with the same columns share a launch (Q / K / V), and so do a gate and an up matrix, with SwiGLU behind.
// The weights stay exact: dequantised to binary16 (one accumulator for all of K) they would be off by ~1e-3 per
// product, measured in the metric of the tests.
#include <hip/hip_fp16.h>

#include "common.h"

namespace prima {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int GM_THREADS = 512;
constexpr int GM_WAVES = GM_THREADS / 64;
constexpr int GM_RT = 2;                        // 16-row tiles per wave
constexpr int GM_TT = 8;                        // 16-token tiles per workgroup
constexpr int GM_HT = GM_TT / 2;                // ... of which one half is in an LDS buffer at a time
constexpr int GM_ROWS = 16 * GM_RT * GM_WAVES;  // rows per workgroup
constexpr int GM_TM = 16 * GM_TT;               // tokens per workgroup
constexpr int GM_SLABS = 17;                    // per (token tile, super-block): 8 sub-blocks x (hi, lo), sums
constexpr int GM_TILE_BYTES = GM_SLABS * 1024;
constexpr int GM_STAGE_BYTES = GM_HT * GM_TILE_BYTES;
constexpr int GM_LDS_BYTES = 2 * GM_STAGE_BYTES; // one workgroup per compute unit
constexpr int GM_XCDS = 8;
constexpr int GM_CUS = 256;
constexpr int GM_PATCH_R = 8, GM_PATCH_C = 4; // row blocks x token blocks that share an XCD at a time
constexpr size_t GM_STAT_ALIGN = 1024;

struct GemmSegDev {
    const uint8_t *W;
    float *y;
    int64_t n_rows, ldy;
    int rb0; // first row block of this matrix (INT_MAX: unused)
};

// Up to three matrices with the same columns against the same activations in one launch (Q / K / V): their row blocks
// are numbered one matrix after the other.  pair: two matrices of equal shape (gate, up); a wave's two row tiles are
// then the same 16 rows of the one and of the other, a row block is 128 rows, and silu(gate) * up is stored to seg[0].y.
struct GemmArgs {
    GemmSegDev seg[3];
    int pair;
    int64_t n_cols;
    const uint8_t *A;   // split activations: [token tile][super-block][17][64 lanes] x 16 bytes
    const float2 *stat; // per token: (2^p [* 1/rms], 2^-p)
    const float *resid; // null: none (added to every stored row; launches with a residual have one matrix)
    int64_t ldr;
    int T, n_tiles, n_rb, n_tb; // 16-token tiles, row blocks, token blocks
    int tiles_wg;               // token tiles of a workgroup: GM_TT, or GM_HT (only its first half) when the grid would not fill the chip
};

// per token: 1/rms (RMSNorm in front) and the power of two that brings max |a| below 1024
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
        int p = 10 - ex;
        p = p > 100 ? 100 : (p < -100 ? -100 : p);
        stat[t] = make_float2(ldexpf(inv_rms, p), ldexpf(1.0f, -p));
    }
}

// The activations of one (16-token tile, super-block) in A-operand order.  Lane (m, g) of an MFMA step holds, for
// token m, the columns 8g .. 8g+7 of a sub-block in the order 0 4 1 5 2 6 3 7 (the order in which the product
// kernel unpacks a dword of eight 4-bit weights into four binary16 pairs).  Tokens past T are zeros.
__global__ void __launch_bounds__(256) gemm_split_kernel(const float *__restrict__ x, int64_t ldx, const float *__restrict__ gain,
                                                         const float2 *__restrict__ stat, int T, int64_t nb, uint8_t *__restrict__ A)
{
    __shared__ float xs[16][8];
    const int64_t b = blockIdx.x;
    const int tile = blockIdx.y;
    const int m = threadIdx.x >> 4, c0 = (threadIdx.x & 15) * 16;
    const int t = tile * 16 + m;
    const bool valid = t < T;
    const int ts = valid ? t : T - 1;
    const float scale = stat[ts].x;
    const float *xp = x + ts * ldx + b * 256 + c0;
    float v[16];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float4 q = *reinterpret_cast<const float4 *>(xp + 4 * i);
        v[4 * i] = q.x; v[4 * i + 1] = q.y; v[4 * i + 2] = q.z; v[4 * i + 3] = q.w;
    }
    if (gain) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float4 q = *reinterpret_cast<const float4 *>(gain + b * 256 + c0 + 4 * i);
            v[4 * i] *= q.x; v[4 * i + 1] *= q.y; v[4 * i + 2] *= q.z; v[4 * i + 3] *= q.w;
        }
    }
    float sum = 0.f;
    _Float16 hh[16], ll[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float sv = valid ? v[i] * scale : 0.f;
        // the product as an opaque fp32 number: left visible, the compiler formed the stored hi from the rounded
        // product and the hi that lo is taken against from the exact one (fused multiply-convert); the two differ
        // now and then by one binary16 step, which lo then does not make up for
        asm volatile("" : "+v"(sv));
        hh[i] = static_cast<_Float16>(sv);
        ll[i] = static_cast<_Float16>(sv - static_cast<float>(hh[i]));
        sum += static_cast<float>(hh[i]) + static_cast<float>(ll[i]); // what the MFMAs will see
    }
    const int s8 = c0 >> 5, g0 = (c0 & 31) >> 3; // sub-block, and the first of this thread's two 8-column groups
    uint8_t *dst = A + (static_cast<int64_t>(tile) * nb + b) * GM_TILE_BYTES;
#pragma unroll
    for (int gi = 0; gi < 2; ++gi) {
        half8 h, l;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int c = 8 * gi + (j & 1) * 4 + (j >> 1);
            h[j] = hh[c];
            l[j] = ll[c];
        }
        *reinterpret_cast<half8 *>(dst + (2 * s8) * 1024 + (m + 16 * (g0 + gi)) * 16) = h;
        *reinterpret_cast<half8 *>(dst + (2 * s8 + 1) * 1024 + (m + 16 * (g0 + gi)) * 16) = l;
    }
    sum += __shfl_xor(sum, 1, 64); // the two threads of a sub-block are neighbours
    if ((threadIdx.x & 1) == 0) xs[m][s8] = sum;
    __syncthreads();
    if (threadIdx.x < 64) { // slab 16: lane (m, 0) the sums' hi parts, lane (m, 1) their lo parts, lanes (m, 2..3) zeros
        const int mm = threadIdx.x & 15, gg = threadIdx.x >> 4;
        half8 o;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float s = xs[mm][j];
            const _Float16 sh = static_cast<_Float16>(s);
            const _Float16 sl = static_cast<_Float16>(s - static_cast<float>(sh));
            o[j] = gg == 0 ? sh : (gg == 1 ? sl : static_cast<_Float16>(0.f));
        }
        *reinterpret_cast<half8 *>(dst + 16 * 1024 + threadIdx.x * 16) = o;
    }
}

__global__ void __launch_bounds__(GM_THREADS) q4k_gemm_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, g = lane >> 4;
    // Consecutive workgroup numbers go to consecutive XCDs.  The 32 workgroups that run on one XCD (one L2) at a time
    // are 8 row blocks x 4 token blocks: per super-block step they fetch 8 x 36 KiB of weights and 4 x 136 KiB of
    // activations between them instead of 32 of either.  An XCD owns the row blocks xcd, xcd + 8, ...
    const int xcd = blockIdx.x % GM_XCDS, seq = blockIdx.x / GM_XCDS;
    const int patch = seq / (GM_PATCH_R * GM_PATCH_C), within = seq % (GM_PATCH_R * GM_PATCH_C);
    const int patches_tb = (a.n_tb + GM_PATCH_C - 1) / GM_PATCH_C;
    const int rb = ((patch / patches_tb) * GM_PATCH_R + within / GM_PATCH_C) * GM_XCDS + xcd;
    const int tb = (patch % patches_tb) * GM_PATCH_C + within % GM_PATCH_C;
    if (rb >= a.n_rb || tb >= a.n_tb) return; // the whole workgroup, before any barrier
    const int64_t nb = a.n_cols >> 8;
    const int sg = a.pair ? 0 : (rb >= a.seg[2].rb0 ? 2 : (rb >= a.seg[1].rb0 ? 1 : 0));
    const GemmSegDev &my = a.seg[sg];
    const int64_t row0 = a.pair ? static_cast<int64_t>(rb) * (GM_ROWS / 2) + wave * 16
                                : static_cast<int64_t>(rb - my.rb0) * GM_ROWS + wave * (16 * GM_RT);
    const uint8_t *wrow[GM_RT];
#pragma unroll
    for (int rt = 0; rt < GM_RT; ++rt) { // past the end: a valid row, not stored
        const int64_t r = min<int64_t>(row0 + (a.pair ? 0 : 16 * rt) + n, my.n_rows - 1);
        wrow[rt] = (a.pair ? a.seg[rt].W : my.W) + r * nb * 144;
    }
    const int tile0 = tb * a.tiles_wg;
    const uint32_t lds0 = lds_address(smem);

    // this wave's share of the 68 slabs of a stage: the token tiles 4 half .. 4 half + 3 of super-block b, into buffer `half`
    auto issue_stage = [&](int64_t b, int half) {
#pragma unroll
        for (int j = 0; j < (GM_HT * GM_SLABS + GM_WAVES - 1) / GM_WAVES; ++j) {
            const int i = wave + GM_WAVES * j;
            if (i < GM_HT * GM_SLABS) {
                const int tt = i / GM_SLABS, sl = i - tt * GM_SLABS;
                const int tile = min(tile0 + GM_HT * half + tt, a.n_tiles - 1); // past the last tile: a valid one, not stored
                const uint8_t *src = a.A + ((static_cast<int64_t>(tile) * nb + b) * GM_SLABS + sl) * 1024 + lane * 16;
                dma16(src, lds0 + half * GM_STAGE_BYTES + i * 1024);
            }
        }
    };
    const bool second_half = a.tiles_wg == GM_TT && tile0 + GM_HT < a.n_tiles; // whether the workgroup has a second half at all
    uint4 hdr[GM_RT];
    uint32_t qw[GM_RT][8];

    v4f yacc[GM_TT][GM_RT];
#pragma unroll
    for (int tt = 0; tt < GM_TT; ++tt)
#pragma unroll
        for (int rt = 0; rt < GM_RT; ++rt) yacc[tt][rt] = {0.f, 0.f, 0.f, 0.f};

    // this lane's place in its rows' current super-block: the header, and its dword of every 16-byte quant chunk
    const uint8_t *hp[GM_RT], *qp[GM_RT];
#pragma unroll
    for (int rt = 0; rt < GM_RT; ++rt) {
        hp[rt] = wrow[rt];
        qp[rt] = wrow[rt] + 16 + 4 * g;
        hdr[rt] = *reinterpret_cast<const uint4 *>(hp[rt]);
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) qw[rt][s8] = *reinterpret_cast<const uint32_t *>(qp[rt] + 16 * s8);
    }

    issue_stage(0, 0);
    uint32_t touch[GM_RT] = {0u, 0u};
    for (int64_t b = 0; b < nb; ++b) {
        // B operands: sc_s * q as binary16 (exact).  A dword holds the eight weights of lane (n, g); masked in pairs
        // (0,4) (1,5) (2,6) (3,7) into the mantissas of 1024 + q, then one fused multiply-add per pair: (1024 + q) sc - 1024 sc
        half8 B[GM_RT][8], Bm[GM_RT];
        float dd[GM_RT], dm[GM_RT];
#pragma unroll
        for (int rt = 0; rt < GM_RT; ++rt) {
            dd[rt] = hdr_d(hdr[rt]);
            dm[rt] = hdr_dmin(hdr[rt]);
#pragma unroll
            for (int s8 = 0; s8 < 8; ++s8) {
                const _Float16 sc = static_cast<_Float16>(static_cast<float>(hdr_field(hdr[rt], s8)));
                const half2v sc2 = {sc, sc};
                const _Float16 off = static_cast<_Float16>(-1024.f) * sc; // exact: at most 64512 in magnitude
                const half2v off2 = {off, off};
                Bm[rt][s8] = static_cast<_Float16>(static_cast<float>(hdr_field(hdr[rt], 8 + s8)));
                const uint32_t w = qw[rt][s8];
#pragma unroll
                for (int pr = 0; pr < 4; ++pr) {
                    const uint32_t bits = ((w >> (4 * pr)) & 0x000f000fu) | 0x64006400u;
                    const half2v r = __builtin_elementwise_fma(__builtin_bit_cast(half2v, bits), sc2, off2);
                    B[rt][s8][2 * pr] = r[0];
                    B[rt][s8][2 * pr + 1] = r[1];
                }
            }
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this half's tiles have landed (this wave's share)
            if (half == 1) asm volatile("" : : "v"(touch[0]), "v"(touch[1])); // (the touches' registers are free again)
            __syncthreads();                                  // everyone's share has, and the other buffer has been read
            if (half == 0) {
                if (second_half) issue_stage(b, 1);
                // the next super-block's weights, into the registers the B tiles were just built from; they have a
                // whole multiplication phase to arrive (the last step loads its own super-block again: in bounds, unused)
                const int step = b + 1 < nb ? 144 : 0;
#pragma unroll
                for (int rt = 0; rt < GM_RT; ++rt) {
                    hp[rt] += step;
                    qp[rt] += step;
                    hdr[rt] = *reinterpret_cast<const uint4 *>(hp[rt]);
#pragma unroll
                    for (int s8 = 0; s8 < 8; ++s8) qw[rt][s8] = *reinterpret_cast<const uint32_t *>(qp[rt] + 16 * s8);
                    // and one dword of the super-block three further on (the four lanes of a row between them touch
                    // all of its 144 bytes): the rows are read nowhere else, so without this every weight load waits
                    // for HBM; with it the loads above find their lines in the L2
                    touch[rt] = b + 4 < nb ? *reinterpret_cast<const uint32_t *>(hp[rt] + 3 * 144 + min(48 * g, 140)) : 0u;
                }
            } else if (b + 1 < nb) {
                issue_stage(b + 1, 0);
            }
            if (half == 1 && !second_half) continue;
            const uint8_t *stage = smem + half * GM_STAGE_BYTES;
#pragma unroll
            for (int ht = 0; ht < GM_HT; ++ht) {
                const int tt = GM_HT * half + ht;
                const half8 *At = reinterpret_cast<const half8 *>(stage + ht * GM_TILE_BYTES);
                v4f acc[GM_RT];
#pragma unroll
                for (int rt = 0; rt < GM_RT; ++rt) acc[rt] = {0.f, 0.f, 0.f, 0.f};
                // The lo parts first: their sums are 2^-11 of the hi parts', so the fp32 roundings of the first eight
                // steps do not count and only the eight hi steps round at the accumulator's full magnitude.
#pragma unroll
                for (int s8 = 0; s8 < 8; ++s8) {
                    const half8 al = At[(2 * s8 + 1) * 64 + lane];
#pragma unroll
                    for (int rt = 0; rt < GM_RT; ++rt) acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(al, B[rt][s8], acc[rt], 0, 0, 0);
                }
#pragma unroll
                for (int s8 = 0; s8 < 8; ++s8) {
                    const half8 ah = At[(2 * s8) * 64 + lane];
#pragma unroll
                    for (int rt = 0; rt < GM_RT; ++rt) acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ah, B[rt][s8], acc[rt], 0, 0, 0);
                }
                const half8 ax = At[16 * 64 + lane];
#pragma unroll
                for (int rt = 0; rt < GM_RT; ++rt) {
                    const v4f zero = {0.f, 0.f, 0.f, 0.f};
                    const v4f am = __builtin_amdgcn_mfma_f32_16x16x32_f16(ax, Bm[rt], zero, 0, 0, 0);
                    // this lane: row n of row tile rt, tokens 4g .. 4g+3 of the tile.  The super-block's term is formed
                    // first, at its own magnitude, and added in one step: one rounding per super-block at the magnitude
                    // of the running sum (the chain of these roundings is the larger part of the product's error)
#pragma unroll
                    for (int i = 0; i < 4; ++i) yacc[tt][rt][i] += fmaf(dd[rt], acc[rt][i], -(dm[rt] * am[i]));
                }
            }
        }
    }

    if (a.pair) {
        const int64_t out_row = row0 + n;
        if (out_row < my.n_rows) {
#pragma unroll
            for (int tt = 0; tt < GM_TT; ++tt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int t = (tile0 + tt) * 16 + 4 * g + i;
                    if (tt < a.tiles_wg && t < a.T) {
                        const float sc = a.stat[t].y;
                        const float gt = yacc[tt][0][i] * sc, up = yacc[tt][1][i] * sc;
                        my.y[t * my.ldy + out_row] = gt / (1.0f + expf(-gt)) * up;
                    }
                }
        }
        return;
    }
#pragma unroll
    for (int rt = 0; rt < GM_RT; ++rt) {
        const int64_t out_row = row0 + 16 * rt + n;
        if (out_row >= my.n_rows) continue;
#pragma unroll
        for (int tt = 0; tt < GM_TT; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = (tile0 + tt) * 16 + 4 * g + i;
                if (tt < a.tiles_wg && t < a.T) {
                    float v = yacc[tt][rt][i] * a.stat[t].y;
                    if (a.resid) v += a.resid[t * a.ldr + out_row];
                    my.y[t * my.ldy + out_row] = v;
                }
            }
    }
}

} // namespace

size_t gemm_ws_bytes(int T, int64_t n_cols)
{
    const size_t tiles = (static_cast<size_t>(T) + 15) / 16;
    return round_up(static_cast<size_t>(T) * sizeof(float2), GM_STAT_ALIGN) + tiles * static_cast<size_t>(n_cols / QK) * GM_TILE_BYTES;
}

prima_status launch_q4k_gemm_multi(const GemmMat *mats, int n_mats, bool pair, int64_t n_cols, const float *x, int64_t ldx, int T,
                                   const float *gain, float eps, const float *resid, int64_t ldr, void *ws, hipStream_t st, bool split_ready)
{
    if (n_mats < 1 || n_mats > 3 || (pair && (n_mats != 2 || mats[0].n_rows != mats[1].n_rows || resid))) return PRIMA_E_SHAPE;
    if (T == 0) return PRIMA_OK;
    GemmArgs a{};
    int64_t n_rb = 0;
    for (int i = 0; i < 3; ++i) {
        a.seg[i].rb0 = 0x7fffffff;
        if (i >= n_mats || mats[i].n_rows == 0 || (pair && i == 1)) {
            if (i < n_mats) a.seg[i] = GemmSegDev{mats[i].W, mats[i].y, mats[i].n_rows, mats[i].ldy, 0x7fffffff};
            continue;
        }
        a.seg[i] = GemmSegDev{mats[i].W, mats[i].y, mats[i].n_rows, mats[i].ldy, static_cast<int>(n_rb)};
        n_rb += pair ? (mats[i].n_rows + GM_ROWS / 2 - 1) / (GM_ROWS / 2) : (mats[i].n_rows + GM_ROWS - 1) / GM_ROWS;
        if (n_rb >= (int64_t{1} << 30)) return PRIMA_E_SHAPE;
    }
    if (n_rb == 0) return PRIMA_OK;
    const int64_t nb = n_cols / QK;
    // 128 tokens per workgroup; 64 when the workgroups then still fit the compute units in one round (a workgroup with
    // one half takes ~0.63 of the time of one with two; 8192 x 28672 at 512 tokens: 1138 -> 801 us)
    const int n_tiles = (T + 15) / 16;
    const int tiles_wg = n_rb * ((T + GM_TM / 2 - 1) / (GM_TM / 2)) <= GM_CUS ? GM_HT : GM_TT;
    const int n_tb = (n_tiles + tiles_wg - 1) / tiles_wg;
    const int64_t rb_per_xcd = (n_rb + GM_XCDS - 1) / GM_XCDS;
    const int64_t grid = (rb_per_xcd + GM_PATCH_R - 1) / GM_PATCH_R * ((n_tb + GM_PATCH_C - 1) / GM_PATCH_C) * (GM_PATCH_R * GM_PATCH_C) * GM_XCDS;
    if (grid >= (int64_t{1} << 31) || n_tiles > 65535 || nb >= (int64_t{1} << 31)) return PRIMA_E_SHAPE;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(q4k_gemm_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, GM_LDS_BYTES) != hipSuccess)
            return PRIMA_E_DEVICE;
        attr_set = true;
    }
    float2 *stat = static_cast<float2 *>(ws);
    uint8_t *A = static_cast<uint8_t *>(ws) + round_up(static_cast<size_t>(T) * sizeof(float2), GM_STAT_ALIGN);
    // split_ready: ws holds the split of these very activations (the call before this one had the same x, gain, eps, T)
    if (!split_ready) {
        hipLaunchKernelGGL(gemm_token_scale_kernel, dim3(T), dim3(256), 0, st, x, ldx, n_cols, gain, eps, stat);
        hipLaunchKernelGGL(gemm_split_kernel, dim3(static_cast<unsigned>(nb), n_tiles), dim3(256), 0, st, x, ldx, gain, stat, T, nb, A);
    }
    a.pair = pair ? 1 : 0;
    a.n_cols = n_cols; a.A = A; a.stat = stat; a.resid = resid; a.ldr = ldr;
    a.T = T; a.n_tiles = n_tiles; a.n_rb = static_cast<int>(n_rb); a.n_tb = n_tb; a.tiles_wg = tiles_wg;
    hipLaunchKernelGGL(q4k_gemm_kernel, dim3(static_cast<unsigned>(grid)), dim3(GM_THREADS), GM_LDS_BYTES, st, a);
    return last_launch_status();
}

prima_status launch_q4k_gemm(const uint8_t *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int T,
                             const float *gain, float eps, const float *resid, int64_t ldr, float *y, int64_t ldy,
                             void *ws, hipStream_t st, bool split_ready)
{
    const GemmMat m{W, y, n_rows, ldy};
    return launch_q4k_gemm_multi(&m, 1, false, n_cols, x, ldx, T, gain, eps, resid, ldr, ws, st, split_ready);
}

} // namespace prima
