// Dequant-fused Q4_K mat-vec on the matrix cores with exact integer accumulation (gfx950).
//
// The weight stream (the b bytes per layer of arXiv 2504.08791, App. A.3) is what bounds decode;
// the arithmetic has to hide behind it.  At 8 TB/s a CU receives ~26 four-bit weights per clock
// but its vector ALUs issue 64 lane-operations per clock, so a multiply-add per weight per token
// plus the nibble unpacking does not fit.  The multiply-adds run on the MFMA units instead:
//
//  * each activation vector is turned into block fixed point once per mat-vec: x = xfix * 2^-p,
//    |xfix| < 2^30, split into four signed 8-bit digits (xfix = sum_r digit_r * 256^r);
//  * a wave owns 16 output rows; lane (j, g) = (lane % 16, lane / 16) loads the 16-byte quant
//    chunk of row j, sub-block s0+g (128-bit loads; one instruction covers 16 rows x 64 B), splits
//    it into two int8 vectors with three ALU ops per 8 weights, and feeds them as the B operand of
//    v_mfma_i32_16x16x32_i8;
//  * the A operand holds the digits, arranged block-diagonally: output slot 4g'+r carries digit r
//    restricted to k-group g'.  The MFMA result on lane (j, g) is then exactly the four digit
//    sums of row j with *its own* sub-block s0+g: sum_k q_k * digit_r(x_k);
//  * the 6-bit sub-scale multiplies these integers (still exact), the four digits are recombined
//    in fp32, and d (fp16) scales the super-block.  The min term uses per-sub-block sums of xfix:
//        y = 2^-p * sum_blocks [ d * sum_s sc_s * (q . xfix)_s  -  dmin * sum_s m_s * Xsum_s ].
//    For T tokens the unpacked weights are reused against each token's digits.
//
// Launch shape: one 1024-thread workgroup per compute unit, persistent.  Each workgroup owns a
// contiguous range of 16-row tiles with all of K, so no result crosses workgroups and every sum
// has a fixed order (bit-reproducible).  The activations are transformed (RMSNorm or SwiGLU when
// asked), quantised and laid out in LDS by every workgroup for itself; the 16 waves then stream
// (tile, K-piece) units, three super-blocks of loads in flight per wave, and leave per-unit
// partial sums in LDS that the epilogue adds in piece order.
#include "common.h"

namespace prima {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int SUB_LDS = 144;   // bytes of LDS per sub-block of digits: 4 digits x 32 B + 16 B skew
constexpr int MAX_WAVES = 16;
// workgroup size: 16 waves leave 128 VGPRs per lane, enough for up to 4 tokens' accumulators next to
// the three load stages; 5..8 tokens run 8 waves with 256 VGPRs
constexpr int threads_for(int tt) { return tt <= 4 ? 1024 : 512; }
constexpr size_t LDS_BUDGET = 160 * 1024;

struct PGemvArgs {
    GemvSeg seg[3];
    int seg_tile0[3]; // first 16-row tile of each segment
    int nseg, n_tiles, nb, T;
    // activations
    int xmode;
    const float *x, *x2, *gain;
    int64_t ldx;
    float eps;
    float *x_tap; // optional [T][K]: transformed fp32 activations (written by workgroup 0)
    // decomposition
    int pb;          // super-blocks per unit (K-piece)
    int ppt;         // pieces per tile
    int pps;         // pieces per slab
    int n_slabs;     // K slabs staged in LDS one after the other
    int units_cap;   // partial-sum slots per workgroup
    int n_wg;
};

struct BlockRegs {
    uint4 hdr, qa, qb;
};

__device__ __forceinline__ void load_block(BlockRegs &r, const uint4 *bp, int g)
{
    r.hdr = bp[0];
    r.qa = bp[1 + g];
    r.qb = bp[5 + g];
}

__device__ __forceinline__ long pack64(uint32_t lo, uint32_t hi)
{
    return static_cast<long>(static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32));
}

template <int GEMV_WAVES>
__device__ __forceinline__ float wg_reduce(float v, float *red, bool is_max)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(v, off, 64);
        v = is_max ? fmaxf(v, o) : v + o;
    }
    __syncthreads(); // red may still be read from the previous use
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
#pragma unroll
    for (int i = 1; i < GEMV_WAVES; ++i) r = is_max ? fmaxf(r, red[i]) : r + red[i]; // fixed order
    return r;
}

// eight consecutive transformed activations of token t starting at column c0
__device__ __forceinline__ void load_act8(const PGemvArgs &a, int t, int c0, float inv_rms, float *f)
{
    const float *xp = a.x + t * a.ldx + c0;
    const float4 v0 = *reinterpret_cast<const float4 *>(xp), v1 = *reinterpret_cast<const float4 *>(xp + 4);
    f[0] = v0.x; f[1] = v0.y; f[2] = v0.z; f[3] = v0.w; f[4] = v1.x; f[5] = v1.y; f[6] = v1.z; f[7] = v1.w;
    if (a.xmode == X_RMSNORM) {
        const float4 g0 = *reinterpret_cast<const float4 *>(a.gain + c0), g1 = *reinterpret_cast<const float4 *>(a.gain + c0 + 4);
        const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = f[e] * inv_rms * gg[e];
    } else if (a.xmode == X_SWIGLU) {
        const float *up = a.x2 + t * a.ldx + c0;
        const float4 u0 = *reinterpret_cast<const float4 *>(up), u1 = *reinterpret_cast<const float4 *>(up + 4);
        const float uu[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = f[e] / (1.0f + expf(-f[e])) * uu[e];
    }
}

template <int TT>
__global__ void __launch_bounds__(threads_for(TT)) gemv_q4k_persistent_kernel(PGemvArgs a)
{
    constexpr int GEMV_THREADS = threads_for(TT);
    constexpr int GEMV_WAVES = GEMV_THREADS / 64;
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int K = a.nb * QK;

    // tiles of this workgroup
    const int tl0 = static_cast<int>(static_cast<int64_t>(a.n_tiles) * blockIdx.x / a.n_wg);
    const int tl1 = static_cast<int>(static_cast<int64_t>(a.n_tiles) * (blockIdx.x + 1) / a.n_wg);
    const int ntl = tl1 - tl0;
    if (ntl == 0) return;

    // LDS carve: digits [TT][slab_sub][SUB_LDS] | zeros 32 B | xsum [TT][slab_sub] | partial [units_cap][TT][16] | red[16] | stats
    const int slab_blocks = a.pps * a.pb;
    const int slab_sub = slab_blocks * 8;
    uint8_t *l_dig = smem;
    const int dig_t_stride = slab_sub * SUB_LDS;
    const int zero_off = TT * dig_t_stride;
    float *l_xs = reinterpret_cast<float *>(smem + zero_off + 32);
    float *l_part = l_xs + TT * slab_sub;
    float *l_red = l_part + a.units_cap * TT * 16;
    float *l_scale = l_red + MAX_WAVES;   // [TT] 2^p
    float *l_inv = l_scale + TT;           // [TT] 2^-p
    float *l_rms = l_inv + TT;             // [TT] 1/rms

    if (threadIdx.x < 8) reinterpret_cast<uint32_t *>(smem + zero_off)[threadIdx.x] = 0u;

    // ---- statistics of the activations: 1/rms (RMSNorm input) and the power-of-two scale ----
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        float inv_rms = 1.f;
        if (a.xmode == X_RMSNORM) {
            float ss = 0.f;
            for (int gi = threadIdx.x; gi < K / 8; gi += GEMV_THREADS) {
                const float *xp = a.x + t * a.ldx + gi * 8;
                const float4 v0 = *reinterpret_cast<const float4 *>(xp), v1 = *reinterpret_cast<const float4 *>(xp + 4);
                ss += ((v0.x * v0.x + v0.y * v0.y) + (v0.z * v0.z + v0.w * v0.w)) + ((v1.x * v1.x + v1.y * v1.y) + (v1.z * v1.z + v1.w * v1.w));
            }
            ss = wg_reduce<GEMV_WAVES>(ss, l_red, false);
            inv_rms = 1.0f / sqrtf(ss / static_cast<float>(K) + a.eps);
        }
        float amax = 0.f;
        for (int gi = threadIdx.x; gi < K / 8; gi += GEMV_THREADS) {
            float f[8];
            load_act8(a, t, gi * 8, inv_rms, f);
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(f[e]));
        }
        amax = wg_reduce<GEMV_WAVES>(amax, l_red, true);
        int ex = 0;
        if (amax > 0.f) frexpf(amax, &ex); // amax = m * 2^ex, m in [0.5, 1)  ->  |x| * 2^(30-ex) < 2^30
        int p = 30 - ex;
        p = p > 120 ? 120 : p;
        if (threadIdx.x == 0) {
            l_scale[t] = ldexpf(1.0f, p);
            l_inv[t] = ldexpf(1.0f, -p);
            l_rms[t] = inv_rms;
        }
    }
    __syncthreads();

    // lanes whose output slots hold this lane's k-group carry digits; all others feed zeros
    const bool active = (j >> 2) == g;
    const int a_base = active ? g * SUB_LDS + (j & 3) * 32 : zero_off;
    const int a_step = active ? SUB_LDS : 0;
    const int a_tstep = active ? dig_t_stride : 0;
    const int fsh = 6 * g;
    const int64_t pitch16 = static_cast<int64_t>(a.nb) * 9; // row pitch in 16-byte units

    for (int slab = 0; slab < a.n_slabs; ++slab) {
        const int p0 = slab * a.pps;                       // first piece of the slab
        const int p1 = min(p0 + a.pps, a.ppt);
        const int sb0 = p0 * a.pb;                         // first super-block of the slab
        const int sb1 = min(p1 * a.pb, a.nb);
        if (slab > 0) __syncthreads();                     // previous slab's digits no longer in use

        // ---- transform + quantise this slab's activations into LDS ----
        // digits [S][4][32 bytes]; byte order inside a digit row: for each group a of 8 values,
        // values 8a + {0,2,4,6,1,3,5,7}, the order in which the nibble split delivers the weights.
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const float S = l_scale[t], inv_rms = l_rms[t];
            for (int gi = sb0 * 32 + threadIdx.x; gi < sb1 * 32; gi += GEMV_THREADS) {
                float f[8];
                load_act8(a, t, gi * 8, inv_rms, f);
                if (a.x_tap && blockIdx.x == 0) {
                    float *tp = a.x_tap + static_cast<int64_t>(t) * K + gi * 8;
                    *reinterpret_cast<float4 *>(tp) = make_float4(f[0], f[1], f[2], f[3]);
                    *reinterpret_cast<float4 *>(tp + 4) = make_float4(f[4], f[5], f[6], f[7]);
                }
                int r[8];
                long long sum = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    r[e] = static_cast<int>(rintf(f[e] * S)); // power-of-two scaling is exact; one rounding to integer
                    sum += r[e];
                }
                const int s_loc = (gi >> 2) - sb0 * 8, grp = gi & 3;
                uint8_t *dp = l_dig + t * dig_t_stride + s_loc * SUB_LDS + grp * 8;
#pragma unroll
                for (int dg = 0; dg < 4; ++dg) {
                    uint32_t by[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int lowb = static_cast<int>(static_cast<int8_t>(r[e] & 255)); // signed low byte
                        by[e] = static_cast<uint32_t>(lowb) & 255u;
                        r[e] = (r[e] - lowb) >> 8;
                    }
                    uint2 o;
                    o.x = by[0] | (by[2] << 8) | (by[4] << 16) | (by[6] << 24);
                    o.y = by[1] | (by[3] << 8) | (by[5] << 16) | (by[7] << 24);
                    *reinterpret_cast<uint2 *>(dp + dg * 32) = o;
                }
                sum += __shfl_xor(sum, 1, 64);
                sum += __shfl_xor(sum, 2, 64);
                if (grp == 0) l_xs[t * slab_sub + s_loc] = static_cast<float>(sum);
            }
        }
        __syncthreads();

        // ---- stream the (tile, piece) units of this slab ----
        const int pps_here = p1 - p0;
        const int n_units = ntl * pps_here;

        struct Cursor {
            int k, b, b_end, tile_local, piece;
            const uint4 *rowp;
        };
        auto seek = [&](Cursor &c) { // position on unit c.k (must be < n_units)
            c.tile_local = c.k / pps_here;
            c.piece = p0 + (c.k - c.tile_local * pps_here);
            c.b = c.piece * a.pb;
            c.b_end = min(c.b + a.pb, sb1);
            const int tile = tl0 + c.tile_local;
            int sg = 0;
            while (sg + 1 < a.nseg && tile >= a.seg_tile0[sg + 1]) ++sg;
            const int64_t row = static_cast<int64_t>(tile - a.seg_tile0[sg]) * 16 + j;
            const int64_t row_ld = row < a.seg[sg].n_rows ? row : a.seg[sg].n_rows - 1; // rows past the end re-read the last row
            c.rowp = reinterpret_cast<const uint4 *>(a.seg[sg].W) + row_ld * pitch16;
        };
        auto advance = [&](Cursor &c) { // next super-block of this wave's stream; sticks on the last one
            if (c.b + 1 < c.b_end) { ++c.b; return; }
            if (c.k + GEMV_WAVES < n_units) { c.k += GEMV_WAVES; seek(c); }
        };

        if (wave < n_units) {
            float yacc[TT], macc[TT];
#pragma unroll
            for (int t = 0; t < TT; ++t) { yacc[t] = 0.f; macc[t] = 0.f; }

            // one super-block against all tokens: 8 MFMAs per token + integer sub-scales + fp32 recombination
            auto compute = [&](const BlockRegs &c, int b) {
                const uint32_t w[8] = {c.qa.x, c.qa.y, c.qa.z, c.qa.w, c.qb.x, c.qb.y, c.qb.z, c.qb.w};
                long B[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) B[i] = pack64(w[i] & 0x0f0f0f0fu, (w[i] >> 4) & 0x0f0f0f0fu); // weights 8i+{0,2,4,6 | 1,3,5,7}
                const int sc0 = static_cast<int>(__builtin_amdgcn_ubfe(c.hdr.y, fsh, 6));
                const int sc1 = static_cast<int>(__builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(c.hdr.z, c.hdr.y, 24), fsh, 6));
                const float m0 = static_cast<float>(__builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(c.hdr.w, c.hdr.z, 16), fsh, 6));
                const float m1 = static_cast<float>(__builtin_amdgcn_ubfe(c.hdr.w, 8 + fsh, 6));
                const float d = hdr_d(c.hdr), dmin = hdr_dmin(c.hdr);
                const int s_loc = (b - sb0) * 8;
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    const uint8_t *ap = l_dig + a_base + t * a_tstep + s_loc * a_step;
                    const uint4 x0 = *reinterpret_cast<const uint4 *>(ap);
                    const uint4 x1 = *reinterpret_cast<const uint4 *>(ap + 16);
                    const uint4 x2 = *reinterpret_cast<const uint4 *>(ap + 4 * a_step);
                    const uint4 x3 = *reinterpret_cast<const uint4 *>(ap + 4 * a_step + 16);
                    v4i d0 = {0, 0, 0, 0}, d1 = {0, 0, 0, 0};
                    d0 = __builtin_amdgcn_mfma_i32_16x16x32_i8(pack64(x0.x, x0.y), B[0], d0, 0, 0, 0);
                    d1 = __builtin_amdgcn_mfma_i32_16x16x32_i8(pack64(x2.x, x2.y), B[4], d1, 0, 0, 0);
                    d0 = __builtin_amdgcn_mfma_i32_16x16x32_i8(pack64(x0.z, x0.w), B[1], d0, 0, 0, 0);
                    d1 = __builtin_amdgcn_mfma_i32_16x16x32_i8(pack64(x2.z, x2.w), B[5], d1, 0, 0, 0);
                    d0 = __builtin_amdgcn_mfma_i32_16x16x32_i8(pack64(x1.x, x1.y), B[2], d0, 0, 0, 0);
                    d1 = __builtin_amdgcn_mfma_i32_16x16x32_i8(pack64(x3.x, x3.y), B[6], d1, 0, 0, 0);
                    d0 = __builtin_amdgcn_mfma_i32_16x16x32_i8(pack64(x1.z, x1.w), B[3], d0, 0, 0, 0);
                    d1 = __builtin_amdgcn_mfma_i32_16x16x32_i8(pack64(x3.z, x3.w), B[7], d1, 0, 0, 0);
                    const int i0 = __mul24(d0[0], sc0) + __mul24(d1[0], sc1);
                    const int i1 = __mul24(d0[1], sc0) + __mul24(d1[1], sc1);
                    const int i2 = __mul24(d0[2], sc0) + __mul24(d1[2], sc1);
                    const int i3 = __mul24(d0[3], sc0) + __mul24(d1[3], sc1);
                    float f = static_cast<float>(i3);
                    f = fmaf(f, 256.f, static_cast<float>(i2));
                    f = fmaf(f, 256.f, static_cast<float>(i1));
                    f = fmaf(f, 256.f, static_cast<float>(i0));
                    yacc[t] = fmaf(d, f, yacc[t]);
                    const float *xs = l_xs + t * slab_sub + s_loc;
                    macc[t] = fmaf(dmin, fmaf(m0, xs[g], m1 * xs[4 + g]), macc[t]);
                }
            };
            // leave the unit's sums in its LDS slot: [unit][t][row]
            auto flush = [&](const Cursor &c) {
                float *slot = l_part + (c.tile_local * a.ppt + c.piece) * (TT * 16);
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    float v = yacc[t] - macc[t];
                    v += __shfl_xor(v, 16, 64);
                    v += __shfl_xor(v, 32, 64);
                    if (g == 0) slot[t * 16 + j] = v;
                    yacc[t] = 0.f;
                    macc[t] = 0.f;
                }
            };

            Cursor cc, lc; // compute cursor and load cursor (two super-blocks ahead)
            cc.k = wave;
            seek(cc);
            lc = cc;
            BlockRegs r0, r1, r2;
            load_block(r0, lc.rowp + lc.b * 9, g);
            advance(lc);
            load_block(r1, lc.rowp + lc.b * 9, g);
            advance(lc);
            // blocks this wave computes in the slab
            int remaining = 0;
            for (int k = wave; k < n_units; k += GEMV_WAVES) {
                const int piece = p0 + k % pps_here;
                remaining += min(piece * a.pb + a.pb, sb1) - piece * a.pb;
            }
            auto step = [&](BlockRegs &use, BlockRegs &refill) {
                load_block(refill, lc.rowp + lc.b * 9, g);
                advance(lc);
                compute(use, cc.b);
                if (cc.b + 1 == cc.b_end) {
                    flush(cc);
                    if (cc.k + GEMV_WAVES < n_units) { cc.k += GEMV_WAVES; seek(cc); }
                } else {
                    ++cc.b;
                }
                --remaining;
            };
            while (remaining > 0) {
                step(r0, r2);
                if (remaining > 0) step(r1, r0);
                if (remaining > 0) step(r2, r1);
            }
        }
    }
    __syncthreads();

    // ---- epilogue: add the pieces of every (tile, row, token) in piece order, scale, residual, store ----
    for (int idx = threadIdx.x; idx < ntl * 16 * TT; idx += GEMV_THREADS) {
        const int tile_local = idx / (16 * TT);
        const int rem = idx - tile_local * (16 * TT);
        const int t = rem >> 4, jj = rem & 15;
        float v = 0.f;
        for (int p = 0; p < a.ppt; ++p) v += l_part[(tile_local * a.ppt + p) * (TT * 16) + t * 16 + jj];
        const int tile = tl0 + tile_local;
        int sg = 0;
        while (sg + 1 < a.nseg && tile >= a.seg_tile0[sg + 1]) ++sg;
        const int64_t row = static_cast<int64_t>(tile - a.seg_tile0[sg]) * 16 + jj;
        if (row < a.seg[sg].n_rows) {
            v *= l_inv[t];
            if (a.seg[sg].resid) v += a.seg[sg].resid[t * a.seg[sg].ldr + row];
            a.seg[sg].y[t * a.seg[sg].ldy + row] = v;
        }
    }
}

// ------------------------------------------------------------------------------------------
struct PPlan {
    int n_tiles, nb, n_wg, pb, ppt, pps, n_slabs, units_cap;
    size_t lds_bytes;
    bool ok;
};

static int device_cu_count()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

static size_t plan_lds(int T, int slab_blocks, int units_cap)
{
    return static_cast<size_t>(T) * slab_blocks * 8 * SUB_LDS + 32 + static_cast<size_t>(T) * slab_blocks * 8 * 4 +
           static_cast<size_t>(units_cap) * T * 16 * 4 + (MAX_WAVES + 3 * T) * 4 + 64;
}

static PPlan plan_persistent(const GemvArgs &ga, int T)
{
    PPlan p{};
    p.nb = static_cast<int>(ga.n_cols / QK);
    p.n_tiles = 0;
    for (int i = 0; i < ga.nseg; ++i) p.n_tiles += static_cast<int>((ga.seg[i].n_rows + 15) / 16);
    p.n_wg = device_cu_count();
    if (p.n_wg > p.n_tiles) p.n_wg = p.n_tiles;
    const int tiles_wg = (p.n_tiles + p.n_wg - 1) / p.n_wg;
    // super-blocks per unit: spread a workgroup's super-blocks over its 16 waves, 2..16 per unit
    int pb = tiles_wg * p.nb / (threads_for(T) / 64);
    pb = pb < 2 ? 2 : (pb > 16 ? 16 : pb);
    if (pb > p.nb) pb = p.nb;
    p.ppt = (p.nb + pb - 1) / pb;
    p.pb = (p.nb + p.ppt - 1) / p.ppt;
    p.ppt = (p.nb + p.pb - 1) / p.pb;
    p.units_cap = tiles_wg * p.ppt;
    // pieces per slab: as many as fit in LDS
    p.pps = p.ppt;
    while (p.pps > 1 && plan_lds(T, p.pps * p.pb, p.units_cap) > LDS_BUDGET) --p.pps;
    p.n_slabs = (p.ppt + p.pps - 1) / p.pps;
    p.lds_bytes = plan_lds(T, p.pps * p.pb, p.units_cap);
    p.ok = p.lds_bytes <= LDS_BUDGET;
    return p;
}

template <int TT>
static hipError_t launch_tt(const PGemvArgs &a, const PPlan &p, hipStream_t st)
{
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemv_q4k_persistent_kernel<TT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(LDS_BUDGET));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(gemv_q4k_persistent_kernel<TT>, dim3(p.n_wg), dim3(threads_for(TT)), p.lds_bytes, st, a);
    return hipGetLastError();
}

size_t gemv_mfma_ws_bytes(int64_t, int64_t, int) { return 256; }

prima_status launch_gemv_mfma(const GemvArgs &ga, hipStream_t st)
{
    // up to 8 tokens per pass over the weights
    for (int t0 = 0; t0 < ga.T; t0 += 8) {
        const int T = ga.T - t0 < 8 ? ga.T - t0 : 8;
        const PPlan p = plan_persistent(ga, T);
        if (!p.ok) return PRIMA_E_SHAPE;
        PGemvArgs a{};
        int tile0 = 0;
        for (int i = 0; i < ga.nseg; ++i) {
            a.seg[i] = ga.seg[i];
            a.seg[i].y += t0 * ga.seg[i].ldy;
            if (a.seg[i].resid) a.seg[i].resid += t0 * ga.seg[i].ldr;
            a.seg_tile0[i] = tile0;
            tile0 += static_cast<int>((ga.seg[i].n_rows + 15) / 16);
        }
        a.nseg = ga.nseg;
        a.n_tiles = p.n_tiles;
        a.nb = p.nb;
        a.T = T;
        a.xmode = ga.xmode;
        a.x = ga.x + t0 * ga.ldx;
        a.x2 = ga.x2 ? ga.x2 + t0 * ga.ldx : nullptr;
        a.gain = ga.gain;
        a.ldx = ga.ldx;
        a.eps = ga.eps;
        a.x_tap = ga.x_tap ? ga.x_tap + static_cast<int64_t>(t0) * ga.n_cols : nullptr;
        a.pb = p.pb;
        a.ppt = p.ppt;
        a.pps = p.pps;
        a.n_slabs = p.n_slabs;
        a.units_cap = p.units_cap;
        a.n_wg = p.n_wg;
        hipError_t e;
        switch (T) {
        case 1: e = launch_tt<1>(a, p, st); break;
        case 2: e = launch_tt<2>(a, p, st); break;
        case 3: e = launch_tt<3>(a, p, st); break;
        case 4: e = launch_tt<4>(a, p, st); break;
        case 5: e = launch_tt<5>(a, p, st); break;
        case 6: e = launch_tt<6>(a, p, st); break;
        case 7: e = launch_tt<7>(a, p, st); break;
        default: e = launch_tt<8>(a, p, st); break;
        }
        if (e != hipSuccess) return PRIMA_E_DEVICE;
    }
    return PRIMA_OK;
}

} // namespace prima
