// Single-token Q4_K mat-vec on the matrix cores with exact integer accumulation (gfx950).
//
// The weight stream (the b bytes per layer of arXiv 2504.08791, App. A.3) is what bounds decode;
// the arithmetic has to hide behind it.  At 8 TB/s a CU receives ~26 four-bit weights per clock
// but its vector ALUs issue 64 lane-operations per clock, so a multiply-add per weight plus the
// nibble unpacking does not fit.  Here the multiply-adds run on the MFMA units instead:
//
//  * the activation vector is turned into block fixed point once per mat-vec: x = xfix * 2^-p,
//    |xfix| < 2^30, split into four signed 8-bit digits (xfix = sum_r digit_r * 256^r);
//  * a wave owns 16 output rows; lane (j, g) = (lane % 16, lane / 16) loads the 16-byte quant
//    chunk of row j, sub-block s0+g (128-bit loads; each instruction covers 16 rows x 64 B), splits
//    it into two int8 vectors with three ALU ops per 8 weights, and feeds them as the B operand of
//    v_mfma_i32_16x16x32_i8;
//  * the A operand holds the digits, arranged block-diagonally: output slot 4g'+r carries digit r
//    restricted to k-group g'.  The MFMA result on lane (j, g) is then exactly the four digit
//    sums of row j with *its own* sub-block s0+g: sum_k q_k * digit_r(x_k);
//  * the 6-bit sub-scale multiplies these integers (still exact), the four digits are recombined
//    in fp32, and d (fp16) scales the super-block.  The min term uses per-sub-block sums of xfix:
//        y = 2^-p * sum_blocks [ d * sum_s sc_s * (q . xfix)_s  -  dmin * sum_s m_s * Xsum_s ].
//
// Nothing is rounded until the fp32 recombination, so the product is accurate to fp32 level
// independent of the dynamic range of x.
#include "common.h"

namespace prima {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int SUB_LDS = 144; // bytes of LDS per sub-block of digits: 4 digits x 32 B + 16 B skew

// ------------------------------------------------------------------------------------------
// x (fp32) -> digits [S][4][32 bytes] (128 B per sub-block of 32 values), Xsum[S], 2^-p.
// Byte order inside a digit row: for each group a of 8 values, values 8a + {0,2,4,6,1,3,5,7}:
// the order in which the nibble split below delivers the weights.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
quantize_x_kernel(const float *__restrict__ x, int64_t ldx, int K, uint8_t *__restrict__ dig, float *__restrict__ xsum,
                  float *__restrict__ inv_scale, int64_t dig_stride, int64_t xs_stride)
{
    __shared__ float red[16];
    const int t = blockIdx.x;
    const float *xt = x + t * ldx;
    float amax = 0.f;
    for (int i = threadIdx.x * 4; i < K; i += blockDim.x * 4) {
        const float4 v = *reinterpret_cast<const float4 *>(xt + i);
        amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = amax;
    __syncthreads();
    amax = 0.f;
    for (int i = 0; i < static_cast<int>(blockDim.x >> 6); ++i) amax = fmaxf(amax, red[i]);
    int ex = 0;
    if (amax > 0.f) frexpf(amax, &ex); // amax = m * 2^ex, m in [0.5, 1)  ->  |x| * 2^(30-ex) < 2^30
    int p = 30 - ex;
    p = p > 120 ? 120 : p;
    const float S = ldexpf(1.0f, p);
    if (threadIdx.x == 0) inv_scale[t] = ldexpf(1.0f, -p);

    uint8_t *dt = dig + t * dig_stride;
    float *xs = xsum + t * xs_stride;
    for (int gi = threadIdx.x; gi < K / 8; gi += blockDim.x) {
        const int S_idx = gi >> 2, a = gi & 3;
        const float4 v0 = *reinterpret_cast<const float4 *>(xt + gi * 8);
        const float4 v1 = *reinterpret_cast<const float4 *>(xt + gi * 8 + 4);
        const float f[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
        int r[8];
        long long sum = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            r[e] = static_cast<int>(rintf(f[e] * S)); // power-of-two scaling is exact; one rounding to integer
            sum += r[e];
        }
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
            *reinterpret_cast<uint2 *>(dt + static_cast<int64_t>(S_idx) * 128 + dg * 32 + a * 8) = o;
        }
        sum += __shfl_xor(sum, 1, 64);
        sum += __shfl_xor(sum, 2, 64);
        if (a == 0) xs[S_idx] = static_cast<float>(sum);
    }
}

// ------------------------------------------------------------------------------------------
struct MfmaSeg {
    const uint8_t *W;
    float *y;
    const float *resid;
    int64_t n_rows;
    int tile0; // first 16-row tile of this segment in the launch
};

struct MfmaArgs {
    MfmaSeg seg[3];
    int nseg, n_tiles, nb; // nb: super-blocks per row
    int slab_blocks;       // super-blocks per K slab (grid.y slabs)
    const uint8_t *dig;    // digits of x
    const float *xsum;     // per-sub-block sums of xfix
    const float *inv_scale;
    float *part;           // [n_slabs][n_tiles*16] partial sums when n_slabs > 1
    int n_slabs;
};

struct BlockRegs {
    uint4 hdr, qa, qb;
};

__device__ __forceinline__ void load_block(BlockRegs &r, const uint4 *rowp, int blk, int g)
{
    const uint4 *bp = rowp + blk * 9;
    r.hdr = bp[0];
    r.qa = bp[1 + g];
    r.qb = bp[5 + g];
}

__device__ __forceinline__ long pack64(uint32_t lo, uint32_t hi)
{
    return static_cast<long>(static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32));
}

// four MFMAs: one 16-byte quant chunk per lane against the digits of its sub-block
__device__ __forceinline__ v4i chunk_dot(const uint4 &q, const uint4 &xa, const uint4 &xb)
{
    v4i acc = {0, 0, 0, 0};
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
    const long A[4] = {pack64(xa.x, xa.y), pack64(xa.z, xa.w), pack64(xb.x, xb.y), pack64(xb.z, xb.w)};
#pragma unroll
    for (int a = 0; a < 4; ++a) {
        const uint32_t lo = w[a] & 0x0f0f0f0fu;        // weights 8a + 0,2,4,6
        const uint32_t hi = (w[a] >> 4) & 0x0f0f0f0fu; // weights 8a + 1,3,5,7
        acc = __builtin_amdgcn_mfma_i32_16x16x32_i8(A[a], pack64(lo, hi), acc, 0, 0, 0);
    }
    return acc;
}

// KSW waves of a 4-wave block split the slab's super-blocks; 4/KSW row tiles per block.
template <int KSW>
__global__ void __launch_bounds__(256) gemv_t1_mfma_kernel(MfmaArgs a)
{
    constexpr int TPW = 4 / KSW;
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, g = lane >> 4;
    const int tw = wave / KSW, kw = wave % KSW;
    const int tile = blockIdx.x * TPW + tw;
    const int slab = blockIdx.y;
    const int sb0 = slab * a.slab_blocks;
    const int sb1 = min(sb0 + a.slab_blocks, a.nb);
    const int nbs = sb1 - sb0;

    // LDS: digits [nbs*8][SUB_LDS] | zeros [32] | xsum [slab_blocks*8] | reduction [4][16]
    uint8_t *l_dig = smem;
    const int zero_off = a.slab_blocks * 8 * SUB_LDS;
    float *l_xs = reinterpret_cast<float *>(smem + zero_off + 32);
    float *l_red = l_xs + a.slab_blocks * 8;

    {
        const uint4 *src = reinterpret_cast<const uint4 *>(a.dig) + static_cast<int64_t>(sb0) * 64;
        for (int i = threadIdx.x; i < nbs * 64; i += 256) {
            const int s = i >> 3, c = i & 7;
            *reinterpret_cast<uint4 *>(l_dig + s * SUB_LDS + c * 16) = src[i];
        }
        for (int i = threadIdx.x; i < nbs * 8; i += 256) l_xs[i] = a.xsum[sb0 * 8 + i];
        if (threadIdx.x < 8) reinterpret_cast<uint32_t *>(smem + zero_off)[threadIdx.x] = 0u;
    }
    __syncthreads();

    float total = 0.f;
    const bool tile_ok = tile < a.n_tiles;
    int sg = 0;
    int64_t row_in_seg = 0;
    if (tile_ok) {
        while (sg + 1 < a.nseg && tile >= a.seg[sg + 1].tile0) ++sg;
        const MfmaSeg seg = a.seg[sg];
        row_in_seg = static_cast<int64_t>(tile - seg.tile0) * 16 + j;
        const int64_t row_ld = row_in_seg < seg.n_rows ? row_in_seg : seg.n_rows - 1; // rows past the end re-read the last row
        const uint4 *rowp = reinterpret_cast<const uint4 *>(seg.W + row_ld * a.nb * BLOCK_BYTES);

        const int per = (nbs + KSW - 1) / KSW;
        const int wb0 = sb0 + kw * per;
        const int wb1 = min(wb0 + per, sb1);

        // lanes whose output slots hold this lane's k-group carry digits; all others feed zeros
        const bool active = (j >> 2) == g;
        const int a_base = active ? g * SUB_LDS + (j & 3) * 32 : zero_off;
        const int a_step = active ? SUB_LDS : 0;
        const int fsh = 6 * g;

        float yacc = 0.f, macc = 0.f;
        // one super-block: 8 MFMAs + integer sub-scales + fp32 recombination
        auto compute = [&](const BlockRegs &c, int b) {
            const int s_loc = (b - sb0) * 8;
            const uint8_t *ap = l_dig + a_base + s_loc * a_step;
            const uint4 x0 = *reinterpret_cast<const uint4 *>(ap);
            const uint4 x1 = *reinterpret_cast<const uint4 *>(ap + 16);
            const uint4 x2 = *reinterpret_cast<const uint4 *>(ap + 4 * a_step);
            const uint4 x3 = *reinterpret_cast<const uint4 *>(ap + 4 * a_step + 16);
            const v4i d0 = chunk_dot(c.qa, x0, x1);
            const v4i d1 = chunk_dot(c.qb, x2, x3);
            const int sc0 = static_cast<int>(__builtin_amdgcn_ubfe(c.hdr.y, fsh, 6));
            const int sc1 = static_cast<int>(__builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(c.hdr.z, c.hdr.y, 24), fsh, 6));
            const uint32_t m0 = __builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(c.hdr.w, c.hdr.z, 16), fsh, 6);
            const uint32_t m1 = __builtin_amdgcn_ubfe(c.hdr.w, 8 + fsh, 6);
            const int i0 = __mul24(d0[0], sc0) + __mul24(d1[0], sc1);
            const int i1 = __mul24(d0[1], sc0) + __mul24(d1[1], sc1);
            const int i2 = __mul24(d0[2], sc0) + __mul24(d1[2], sc1);
            const int i3 = __mul24(d0[3], sc0) + __mul24(d1[3], sc1);
            float f = static_cast<float>(i3);
            f = fmaf(f, 256.f, static_cast<float>(i2));
            f = fmaf(f, 256.f, static_cast<float>(i1));
            f = fmaf(f, 256.f, static_cast<float>(i0));
            yacc = fmaf(hdr_d(c.hdr), f, yacc);
            const float ms = fmaf(static_cast<float>(m0), l_xs[s_loc + g], static_cast<float>(m1) * l_xs[s_loc + 4 + g]);
            macc = fmaf(hdr_dmin(c.hdr), ms, macc);
        };
        if (wb0 < wb1) {
            // three register stages, two super-blocks of loads in flight ahead of the one in use
            const int last = wb1 - 1;
            BlockRegs r0, r1, r2;
            load_block(r0, rowp, wb0, g);
            load_block(r1, rowp, min(wb0 + 1, last), g);
            for (int b = wb0; b < wb1; b += 3) {
                load_block(r2, rowp, min(b + 2, last), g);
                compute(r0, b);
                if (b + 1 < wb1) {
                    load_block(r0, rowp, min(b + 3, last), g);
                    compute(r1, b + 1);
                }
                if (b + 2 < wb1) {
                    load_block(r1, rowp, min(b + 4, last), g);
                    compute(r2, b + 2);
                }
            }
        }
        total = yacc - macc;
        total += __shfl_xor(total, 16, 64);
        total += __shfl_xor(total, 32, 64);
        if (g == 0) l_red[wave * 16 + j] = total;
    }
    __syncthreads();
    if (tile_ok && kw == 0 && g == 0) {
        float v = 0.f;
#pragma unroll
        for (int k = 0; k < KSW; ++k) v += l_red[(tw * KSW + k) * 16 + j]; // fixed order
        const MfmaSeg seg = a.seg[sg];
        if (a.n_slabs > 1) {
            a.part[static_cast<int64_t>(slab) * a.n_tiles * 16 + tile * 16 + j] = v;
        } else if (row_in_seg < seg.n_rows) {
            v *= a.inv_scale[0];
            if (seg.resid) v += seg.resid[row_in_seg];
            seg.y[row_in_seg] = v;
        }
    }
}

// y = 2^-p * sum over slabs (fixed order) + residual
__global__ void __launch_bounds__(256) gemv_t1_reduce_kernel(MfmaArgs a)
{
    const int64_t R = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; // padded row index
    if (R >= static_cast<int64_t>(a.n_tiles) * 16) return;
    const int tile = static_cast<int>(R >> 4);
    int sg = 0;
    while (sg + 1 < a.nseg && tile >= a.seg[sg + 1].tile0) ++sg;
    const MfmaSeg seg = a.seg[sg];
    const int64_t r = R - static_cast<int64_t>(seg.tile0) * 16;
    if (r >= seg.n_rows) return;
    float v = 0.f;
    for (int s = 0; s < a.n_slabs; ++s) v += a.part[static_cast<int64_t>(s) * a.n_tiles * 16 + R];
    v *= a.inv_scale[0];
    if (seg.resid) v += seg.resid[r];
    seg.y[r] = v;
}

// workspace: digits K*4 B | xsum K/32 floats | inv scale | partials
struct T1Plan {
    int n_tiles, nb, ksw, n_slabs, slab_blocks;
    size_t off_dig, off_xs, off_inv, off_part, total;
    size_t lds_bytes;
};

// upper bound of the partial-sum buffer for any segmentation of rows_total rows
static size_t t1_part_bound(int64_t rows_total, int64_t n_cols)
{
    const size_t nb = static_cast<size_t>(n_cols / QK);
    return (nb / 7 + 2) * static_cast<size_t>(rows_total + 48) * sizeof(float);
}

static T1Plan plan_t1(const int64_t *seg_rows, int nseg, int64_t n_cols)
{
    T1Plan p{};
    p.nb = static_cast<int>(n_cols / QK);
    p.n_tiles = 0;
    for (int i = 0; i < nseg; ++i) p.n_tiles += static_cast<int>((seg_rows[i] + 15) / 16);
    // aim at ~16 waves per CU on 256 CUs, but keep at least ~7 super-blocks per wave
    int splits = (4096 + p.n_tiles - 1) / (p.n_tiles > 0 ? p.n_tiles : 1);
    const int max_splits = p.nb / 7 > 0 ? p.nb / 7 : 1;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    p.ksw = splits >= 4 ? 4 : (splits >= 2 ? 2 : 1);
    int slabs = (splits + p.ksw - 1) / p.ksw;
    const int min_slabs = (p.nb + 31) / 32; // at most 32 super-blocks of digits in LDS
    if (slabs < min_slabs) slabs = min_slabs;
    p.slab_blocks = (p.nb + slabs - 1) / slabs;
    p.n_slabs = (p.nb + p.slab_blocks - 1) / p.slab_blocks;
    int64_t rows_total = 0;
    for (int i = 0; i < nseg; ++i) rows_total += seg_rows[i];
    size_t off = 0;
    auto take = [&](size_t b) { size_t o = off; off += round_up(b, 256); return o; };
    p.off_dig = take(static_cast<size_t>(n_cols) * 4);
    p.off_xs = take(static_cast<size_t>(n_cols / 32) * sizeof(float));
    p.off_inv = take(sizeof(float));
    p.off_part = take(t1_part_bound(rows_total, n_cols));
    p.total = off;
    p.lds_bytes = static_cast<size_t>(p.slab_blocks) * 8 * SUB_LDS + 32 + static_cast<size_t>(p.slab_blocks) * 8 * 4 + 4 * 16 * 4;
    return p;
}

size_t gemv_t1_ws_bytes(int64_t n_rows_total, int64_t n_cols)
{
    const int64_t rows[1] = {n_rows_total};
    return plan_t1(rows, 1, n_cols).total;
}

prima_status launch_gemv_t1(const GemvArgs &ga, void *ws, size_t ws_bytes, hipStream_t st)
{
    int64_t rows[3];
    for (int i = 0; i < ga.nseg; ++i) rows[i] = ga.seg[i].n_rows;
    const T1Plan p = plan_t1(rows, ga.nseg, ga.n_cols);
    if (p.total > ws_bytes) return PRIMA_E_WORKSPACE;
    char *base = static_cast<char *>(ws);
    uint8_t *dig = reinterpret_cast<uint8_t *>(base + p.off_dig);
    float *xs = reinterpret_cast<float *>(base + p.off_xs);
    float *inv = reinterpret_cast<float *>(base + p.off_inv);

    hipLaunchKernelGGL(quantize_x_kernel, dim3(1), dim3(1024), 0, st, ga.x, ga.ldx, static_cast<int>(ga.n_cols), dig, xs, inv,
                       static_cast<int64_t>(0), static_cast<int64_t>(0));

    MfmaArgs a{};
    int tile0 = 0;
    for (int i = 0; i < ga.nseg; ++i) {
        a.seg[i] = MfmaSeg{ga.seg[i].W, ga.seg[i].y, ga.seg[i].resid, ga.seg[i].n_rows, tile0};
        tile0 += static_cast<int>((ga.seg[i].n_rows + 15) / 16);
    }
    a.nseg = ga.nseg;
    a.n_tiles = p.n_tiles;
    a.nb = p.nb;
    a.slab_blocks = p.slab_blocks;
    a.dig = dig;
    a.xsum = xs;
    a.inv_scale = inv;
    a.part = reinterpret_cast<float *>(base + p.off_part);
    a.n_slabs = p.n_slabs;
    const int tpw = 4 / p.ksw;
    const dim3 grid((p.n_tiles + tpw - 1) / tpw, p.n_slabs), block(256);
    switch (p.ksw) {
    case 1: hipLaunchKernelGGL(gemv_t1_mfma_kernel<1>, grid, block, p.lds_bytes, st, a); break;
    case 2: hipLaunchKernelGGL(gemv_t1_mfma_kernel<2>, grid, block, p.lds_bytes, st, a); break;
    default: hipLaunchKernelGGL(gemv_t1_mfma_kernel<4>, grid, block, p.lds_bytes, st, a); break;
    }
    if (p.n_slabs > 1)
        hipLaunchKernelGGL(gemv_t1_reduce_kernel, dim3((p.n_tiles * 16 + 255) / 256), dim3(256), 0, st, a);
    return last_launch_status();
}

} // namespace prima
