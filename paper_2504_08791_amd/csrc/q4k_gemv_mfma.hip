// Dequant-fused Q4_K mat-vec on the matrix cores with exact integer accumulation (gfx950).
//
// The weight stream (the b bytes per layer of arXiv 2504.08791, App. A.3) is what bounds decode;
// everything else has to hide behind it.
//
// Arithmetic.  At 8 TB/s a CU receives ~26 four-bit weights per clock but its vector ALUs issue 64
// lane-operations per clock, so a multiply-add per weight per token plus the nibble unpacking does
// not fit.  The multiply-adds run on the MFMA units instead:
//  * each activation vector is turned into block fixed point once per mat-vec: x = xfix * 2^-p,
//    |xfix| < 2^30, split into four signed 8-bit digits (xfix = sum_r digit_r * 256^r);
//  * a wave owns 16 output rows; lane (j, g) = (lane % 16, lane / 16) takes the 16-byte quant chunk
//    of row j, sub-block s0+g, splits it into two int8 vectors with three ALU ops per 8 weights and
//    feeds them as the B operand of v_mfma_i32_16x16x32_i8;
//  * the A operand holds the digits, arranged block-diagonally: output slot 4g'+r carries digit r
//    restricted to k-group g'.  The MFMA result on lane (j, g) is then exactly the four digit sums
//    of row j with *its own* sub-block s0+g: sum_k q_k * digit_r(x_k);
//  * the 6-bit sub-scale multiplies these integers (still exact), the four digits are recombined
//    in fp32, and d (fp16) scales the super-block.  The min term uses per-sub-block sums of xfix:
//        y = 2^-p * sum_blocks [ d * sum_s sc_s * (q . xfix)_s  -  dmin * sum_s m_s * Xsum_s ].
//    For T tokens the unpacked weights are reused against each token's digits.
//
// Data movement.  One 512-thread workgroup per compute unit, persistent; it owns a contiguous range
// of 16-row tiles with all of K, so no sum crosses workgroups and every sum has a fixed order.
// Each wave streams its share of the weights through a private three-stage LDS ring filled by
// 128-bit global->LDS loads (no VGPR staging): a stage is 16 rows x 2 super-blocks, requested as
// runs of 288 contiguous bytes per row, laid out with an odd row stride so that the MFMA-order
// reads (lane (j, g) reads row j) are free of bank conflicts.  Two stages are always in flight
// per wave while the third is consumed; only s_waitcnt orders them, no barrier.  The activations
// are transformed (RMSNorm or SwiGLU when asked), quantised and laid out in LDS by every
// workgroup for itself, slab by slab when K is too long for the LDS left over by the rings.
#include "common.h"

namespace prima {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int GEMV_THREADS = 512;
constexpr int GEMV_WAVES = GEMV_THREADS / 64;
constexpr int NST = 3;                       // ring stages per wave
constexpr int PBS = 2;                       // super-blocks per stage
constexpr int RS = 9 * PBS + 1;              // row stride of a stage in 16-byte slots (odd)
constexpr int STAGE_SLOTS = 16 * RS;         // 304
constexpr int NI = (STAGE_SLOTS + 63) / 64;  // load instructions per stage (5; the last one uses 48 lanes)
constexpr int STAGE_BYTES = STAGE_SLOTS * 16;
constexpr int RING_BYTES = GEMV_WAVES * NST * STAGE_BYTES;
constexpr int SUB_BYTES = 128;               // digits of one sub-block: 4 digits x 32 values
constexpr size_t LDS_BUDGET = 160 * 1024;
constexpr int MAX_T_PASS = 8;                // tokens per pass over the weights

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
    int ksplit;      // waves sharing a tile: unit = (tile, part), part p takes chunks p, p+ksplit, ...
    int slab_blocks; // super-blocks of activations staged in LDS at a time (even)
    int n_slabs;
    int units_cap;   // partial-sum slots per workgroup
    int n_wg;
};

// 16 bytes per lane from global memory straight into LDS: lane l writes bytes [16 l, 16 l + 16) of the
// 1 KiB at LDS byte address lds_addr (wave-uniform, goes through M0).  Written as inline assembly on
// purpose: the compiler then does not know these loads write LDS and leaves the ordering against the
// later LDS reads to the explicit s_waitcnt vmcnt(N) below, which lets newer stages stay in flight
// (with the builtin it waits for *all* outstanding loads before any LDS read).  Loads complete in
// order, so loads the compiler does not know about can only make its own waits stricter.
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_addr)
{
    // one wait state is required between the SALU write of M0 and the load that reads it; M0 is a reserved
    // register that nothing else in this file uses
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_addr) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(p)); // low half of a flat LDS pointer is the LDS byte address
}

__device__ __forceinline__ long pack64(uint32_t lo, uint32_t hi)
{
    return static_cast<long>(static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32));
}

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

// eight consecutive activations of token t starting at column c0, before the RMSNorm scale:
// X_PLAIN x, X_RMSNORM x*gain (the 1/rms factor is applied by the caller), X_SWIGLU silu(x)*x2
template <int XMODE>
__device__ __forceinline__ void load_act8(const PGemvArgs &a, int t, int c0, float *f)
{
    const float *xp = a.x + t * a.ldx + c0;
    const float4 v0 = *reinterpret_cast<const float4 *>(xp), v1 = *reinterpret_cast<const float4 *>(xp + 4);
    f[0] = v0.x; f[1] = v0.y; f[2] = v0.z; f[3] = v0.w; f[4] = v1.x; f[5] = v1.y; f[6] = v1.z; f[7] = v1.w;
    if (XMODE == X_RMSNORM) {
        const float4 g0 = *reinterpret_cast<const float4 *>(a.gain + c0), g1 = *reinterpret_cast<const float4 *>(a.gain + c0 + 4);
        const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] *= gg[e];
    } else if (XMODE == X_SWIGLU) {
        const float *up = a.x2 + t * a.ldx + c0;
        const float4 u0 = *reinterpret_cast<const float4 *>(up), u1 = *reinterpret_cast<const float4 *>(up + 4);
        const float uu[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = f[e] / (1.0f + expf(-f[e])) * uu[e];
    }
}

// position of a wave in its stream of stages: slab -> unit (tile, part) -> chunk of PBS super-blocks
struct Cursor {
    int slab, u, c;
    bool valid;
};

// TT tokens; XMODE how the activations are obtained; NSEG matrices sharing the activations (compile-time
// so that the projections of a layer appear as separate kernels in a profile)
template <int TT, int XMODE, int NSEG>
__global__ void __launch_bounds__(GEMV_THREADS) gemv_q4k_persistent_kernel(PGemvArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 15, g = lane >> 4;
    const int K = a.nb * QK;

    // tiles of this workgroup
    const int tl0 = static_cast<int>(static_cast<int64_t>(a.n_tiles) * blockIdx.x / a.n_wg);
    const int tl1 = static_cast<int>(static_cast<int64_t>(a.n_tiles) * (blockIdx.x + 1) / a.n_wg);
    const int ntl = tl1 - tl0;
    if (ntl == 0) return;
    const int n_units = ntl * a.ksplit;

    // LDS carve: rings | 32 zero bytes | digits [TT][slab_sub][128] | xsum [TT][slab_sub] | partial [units_cap][TT][16] | red[16] | stats [3 TT]
    const int slab_sub = a.slab_blocks * 8;
    uint8_t *l_ring = smem + wave * (NST * STAGE_BYTES);
    uint8_t *l_zero = smem + RING_BYTES;      // 32 zero bytes: the A operand of lanes that carry no digits
    uint8_t *l_dig = l_zero + 32;
    const int dig_t_stride = slab_sub * SUB_BYTES;
    float *l_xs = reinterpret_cast<float *>(l_dig + TT * dig_t_stride);
    float *l_part = l_xs + TT * slab_sub;
    float *l_red = l_part + a.units_cap * TT * 16;
    float *l_scale = l_red + 16;  // [TT] 2^p (times 1/rms for RMSNorm input)
    float *l_inv = l_scale + TT;  // [TT] 2^-p

    // ---- stream geometry (wave-uniform) ----
    const int cps_full = a.slab_blocks / PBS; // chunks per full slab
    auto slab_chunks = [&](int slab) {
        const int blocks = min(a.slab_blocks, a.nb - slab * a.slab_blocks);
        return (blocks + PBS - 1) / PBS;
    };
    auto normalize = [&](Cursor &c) {
        for (;;) {
            if (c.slab >= a.n_slabs) { c.valid = false; return; }
            if (c.u >= n_units) { ++c.slab; c.u = wave; c.c = c.u % a.ksplit; continue; }
            if (c.c >= slab_chunks(c.slab)) { c.u += GEMV_WAVES; c.c = c.u % a.ksplit; continue; }
            c.valid = true;
            return;
        }
    };
    auto advance = [&](Cursor &c) { c.c += a.ksplit; normalize(c); };
    (void)cps_full;

    // per-lane slot decomposition of the NI load instructions of a stage: slot = i*64 + lane -> (row r, chunk c)
    int slot_r[NI], slot_c[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int slot = i * 64 + lane;
        const int r = slot / RS;
        slot_r[i] = r < 16 ? r : 15;
        slot_c[i] = slot - r * RS; // RS-1 is the padding slot
    }
    const int64_t pitch16 = static_cast<int64_t>(a.nb) * 9; // row pitch in 16-byte units

    // request the stage at cursor c into ring stage st: exactly NI load instructions, always
    auto issue = [&](const Cursor &c, int st) {
        const int tile = tl0 + c.u / a.ksplit;
        int sg = 0;
        while (sg + 1 < NSEG && tile >= a.seg_tile0[sg + 1]) ++sg;
        const int64_t row0 = static_cast<int64_t>(tile - a.seg_tile0[sg]) * 16;
        const int rows_valid = static_cast<int>(min<int64_t>(16, a.seg[sg].n_rows - row0));
        const int blk0 = c.slab * a.slab_blocks + c.c * PBS;
        const int ncol = 9 * min(PBS, a.nb - blk0); // valid 16-byte chunks per row in this stage
        const uint4 *base = reinterpret_cast<const uint4 *>(a.seg[sg].W) + row0 * pitch16 + static_cast<int64_t>(blk0) * 9;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_address(l_ring + st * STAGE_BYTES));
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // reads of the stage being overwritten have returned
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            // rows past the end of the matrix and chunks past the end of the row re-read valid data
            const int r = min(slot_r[i], rows_valid - 1);
            const int cc = min(slot_c[i], ncol - 1);
            const uint4 *src = base + r * pitch16 + cc;
            if (i * 64 + 63 < STAGE_SLOTS || lane < STAGE_SLOTS - i * 64)
                dma16(src, dst + i * 1024);
        }
    };

    // ---- start the weight stream before touching the activations ----
    Cursor lc;
    lc.slab = 0; lc.u = wave; lc.c = lc.u % a.ksplit; lc.valid = false;
    normalize(lc);
    int issued = 0;
    for (int s = 0; s < NST - 1 && lc.valid; ++s) {
        issue(lc, s);
        advance(lc);
        ++issued;
    }

    // zero the partial sums and the zero operand
    if (threadIdx.x < 8) reinterpret_cast<uint32_t *>(l_zero)[threadIdx.x] = 0u;
    for (int i = threadIdx.x; i < n_units * TT * 16; i += GEMV_THREADS) l_part[i] = 0.f;

    // ---- statistics of the activations: 1/rms (RMSNorm input) and the power-of-two scale ----
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        float ss = 0.f, amax = 0.f;
        for (int gi = threadIdx.x; gi < K / 8; gi += GEMV_THREADS) {
            float f[8];
            if (XMODE == X_RMSNORM) {
                const float *xp = a.x + t * a.ldx + gi * 8;
                const float4 v0 = *reinterpret_cast<const float4 *>(xp), v1 = *reinterpret_cast<const float4 *>(xp + 4);
                ss += ((v0.x * v0.x + v0.y * v0.y) + (v0.z * v0.z + v0.w * v0.w)) + ((v1.x * v1.x + v1.y * v1.y) + (v1.z * v1.z + v1.w * v1.w));
            }
            load_act8<XMODE>(a, t, gi * 8, f);
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(f[e]));
        }
        float inv_rms = 1.f;
        if (XMODE == X_RMSNORM) {
            ss = wg_reduce(ss, l_red, false);
            inv_rms = 1.0f / sqrtf(ss / static_cast<float>(K) + a.eps);
        }
        amax = wg_reduce(amax, l_red, true) * inv_rms; // max |x*gain| / rms
        int ex = 0;
        if (amax > 0.f) frexpf(amax, &ex); // amax = m * 2^ex, m in [0.5, 1)
        // |v| * 2^(29-ex) < 2^29 leaves room for the rounding of (x*gain)*(inv_rms*2^p) against x*gain*inv_rms
        int p = 29 - ex;
        p = p > 120 ? 120 : p;
        if (threadIdx.x == 0) {
            l_scale[t] = ldexpf(inv_rms, p);
            l_inv[t] = ldexpf(1.0f, -p);
        }
    }
    __syncthreads();

    // lanes whose output slots hold this lane's k-group carry digits; all others feed zeros.
    // Digit r of sub-block S sits at byte ((r + S) & 3) * 32 of its 128 bytes (S = s0 + g with s0 % 4 == 0),
    // so the 16 reading lanes (4 k-groups x 4 digits) fall into different banks.
    const bool active = (j >> 2) == g;
    const int a_lane = active ? 32 + g * SUB_BYTES + (((j & 3) + g) & 3) * 32 : 0; // byte offset from l_zero
    const int a_mul = active ? 1 : 0;                                              // inactive lanes stay on the zeros
    const int fsh = 6 * g;

    Cursor cc;
    cc.slab = 0; cc.u = wave; cc.c = cc.u % a.ksplit; cc.valid = false;
    normalize(cc);
    int step = 0, st = 0;

    float yacc[TT], macc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) { yacc[t] = 0.f; macc[t] = 0.f; }

    for (int slab = 0; slab < a.n_slabs; ++slab) {
        const int sb0 = slab * a.slab_blocks;
        const int sb1 = min(sb0 + a.slab_blocks, a.nb);
        if (slab > 0) __syncthreads(); // previous slab's digits no longer in use

        // ---- transform + quantise this slab's activations into LDS ----
        // digits [S][4][32 bytes]; byte order inside a digit row: for each group a of 8 values,
        // values 8a + {0,2,4,6,1,3,5,7}, the order in which the nibble split delivers the weights.
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const float S = l_scale[t];
            for (int gi = sb0 * 32 + threadIdx.x; gi < sb1 * 32; gi += GEMV_THREADS) {
                float f[8];
                load_act8<XMODE>(a, t, gi * 8, f);
                if (a.x_tap && blockIdx.x == 0) {
                    const float unq = S * l_inv[t]; // 1/rms for RMSNorm input, 1 otherwise
                    float *tp = a.x_tap + static_cast<int64_t>(t) * K + gi * 8;
                    *reinterpret_cast<float4 *>(tp) = make_float4(f[0] * unq, f[1] * unq, f[2] * unq, f[3] * unq);
                    *reinterpret_cast<float4 *>(tp + 4) = make_float4(f[4] * unq, f[5] * unq, f[6] * unq, f[7] * unq);
                }
                int r[8];
                long long sum = 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    r[e] = static_cast<int>(rintf(f[e] * S)); // one rounding to integer
                    sum += r[e];
                }
                const int s_glob = gi >> 2, s_loc = s_glob - sb0 * 8, grp = gi & 3;
                uint8_t *dp = l_dig + t * dig_t_stride + s_loc * SUB_BYTES + grp * 8;
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
                    *reinterpret_cast<uint2 *>(dp + ((dg + s_glob) & 3) * 32) = o;
                }
                sum += __shfl_xor(sum, 1, 64);
                sum += __shfl_xor(sum, 2, 64);
                if (grp == 0) l_xs[t * slab_sub + s_loc] = static_cast<float>(sum);
            }
        }
        __syncthreads();

        // ---- consume this wave's stages of the slab ----
        while (cc.valid && cc.slab == slab) {
            if (lc.valid) {
                issue(lc, (st + NST - 1) % NST);
                advance(lc);
                ++issued;
            }
            const int newer = issued - (step + 1); // stages requested after the one consumed now
            if (newer >= 2) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
            else if (newer == 1) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            static_assert(NI == 5 && NST == 3, "the vmcnt immediates above assume 5 loads per stage, 3 stages");

            const int blk0 = sb0 + cc.c * PBS;
            const int nblk = min(PBS, a.nb - blk0);
            const uint4 *stage = reinterpret_cast<const uint4 *>(l_ring + st * STAGE_BYTES) + j * RS;
#pragma unroll
            for (int b = 0; b < PBS; ++b) {
                if (b >= nblk) break;
                const uint4 hdr = stage[b * 9], qa = stage[b * 9 + 1 + g], qb = stage[b * 9 + 5 + g];
                const uint32_t w[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
                long B[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) B[i] = pack64(w[i] & 0x0f0f0f0fu, (w[i] >> 4) & 0x0f0f0f0fu); // weights 8i+{0,2,4,6 | 1,3,5,7}
                const int sc0 = static_cast<int>(__builtin_amdgcn_ubfe(hdr.y, fsh, 6));
                const int sc1 = static_cast<int>(__builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(hdr.z, hdr.y, 24), fsh, 6));
                const float m0 = static_cast<float>(__builtin_amdgcn_ubfe(__builtin_amdgcn_alignbit(hdr.w, hdr.z, 16), fsh, 6));
                const float m1 = static_cast<float>(__builtin_amdgcn_ubfe(hdr.w, 8 + fsh, 6));
                const float d = hdr_d(hdr), dmin = hdr_dmin(hdr);
                const int s_loc = (blk0 + b - sb0) * 8;
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    const uint8_t *ap = l_zero + a_lane + (t * dig_t_stride + s_loc * SUB_BYTES) * a_mul;
                    const uint4 x0 = *reinterpret_cast<const uint4 *>(ap);
                    const uint4 x1 = *reinterpret_cast<const uint4 *>(ap + 16);
                    const uint4 x2 = *reinterpret_cast<const uint4 *>(ap + 4 * SUB_BYTES * a_mul);
                    const uint4 x3 = *reinterpret_cast<const uint4 *>(ap + 4 * SUB_BYTES * a_mul + 16);
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
            }

            // next stage of this wave; leave the unit's sums in its slot when the unit (or the slab) ends
            const int u_done = cc.u;
            advance(cc);
            if (!cc.valid || cc.u != u_done || cc.slab != slab) {
                float *slot = l_part + u_done * (TT * 16);
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    float v = yacc[t] - macc[t];
                    v += __shfl_xor(v, 16, 64);
                    v += __shfl_xor(v, 32, 64);
                    if (g == 0) slot[t * 16 + j] += v;
                    yacc[t] = 0.f;
                    macc[t] = 0.f;
                }
            }
            st = (st + 1) % NST;
            ++step;
        }
    }
    __syncthreads();

    // ---- epilogue: add the parts of every (tile, row, token) in part order, scale, residual, store ----
    for (int idx = threadIdx.x; idx < ntl * 16 * TT; idx += GEMV_THREADS) {
        const int tile_local = idx / (16 * TT);
        const int rem = idx - tile_local * (16 * TT);
        const int t = rem >> 4, jj = rem & 15;
        float v = 0.f;
        for (int p = 0; p < a.ksplit; ++p) v += l_part[(tile_local * a.ksplit + p) * (TT * 16) + t * 16 + jj];
        const int tile = tl0 + tile_local;
        int sg = 0;
        while (sg + 1 < NSEG && tile >= a.seg_tile0[sg + 1]) ++sg;
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
    int n_tiles, nb, n_wg, ksplit, slab_blocks, n_slabs, units_cap;
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

static size_t fixed_lds(int T, int units_cap)
{
    return RING_BYTES + 32 + static_cast<size_t>(units_cap) * T * 16 * 4 + (16 + 2 * T) * 4 + 64;
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
    const int chunks = (p.nb + PBS - 1) / PBS;
    // waves per tile: the smallest of 1, 2, 4, 8 that gives every wave a unit and spreads the units evenly
    int best = 1;
    double best_eff = 0.0;
    for (int ks = 1; ks <= GEMV_WAVES; ks *= 2) {
        if (ks > chunks) break;
        const int units = tiles_wg * ks;
        const int rounds = (units + GEMV_WAVES - 1) / GEMV_WAVES;
        const double eff = static_cast<double>(units) / (rounds * GEMV_WAVES);
        if (eff > best_eff + 1e-9) { best_eff = eff; best = ks; }
    }
    p.ksplit = best;
    p.units_cap = tiles_wg * p.ksplit;
    // activations staged per slab: as many super-blocks (even) as the LDS left by rings and partial sums holds
    const size_t fixed = fixed_lds(T, p.units_cap);
    const size_t per_block = static_cast<size_t>(T) * 8 * (SUB_BYTES + 4);
    int cap = fixed < LDS_BUDGET ? static_cast<int>((LDS_BUDGET - fixed) / per_block) : 0;
    cap &= ~1;
    p.ok = cap >= 2;
    if (!p.ok) return p;
    p.n_slabs = (p.nb + cap - 1) / cap;
    p.slab_blocks = ((p.nb + p.n_slabs - 1) / p.n_slabs + 1) & ~1;
    p.n_slabs = (p.nb + p.slab_blocks - 1) / p.slab_blocks;
    p.lds_bytes = fixed + per_block * p.slab_blocks;
    return p;
}

template <int TT, int XMODE, int NSEG>
static hipError_t launch_inst(const PGemvArgs &a, const PPlan &p, hipStream_t st)
{
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemv_q4k_persistent_kernel<TT, XMODE, NSEG>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(LDS_BUDGET));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemv_q4k_persistent_kernel<TT, XMODE, NSEG>), dim3(p.n_wg), dim3(GEMV_THREADS), p.lds_bytes, st, a);
    return hipGetLastError();
}

// the combinations a decoder layer and the output layer use
template <int TT>
static hipError_t launch_tt(const PGemvArgs &a, const PPlan &p, hipStream_t st)
{
    if (a.xmode == X_RMSNORM && a.nseg == 3) return launch_inst<TT, X_RMSNORM, 3>(a, p, st); // Q/K/V
    if (a.xmode == X_RMSNORM && a.nseg == 2) return launch_inst<TT, X_RMSNORM, 2>(a, p, st); // gate/up
    if (a.xmode == X_RMSNORM && a.nseg == 1) return launch_inst<TT, X_RMSNORM, 1>(a, p, st); // output layer
    if (a.xmode == X_SWIGLU && a.nseg == 1) return launch_inst<TT, X_SWIGLU, 1>(a, p, st);   // down
    if (a.xmode == X_PLAIN && a.nseg == 1) return launch_inst<TT, X_PLAIN, 1>(a, p, st);     // attention output, plain mat-vec
    return hipErrorInvalidValue;
}

prima_status launch_gemv_mfma(const GemvArgs &ga, hipStream_t st)
{
    // up to MAX_T_PASS tokens per pass over the weights
    for (int t0 = 0; t0 < ga.T; t0 += MAX_T_PASS) {
        const int T = ga.T - t0 < MAX_T_PASS ? ga.T - t0 : MAX_T_PASS;
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
        a.ksplit = p.ksplit;
        a.slab_blocks = p.slab_blocks;
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
