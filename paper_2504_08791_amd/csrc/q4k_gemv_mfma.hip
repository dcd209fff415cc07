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
// of 16-row tiles (with all of K whenever the activations fit in LDS); every sum has a fixed order.
// Each wave streams its share of the weights through a private three-stage LDS ring filled by
// 128-bit global->LDS loads (no VGPR staging): a stage is 16 rows x 2 super-blocks, requested as
// runs of 288 contiguous bytes per row, laid out with an odd row stride so that the MFMA-order
// reads (lane (j, g) reads row j) are free of bank conflicts.  Two stages are always in flight
// per wave while the third is consumed; only s_waitcnt orders them, no barrier.  The activations
// are transformed (RMSNorm or SwiGLU when asked), quantised and laid out in LDS by every
// workgroup for itself.  When the digits of all of K do not fit in the LDS left over by the rings, K
// is cut into slabs and a workgroup handles one slab of a (larger) range of tiles; the slabs'
// partial sums meet in global memory, where the workgroup that arrives last at a tile adds them in
// slab order (release/acquire fences and one atomic counter per tile, reset for the next launch).
#include "common.h"

namespace prima {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));

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
    int xmode, epi;
    const float *x, *gain;
    int64_t ldx;
    float eps;
    // decomposition
    int ksplit;      // waves sharing a tile: unit = (tile, part), part p takes chunks p, p+ksplit, ...
    int slab_blocks; // super-blocks of K per slab (even); workgroup w handles slab w % n_slabs
    int n_slabs;
    int units_cap;   // floats reserved for the partial sums (and the per-tile flags of the slab reduction)
    int direct;      // a wave owns whole rows of the slab (ksplit == 1) and stores their sums itself
    int n_wg;
    float *part;        // n_slabs > 1: partial sums [n_slabs][n_tiles*16][T]
    unsigned *arrivals; // n_slabs > 1: per-tile arrival counters, zero between launches
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

// 16 bytes per lane into registers, requested now and waited for by hand: the compiler does not know
// that the result arrives later, which is the point: it cannot put a wait for *all* outstanding loads
// (the ring stages behind them included) in front of the first use.  Until the hand-written wait, which
// names these registers as operands, nothing may touch them.
__device__ __forceinline__ v4f load16_early(const void *gptr)
{
    v4f v;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(v) : "v"(gptr) : "memory");
    return v;
}

// workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding global
// load (vmcnt(0)), which would stall the weight stream at each barrier of the prologue.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(p)); // low half of a flat LDS pointer is the LDS byte address
}

__device__ __forceinline__ long pack64(uint32_t lo, uint32_t hi)
{
    return static_cast<long>(static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32));
}

// eight consecutive activations of token t starting at column c0, before the RMSNorm scale:
// X_PLAIN x, X_RMSNORM x*gain (the 1/rms factor is applied by the caller)
__device__ __forceinline__ void load_act8(const PGemvArgs &a, int t, int c0, float *f)
{
    const float *xp = a.x + t * a.ldx + c0;
    const float4 v0 = *reinterpret_cast<const float4 *>(xp), v1 = *reinterpret_cast<const float4 *>(xp + 4);
    f[0] = v0.x; f[1] = v0.y; f[2] = v0.z; f[3] = v0.w; f[4] = v1.x; f[5] = v1.y; f[6] = v1.z; f[7] = v1.w;
    if (a.xmode == X_RMSNORM) {
        const float4 g0 = *reinterpret_cast<const float4 *>(a.gain + c0), g1 = *reinterpret_cast<const float4 *>(a.gain + c0 + 4);
        const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] *= gg[e];
    }
}

// position of a wave in its stream of stages: k-th unit (tile, part) the wave took -> chunk of PBS super-blocks
struct Cursor {
    int k, u, c;
    bool valid;
};
constexpr int STATIC_UNITS = 2; // units per wave assigned by position; the rest go to whichever wave asks first
constexpr int FIFO = 8;         // units a wave may have requested and not yet consumed (a power of two > NST)

// TT tokens per pass.  The kind of activations, the number of matrices and the epilogue are run-time
// arguments: the projections of a layer then share one piece of code, which stays in the instruction
// caches from launch to launch (with one kernel per projection every launch started on cold caches and
// took 3-4 us longer).
template <int TT>
__global__ void __launch_bounds__(GEMV_THREADS) gemv_q4k_persistent_kernel(PGemvArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j = lane & 15, g = lane >> 4;
    const int K = a.nb * QK;
    const bool rmsnorm = a.xmode == X_RMSNORM;
    const bool pairs = a.epi == EPI_SWIGLU;
    const int gran = pairs ? 2 : 1; // tiles that are finished together: a (gate, up) pair sits on tiles 2p, 2p+1

    // slab and tiles of this workgroup
    const int slab = blockIdx.x % a.n_slabs, rank = blockIdx.x / a.n_slabs;
    const int nwg_slab = (a.n_wg - slab + a.n_slabs - 1) / a.n_slabs; // workgroups that share this slab
    const int n_groups = a.n_tiles / gran;
    const int tl0 = gran * static_cast<int>(static_cast<int64_t>(n_groups) * rank / nwg_slab);
    const int tl1 = gran * static_cast<int>(static_cast<int64_t>(n_groups) * (rank + 1) / nwg_slab);
    const int ntl = tl1 - tl0;
    if (ntl == 0) return;
    const int n_units = ntl * a.ksplit;
    const int sb0 = slab * a.slab_blocks;            // super-blocks [sb0, sb1) of every row
    const int sb1 = min(sb0 + a.slab_blocks, a.nb);
    const int n_chunks = (sb1 - sb0 + PBS - 1) / PBS;

    // LDS carve: rings | 32 zero bytes | digits [TT][slab_sub][128] | xsum [TT][slab_sub] | partial [units_cap][TT][16] | red[TT][16] | stats [2 TT]
    const int slab_sub = a.slab_blocks * 8;
    uint8_t *l_ring = smem + wave * (NST * STAGE_BYTES);
    uint8_t *l_zero = smem + RING_BYTES;      // 32 zero bytes: the A operand of lanes that carry no digits
    uint8_t *l_dig = l_zero + 32;
    const int dig_t_stride = slab_sub * SUB_BYTES;
    float *l_xs = reinterpret_cast<float *>(l_dig + TT * dig_t_stride);
    float *l_part = l_xs + TT * slab_sub;
    float *l_red = l_part + a.units_cap;
    float *l_scale = l_red + 16 * TT;  // [TT] 2^p (times 1/rms for RMSNorm input)
    float *l_inv = l_scale + TT;  // [TT] 2^-p
    int *l_next = reinterpret_cast<int *>(l_inv + TT); // next unit nobody has taken
    int *l_fifo = l_next + 1 + wave * FIFO;            // units this wave has taken, by k % FIFO

    // ---- stream geometry (wave-uniform) ----
    // Units are handed out in order, so the parts of a tile are in flight together; the first STATIC_UNITS of
    // a wave are fixed (they are requested before the counter exists), the others come from the counter.
    // The requesting cursor runs ahead and records what it took; the consuming cursor replays the record.
    auto unit_k = [&](int k, bool requesting) -> int {
        if (k < STATIC_UNITS) return wave + GEMV_WAVES * k;
        int u = 0;
        if (requesting) {
            if (lane == 0) {
                u = __hip_atomic_fetch_add(l_next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                l_fifo[k % FIFO] = u;
            }
        } else {
            u = l_fifo[k % FIFO];
        }
        return __builtin_amdgcn_readfirstlane(u);
    };
    auto start = [&](Cursor &c) { c.k = 0; c.u = wave; c.c = c.u % a.ksplit; c.valid = false; };
    // make the cursor point at a chunk that exists (or find that the units have run out); a cursor that
    // has run out stays so and asks for nothing more
    auto normalize = [&](Cursor &c, bool requesting) {
        for (;;) {
            if (c.u >= n_units) { c.valid = false; return; }
            if (c.c >= n_chunks) { ++c.k; c.u = unit_k(c.k, requesting); c.c = c.u % a.ksplit; continue; }
            c.valid = true;
            return;
        }
    };

    // per-lane slot decomposition of the NI load instructions of a stage: slot = i*64 + lane -> (row r, chunk c)
    int slot_r[NI], slot_c[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int slot = i * 64 + lane;
        const int r = slot / RS;
        slot_r[i] = r < 16 ? r : 15;
        slot_c[i] = slot - r * RS; // RS-1 is the padding slot
    }
    const int64_t pitch16 = static_cast<int64_t>(a.nb) * 9; // row pitch in 16-byte units (< 2^27: n_cols < 2^32)

    // matrix and position of a tile, from statically indexed kernel arguments only (scalar selects, no
    // memory access): sg segment, tis tile inside the segment
    auto seg_of = [&](int tile, int &sg, int &tis) {
        if (pairs) { sg = tile & 1; tis = tile >> 1; return; }
        sg = 0; tis = tile;
        if (a.nseg > 1 && tile >= a.seg_tile0[1]) { sg = 1; tis = tile - a.seg_tile0[1]; }
        if (a.nseg > 2 && tile >= a.seg_tile0[2]) { sg = 2; tis = tile - a.seg_tile0[2]; }
    };
    // offsets (16-byte units) of this lane's slots from the first chunk of a full stage
    int off_full[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) off_full[i] = slot_r[i] * static_cast<int>(pitch16) + min(slot_c[i], 9 * PBS - 1);

    // request the stage at cursor c into ring stage st: exactly NI load instructions, always
    auto issue = [&](const Cursor &c, int st) {
        const int tile = tl0 + c.u / a.ksplit;
        int sg, tis;
        seg_of(tile, sg, tis);
        const uint4 *W16 = reinterpret_cast<const uint4 *>(sg == 0 ? a.seg[0].W : (sg == 1 ? a.seg[1].W : a.seg[2].W));
        const int64_t n_rows = sg == 0 ? a.seg[0].n_rows : (sg == 1 ? a.seg[1].n_rows : a.seg[2].n_rows);
        const int64_t row0 = static_cast<int64_t>(tis) * 16;
        const int rows_valid = static_cast<int>(min<int64_t>(16, n_rows - row0));
        const int blk0 = sb0 + c.c * PBS;
        const int nblk = min(PBS, sb1 - blk0);
        const uint4 *base = W16 + row0 * pitch16 + static_cast<int64_t>(blk0) * 9;
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_address(l_ring + st * STAGE_BYTES));
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // reads of the stage being overwritten have returned
        if (rows_valid == 16 && nblk == PBS) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
                if (i * 64 + 63 < STAGE_SLOTS || lane < STAGE_SLOTS - i * 64) dma16(base + off_full[i], dst + i * 1024);
        } else {
            // rows past the end of the matrix and chunks past the end of the row re-read valid data
            const int ncol = 9 * nblk;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int r = min(slot_r[i], rows_valid - 1);
                const int cc = min(slot_c[i], ncol - 1);
                if (i * 64 + 63 < STAGE_SLOTS || lane < STAGE_SLOTS - i * 64) dma16(base + r * pitch16 + cc, dst + i * 1024);
            }
        }
    };

    // ---- start the weight stream.  Loads return in order per wave and the global->LDS loads of a compute
    // unit go out at only about 1 KiB per 25 ns, so the order is: request the activations (ordinary loads,
    // quick to issue), request the first two ring stages right behind them, and wait for the activations
    // only.  One token and at most two groups of 8 activations per thread: that is done with hand-waited
    // loads.  Otherwise the activations are read (and waited for) first. ----
    Cursor lc;
    start(lc);
    int issued = 0;
    auto first_stages = [&](int n) {
        for (int s = issued; s < n; ++s) { // touches units k = 0, 1 only
            normalize(lc, true);
            if (!lc.valid) break;
            issue(lc, s);
            lc.c += a.ksplit;
            ++issued;
        }
    };
    const bool early = TT == 1 && (sb1 - sb0) * 32 <= 2 * GEMV_THREADS && (!rmsnorm || a.n_slabs == 1);
    v4f ex[2][2], eg[2][2]; // early: activations and gains of this thread's two groups
    if (early) {
        const float *gp = rmsnorm ? a.gain : a.x; // without gains the second set of loads is a dummy
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int gi = min(sb0 * 32 + static_cast<int>(threadIdx.x) + i * GEMV_THREADS, sb1 * 32 - 1); // clamped: always a valid address
            ex[i][0] = load16_early(a.x + gi * 8);
            ex[i][1] = load16_early(a.x + gi * 8 + 4);
            eg[i][0] = load16_early(gp + gi * 8);
            eg[i][1] = load16_early(gp + gi * 8 + 4);
        }
        first_stages(1);
        // the eight loads above are older than the ring stages: with both stages requested, 10 loads may
        // still be out (a wave with fewer stages to request simply waits for everything).  One wait
        // statement names all eight registers, so that every use of them comes after it.
        if (issued < 1) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("s_waitcnt vmcnt(5)" : "+v"(ex[0][0]), "+v"(ex[0][1]), "+v"(ex[1][0]), "+v"(ex[1][1]), "+v"(eg[0][0]), "+v"(eg[0][1]), "+v"(eg[1][0]), "+v"(eg[1][1]) :: "memory");
    }

    // ---- statistics of the activations: 1/rms over the whole row (RMSNorm input) and the power-of-two
    // scale of this slab's part (each slab has its own, its sums are scaled back before they meet) ----
    // One token: every thread keeps its groups of 8 activations in registers from here to the
    // quantisation (no second trip to memory).  Several tokens: they are read again.
    constexpr int MAXG = 8;                                  // register-resident groups per thread
    const int g_lo = rmsnorm ? 0 : sb0 * 32, g_hi = rmsnorm ? K / 8 : sb1 * 32; // groups of 8 columns to look at
    const bool resident = TT == 1 && g_hi - g_lo <= MAXG * GEMV_THREADS;
    float xr[TT == 1 ? MAXG : 1][8];
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        float ss = 0.f, amax = 0.f;
        if (TT == 1 && early) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int gi = sb0 * 32 + threadIdx.x + i * GEMV_THREADS;
                if (gi < sb1 * 32) {
                    const v4f v0 = ex[i][0], v1 = ex[i][1];
                    float *f = xr[TT == 1 ? i : 0];
                    f[0] = v0.x; f[1] = v0.y; f[2] = v0.z; f[3] = v0.w; f[4] = v1.x; f[5] = v1.y; f[6] = v1.z; f[7] = v1.w;
                    if (rmsnorm) {
                        ss += ((v0.x * v0.x + v0.y * v0.y) + (v0.z * v0.z + v0.w * v0.w)) + ((v1.x * v1.x + v1.y * v1.y) + (v1.z * v1.z + v1.w * v1.w));
                        const v4f g0 = eg[i][0], g1 = eg[i][1];
                        f[0] *= g0.x; f[1] *= g0.y; f[2] *= g0.z; f[3] *= g0.w; f[4] *= g1.x; f[5] *= g1.y; f[6] *= g1.z; f[7] *= g1.w;
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(f[e]));
                }
            }
        } else if (TT == 1 && resident) {
#pragma unroll
            for (int i = 0; i < MAXG; ++i) {
                const int gi = g_lo + threadIdx.x + i * GEMV_THREADS;
                if (gi < g_hi) {
                    if (rmsnorm) {
                        const float *xp = a.x + gi * 8;
                        const float4 v0 = *reinterpret_cast<const float4 *>(xp), v1 = *reinterpret_cast<const float4 *>(xp + 4);
                        ss += ((v0.x * v0.x + v0.y * v0.y) + (v0.z * v0.z + v0.w * v0.w)) + ((v1.x * v1.x + v1.y * v1.y) + (v1.z * v1.z + v1.w * v1.w));
                    }
                    if (gi >= sb0 * 32 && gi < sb1 * 32) {
                        load_act8(a, 0, gi * 8, xr[TT == 1 ? i : 0]);
#pragma unroll
                        for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(xr[TT == 1 ? i : 0][e]));
                    }
                }
            }
        } else {
            for (int gi = g_lo + threadIdx.x; gi < g_hi; gi += GEMV_THREADS) {
                float f[8];
                if (rmsnorm) {
                    const float *xp = a.x + t * a.ldx + gi * 8;
                    const float4 v0 = *reinterpret_cast<const float4 *>(xp), v1 = *reinterpret_cast<const float4 *>(xp + 4);
                    ss += ((v0.x * v0.x + v0.y * v0.y) + (v0.z * v0.z + v0.w * v0.w)) + ((v1.x * v1.x + v1.y * v1.y) + (v1.z * v1.z + v1.w * v1.w));
                }
                if (gi >= sb0 * 32 && gi < sb1 * 32) {
                    load_act8(a, t, gi * 8, f);
#pragma unroll
                    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(f[e]));
                }
            }
        }
        // both reductions in one round: wave shuffles here, one barrier and fixed-order sums below
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            ss += __shfl_xor(ss, off, 64);
            amax = fmaxf(amax, __shfl_xor(amax, off, 64));
        }
        float *red = l_red + t * 16;
        if (lane == 0) { red[wave] = ss; red[8 + wave] = amax; }
    }
    first_stages(NST - 1);

    // zero the partial sums and the zero operand
    if (threadIdx.x == 0) *l_next = STATIC_UNITS * GEMV_WAVES;
    if (threadIdx.x < 8) reinterpret_cast<uint32_t *>(l_zero)[threadIdx.x] = 0u;
    if (!a.direct)
        for (int i = threadIdx.x; i < n_units * TT * 16; i += GEMV_THREADS) l_part[i] = 0.f;

    lds_barrier();
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        const float *red = l_red + t * 16;
        float ss = red[0], amax = red[8];
#pragma unroll
        for (int i = 1; i < GEMV_WAVES; ++i) { ss += red[i]; amax = fmaxf(amax, red[8 + i]); } // fixed order
        const float inv_rms = rmsnorm ? 1.0f / sqrtf(ss / static_cast<float>(K) + a.eps) : 1.f;
        amax *= inv_rms; // max |x*gain| / rms
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
    lds_barrier();

    // lanes whose output slots hold this lane's k-group carry digits; all others feed zeros.
    // Digit r of sub-block S sits at byte ((r + S) & 3) * 32 of its 128 bytes (S = s0 + g with s0 % 4 == 0),
    // so the 16 reading lanes (4 k-groups x 4 digits) fall into different banks.
    const bool active = (j >> 2) == g;
    const int a_lane = active ? 32 + g * SUB_BYTES + (((j & 3) + g) & 3) * 32 : 0; // byte offset from l_zero
    const int a_mul = active ? 1 : 0;                                              // inactive lanes stay on the zeros
    const int fsh = 6 * g;

    // residual and store of one finished output of an EPI_ROWS launch (v already scaled back)
    auto out_row = [&](int tile, int jj, int t, float v) {
        int sg, tis;
        seg_of(tile, sg, tis);
        const int64_t n_rows = sg == 0 ? a.seg[0].n_rows : (sg == 1 ? a.seg[1].n_rows : a.seg[2].n_rows);
        const int64_t row = static_cast<int64_t>(tis) * 16 + jj;
        if (row < n_rows) {
            const float *resid = sg == 0 ? a.seg[0].resid : (sg == 1 ? a.seg[1].resid : a.seg[2].resid);
            float *y = sg == 0 ? a.seg[0].y : (sg == 1 ? a.seg[1].y : a.seg[2].y);
            const int64_t ldy = sg == 0 ? a.seg[0].ldy : (sg == 1 ? a.seg[1].ldy : a.seg[2].ldy);
            const int64_t ldr = sg == 0 ? a.seg[0].ldr : (sg == 1 ? a.seg[1].ldr : a.seg[2].ldr);
            if (resid) v += resid[t * ldr + row];
            y[t * ldy + row] = v;
        }
    };
    // EPI_SWIGLU: gate and up sums of row (pair, jj) -> silu(gate) * up
    auto out_pair = [&](int tile_even, int jj, int t, float gt, float up) {
        const int64_t row = static_cast<int64_t>(tile_even >> 1) * 16 + jj;
        if (row < a.seg[0].n_rows) a.seg[0].y[t * a.seg[0].ldy + row] = gt / (1.0f + expf(-gt)) * up;
    };
    const int64_t slab_stride = static_cast<int64_t>(a.n_tiles) * 16 * TT; // elements per slab in the global partial sums

    Cursor cc;
    start(cc);
    normalize(cc, false);
    int step = 0, st = 0;

    float yacc[TT], macc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) { yacc[t] = 0.f; macc[t] = 0.f; }

    {
        // ---- transform + quantise this slab's activations into LDS ----
        // digits [S][4][32 bytes]; byte order inside a digit row: for each group a of 8 values,
        // values 8a + {0,2,4,6,1,3,5,7}, the order in which the nibble split delivers the weights.
        auto quantise8 = [&](int t, int gi, const float *f, float S) {
            // xfix = rint(f*S) (one rounding to integer).  Its four signed base-256 digits are the bytes of
            // (xfix + 0x80808080) ^ 0x80808080: adding 128 to every digit makes them the unsigned bytes of
            // the biased number, and flipping bit 7 of a byte subtracts the 128 again in two's complement.
            uint32_t d4[8];
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float rf = rintf(f[e] * S);
                sum += rf; // per-sub-block sum of xfix, to fp32 accuracy
                d4[e] = (static_cast<uint32_t>(static_cast<int>(rf)) + 0x80808080u) ^ 0x80808080u;
            }
            const int s_glob = gi >> 2, s_loc = s_glob - sb0 * 8, grp = gi & 3;
            uint8_t *dp = l_dig + t * dig_t_stride + s_loc * SUB_BYTES + grp * 8;
#pragma unroll
            for (int dg = 0; dg < 4; ++dg) {
                // byte dg of values 0,2,4,6 and of values 1,3,5,7 (v_perm_b32 picks bytes of a register pair)
                const uint32_t sel = 0x0c0c0400u + 0x0101u * dg; // {byte dg of src1, byte dg of src0, 0, 0}
                const uint32_t e02 = __builtin_amdgcn_perm(d4[2], d4[0], sel), e46 = __builtin_amdgcn_perm(d4[6], d4[4], sel);
                const uint32_t e13 = __builtin_amdgcn_perm(d4[3], d4[1], sel), e57 = __builtin_amdgcn_perm(d4[7], d4[5], sel);
                uint2 o;
                o.x = e02 | (e46 << 16);
                o.y = e13 | (e57 << 16);
                *reinterpret_cast<uint2 *>(dp + ((dg + s_glob) & 3) * 32) = o;
            }
            sum += __shfl_xor(sum, 1, 64);
            sum += __shfl_xor(sum, 2, 64);
            if (grp == 0) l_xs[t * slab_sub + s_loc] = sum;
        };
        if (TT == 1 && early) {
            const float S = l_scale[0];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int gi = sb0 * 32 + threadIdx.x + i * GEMV_THREADS;
                if (gi < sb1 * 32) quantise8(0, gi, xr[TT == 1 ? i : 0], S);
            }
        } else if (TT == 1 && resident) {
            const float S = l_scale[0];
#pragma unroll
            for (int i = 0; i < MAXG; ++i) {
                const int gi = g_lo + threadIdx.x + i * GEMV_THREADS;
                if (gi >= sb0 * 32 && gi < sb1 * 32) quantise8(0, gi, xr[TT == 1 ? i : 0], S);
            }
        } else {
#pragma unroll
            for (int t = 0; t < TT; ++t) {
                const float S = l_scale[t];
                for (int gi = sb0 * 32 + threadIdx.x; gi < sb1 * 32; gi += GEMV_THREADS) {
                    float f[8];
                    load_act8(a, t, gi * 8, f);
                    quantise8(t, gi, f, S);
                }
            }
        }
        // the third stage goes out once this wave's digits are written; from here on a stage is refilled
        // as soon as it has been consumed
        normalize(lc, true);
        if (lc.valid) {
            issue(lc, NST - 1);
            lc.c += a.ksplit;
            ++issued;
        }
        lds_barrier();

        // ---- consume this wave's stages of the slab ----
        while (cc.valid) {
            const int newer = issued - (step + 1); // stages requested after the one consumed now
            if (newer >= 2) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
            else if (newer == 1) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            static_assert(NI == 5 && NST == 3, "the vmcnt immediates above assume 5 loads per stage, 3 stages");

            const int blk0 = sb0 + cc.c * PBS;
            const int nblk = min(PBS, sb1 - blk0);
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

            // next stage of this wave; leave the unit's sums in its slot when the unit ends
            const int u_done = cc.u;
            cc.c += a.ksplit;
            normalize(cc, false);
            if (!cc.valid || cc.u != u_done) {
                float *slot = l_part + u_done * (TT * 16);
                const int tile_done = tl0 + u_done / a.ksplit;
#pragma unroll
                for (int t = 0; t < TT; ++t) {
                    float v = yacc[t] - macc[t];
                    v += __shfl_xor(v, 16, 64);
                    v += __shfl_xor(v, 32, 64);
                    if (g == 0) {
                        if (!a.direct) slot[t * 16 + j] = v;                                  // the parts of a tile meet in LDS
                        else if (a.n_slabs == 1) out_row(tile_done, j, t, v * l_inv[t]);     // the wave owned the whole row: done
                        else __hip_atomic_store(a.part + slab * slab_stride + static_cast<int64_t>(tile_done) * 16 * TT + t * 16 + j, v * l_inv[t],
                                                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    yacc[t] = 0.f;
                    macc[t] = 0.f;
                }
            }
            normalize(lc, true);
            if (lc.valid) {
                issue(lc, st);
                lc.c += a.ksplit;
                ++issued;
            }
            st = (st + 1) % NST;
            ++step;
        }
    }
    lds_barrier();

    // ---- epilogue ----
    // this slab's sum of (local tile, element) over the parts in part order, scaled back to real units
    auto slab_sum = [&](int tile_local, int rem) {
        float v = 0.f;
        for (int p = 0; p < a.ksplit; ++p) v += l_part[(tile_local * a.ksplit + p) * (TT * 16) + rem];
        return v * l_inv[rem >> 4];
    };
    const int ngl = ntl / gran; // output groups (tiles, or gate/up pairs) of this workgroup
    if (a.n_slabs == 1) {
        if (a.direct) return;
        for (int idx = threadIdx.x; idx < ngl * 16 * TT; idx += GEMV_THREADS) {
            const int gl = idx / (16 * TT);
            const int rem = idx - gl * (16 * TT);
            const int t = rem >> 4, jj = rem & 15;
            if (pairs) out_pair(tl0 + 2 * gl, jj, t, slab_sum(2 * gl, rem), slab_sum(2 * gl + 1, rem));
            else out_row(tl0 + gl, jj, t, slab_sum(gl, rem));
        }
        return;
    }

    // several slabs: this slab's sums go to global memory; whoever arrives last at a tile (or pair) adds the slabs
    if (!a.direct)
        for (int idx = threadIdx.x; idx < ntl * 16 * TT; idx += GEMV_THREADS) {
            const int tile_local = idx / (16 * TT);
            const int rem = idx - tile_local * (16 * TT);
            __hip_atomic_store(a.part + slab * slab_stride + static_cast<int64_t>(tl0 + tile_local) * 16 * TT + rem, slab_sum(tile_local, rem),
                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    // The partial sums are written with device-scope (write-through) stores and read back with
    // device-scope loads, so they never sit in one XCD's L2 only; what is left to order is "all of this
    // workgroup's stores have completed" before its arrival is counted: vmcnt(0) + barrier.  (A release
    // fence would do the same but writes back and invalidates the whole L2 per workgroup.)
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const int grp0 = tl0 / gran;
    for (int gl = threadIdx.x; gl < ngl; gl += GEMV_THREADS) {
        const unsigned prev = __hip_atomic_fetch_add(a.arrivals + grp0 + gl, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = prev + 1 == static_cast<unsigned>(a.n_slabs);
        if (last) __hip_atomic_store(a.arrivals + grp0 + gl, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); // ready for the next launch
        l_part[gl] = last ? 1.f : 0.f; // l_part is free again after the barrier above
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    auto all_slabs = [&](int tile, int rem) {
        float v = 0.f;
        for (int sl = 0; sl < a.n_slabs; ++sl) // fixed order
            v += __hip_atomic_load(a.part + sl * slab_stride + static_cast<int64_t>(tile) * 16 * TT + rem, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return v;
    };
    for (int idx = threadIdx.x; idx < ngl * 16 * TT; idx += GEMV_THREADS) {
        const int gl = idx / (16 * TT);
        if (l_part[gl] == 0.f) continue;
        const int rem = idx - gl * (16 * TT);
        const int t = rem >> 4, jj = rem & 15;
        if (pairs) out_pair(tl0 + 2 * gl, jj, t, all_slabs(tl0 + 2 * gl, rem), all_slabs(tl0 + 2 * gl + 1, rem));
        else out_row(tl0 + gl, jj, t, all_slabs(tl0 + gl, rem));
    }
}

// ------------------------------------------------------------------------------------------
struct PPlan {
    int n_tiles, nb, n_wg, ksplit, slab_blocks, n_slabs, units_cap, direct;
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

static size_t fixed_lds(int T, int part_floats)
{
    return RING_BYTES + 32 + static_cast<size_t>(part_floats) * 4 + (16 * T + 2 * T) * 4 + (1 + GEMV_WAVES * FIFO) * 4 + 64;
}

// Decomposition of a launch: slabs of K (as few as the LDS allows), and waves per tile.  Candidates are
// ranked by the longest wave's share of the ideal time; more slabs cost partial-sum traffic.
static PPlan plan_for(int n_tiles, int nb, int T, int epi)
{
    const int gran = epi == EPI_SWIGLU ? 2 : 1; // tiles that stay together on a workgroup
    const int n_groups = n_tiles / gran;
    PPlan best{};
    best.ok = false;
    double best_score = 0.0;
    const int cus = device_cu_count();
    const size_t per_block = static_cast<size_t>(T) * 8 * (SUB_BYTES + 4);
    const double ideal = static_cast<double>(n_tiles) * ((nb + PBS - 1) / PBS) / (static_cast<double>(cus) * GEMV_WAVES);
    int n_min = 0; // the fewest slabs that fit; more (up to twice as many) only if they balance the waves better
    for (int n_slabs = 1; n_slabs <= 64 && (n_min == 0 || n_slabs <= 2 * n_min); ++n_slabs) {
        PPlan p{};
        p.nb = nb;
        p.n_tiles = n_tiles;
        p.n_slabs = n_slabs;
        p.n_wg = cus;
        if (p.n_wg > n_groups * n_slabs) p.n_wg = n_groups * n_slabs;
        if (p.n_wg < n_slabs) continue;
        const int wg_per_slab = p.n_wg / n_slabs;                     // the slabs with most tiles per workgroup
        const int tiles_wg = gran * ((n_groups + wg_per_slab - 1) / wg_per_slab);
        p.slab_blocks = ((nb + n_slabs - 1) / n_slabs + 1) & ~1;
        if ((nb + p.slab_blocks - 1) / p.slab_blocks != n_slabs) continue; // rounding to even merged two slabs
        const int chunks = (p.slab_blocks + PBS - 1) / PBS;
        for (int ks = 1; ks <= 4 * GEMV_WAVES && ks <= chunks; ks *= 2) {
            // ks == 1: a wave owns its tiles and stores their sums itself (a pair's two sums can only meet in
            // global memory, i.e. with several slabs); otherwise the parts meet in LDS
            const bool direct = ks == 1 && (gran == 1 || n_slabs > 1);
            const int part_floats = direct ? tiles_wg : tiles_wg * ks * T * 16;
            const size_t lds = fixed_lds(T, part_floats) + per_block * p.slab_blocks;
            if (lds > LDS_BUDGET || part_floats * 4 > 24 * 1024) continue;
            if (n_min == 0) n_min = n_slabs;
            if (n_min == 1 && n_slabs > 1) continue; // all of K fits: never pay for the reduction across workgroups
            const int units = tiles_wg * ks;
            const int rounds = (units + GEMV_WAVES - 1) / GEMV_WAVES;
            const double longest = static_cast<double>(rounds) * ((chunks + ks - 1) / ks);
            // waves take units as they finish: finer parts even out what the memory system does not
            const double score = ideal / longest * (1.0 - 0.03 * (n_slabs - n_min)) * (1.0 + 0.001 * ks);
            if (score > best_score + 1e-9) {
                best_score = score;
                best = p;
                best.ksplit = ks;
                best.direct = direct ? 1 : 0;
                best.units_cap = part_floats;
                best.lds_bytes = lds;
                best.ok = true;
            }
        }
    }
    return best;
}

static int tiles_of(const GemvArgs &ga)
{
    int n = 0;
    for (int i = 0; i < ga.nseg; ++i) n += static_cast<int>((ga.seg[i].n_rows + 15) / 16);
    return n;
}

// scratch in global memory: partial sums of the slabs and the per-tile arrival counters (which must be
// zero before the first launch and are left zero by every launch)
static size_t part_bytes(const PPlan &p, int T) { return round_up(static_cast<size_t>(p.n_slabs) * p.n_tiles * 16 * T * sizeof(float), 256); }
static size_t arrivals_bytes(int n_tiles) { return round_up(static_cast<size_t>(n_tiles) * sizeof(unsigned), 256); }

size_t gemv_ws_bytes(int64_t n_rows_total, int64_t n_cols, int T)
{
    // any segmentation of the rows into up to three matrices adds at most two tiles
    const int n_tiles = static_cast<int>((n_rows_total + 15) / 16) + 2;
    size_t worst = 0;
    for (int t0 = 0; t0 < T; t0 += MAX_T_PASS) {
        const int Tp = T - t0 < MAX_T_PASS ? T - t0 : MAX_T_PASS;
        for (int epi : {EPI_ROWS, EPI_SWIGLU}) {
            PPlan p = plan_for(n_tiles & ~1, static_cast<int>(n_cols / QK), Tp, epi);
            p.n_tiles = n_tiles;
            p.n_slabs += 1; // a slightly different tile count may need one more slab
            const size_t b = part_bytes(p, Tp);
            worst = b > worst ? b : worst;
        }
    }
    return arrivals_bytes(n_tiles) + worst;
}

size_t gemv_arrivals_bytes(int64_t n_rows_total) { return arrivals_bytes(static_cast<int>((n_rows_total + 15) / 16) + 2); }

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
    hipLaunchKernelGGL((gemv_q4k_persistent_kernel<TT>), dim3(p.n_wg), dim3(GEMV_THREADS), p.lds_bytes, st, a);
    return hipGetLastError();
}

prima_status launch_gemv_mfma(const GemvArgs &ga, void *ws, size_t ws_bytes, size_t arrivals_region, hipStream_t st)
{
    if (ga.xmode != X_PLAIN && ga.xmode != X_RMSNORM) return PRIMA_E_SHAPE;
    if (ga.epi == EPI_SWIGLU && (ga.nseg != 2 || ga.seg[0].n_rows != ga.seg[1].n_rows)) return PRIMA_E_SHAPE;
    if (ga.epi != EPI_SWIGLU && ga.epi != EPI_ROWS) return PRIMA_E_SHAPE;
    const int n_tiles = tiles_of(ga);
    // up to MAX_T_PASS tokens per pass over the weights
    for (int t0 = 0; t0 < ga.T; t0 += MAX_T_PASS) {
        const int T = ga.T - t0 < MAX_T_PASS ? ga.T - t0 : MAX_T_PASS;
        const PPlan p = plan_for(n_tiles, static_cast<int>(ga.n_cols / QK), T, ga.epi);
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
        a.epi = ga.epi;
        a.x = ga.x + t0 * ga.ldx;
        a.gain = ga.gain;
        a.ldx = ga.ldx;
        a.eps = ga.eps;
        a.ksplit = p.ksplit;
        a.slab_blocks = p.slab_blocks;
        a.n_slabs = p.n_slabs;
        a.units_cap = p.units_cap;
        a.direct = p.direct;
        a.n_wg = p.n_wg;
        if (p.n_slabs > 1) {
            // the counters sit in a region of fixed size at the start of the scratch, so that launches of
            // different shapes that share the scratch never write partial sums over each other's counters
            if (arrivals_region < arrivals_bytes(n_tiles)) return PRIMA_E_WORKSPACE;
            if (!ws || ws_bytes < arrivals_region + part_bytes(p, T)) return PRIMA_E_WORKSPACE;
            a.arrivals = static_cast<unsigned *>(ws);
            a.part = reinterpret_cast<float *>(static_cast<char *>(ws) + arrivals_region);
        }
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

__global__ void zero_u32_kernel(unsigned *p, size_t n)
{
    const size_t i = static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// the arrival counters at the start of a mat-vec workspace must be zero before its first use
prima_status launch_zero_arrivals(void *ws, size_t bytes, hipStream_t st)
{
    const size_t n = bytes / sizeof(unsigned);
    if (n == 0) return PRIMA_OK;
    hipLaunchKernelGGL(zero_u32_kernel, dim3(static_cast<unsigned>((n + 255) / 256)), dim3(256), 0, st, static_cast<unsigned *>(ws), n);
    return last_launch_status();
}

} // namespace prima
