// Declarations of the Q4_K mat-vec kernels (the design is described in q4k_gemv_mfma.hip); the body of the
// mat-vec itself is gemv_body.inc.
#pragma once
#include <atomic>
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
    int defer;       // n_slabs > 1: the slabs are added by a second kernel instead of the workgroup that arrives last
    int n_wg;
    // tile ranges, divided on the host: workgroup w has slab w % n_slabs and rank w / n_slabs = umulhi(w, slab_magic);
    // slabs below wg_more have one workgroup more than the others; class c (0: one more, 1: the others) gives every
    // workgroup grp_base[c] groups of tiles (tiles, or gate/up pairs) and the first grp_extra[c] ranks one more
    uint32_t slab_magic;
    int wg_more, grp_base[2], grp_extra[2];
    // How a slab's groups are dealt to its workgroups.  interleave != 0: rank r takes groups r, r + grp_stride[c],
    // r + 2 grp_stride[c], ... (at any moment the workgroups then read one window of the matrix that moves through it,
    // which loads the memory channels evenly: without it whole XCDs finish a launch 10 % apart); 0: a contiguous run
    // (launches whose slabs are added in place: the arrival counters of a workgroup then share cache lines).
    int interleave, grp_stride[2];
    float *part;        // n_slabs > 1: partial sums [n_slabs][n_tiles*16][T]
    unsigned *arrivals; // n_slabs > 1: per-tile arrival counters, zero between launches
};

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

// Tells the compiler that a pointer obtained as a plain value (e.g. read from the kernel-argument segment by
// hand) points to global memory: generic loads count on both memory counters and every wait would then
// drain the weight stream.
template <class T>
__device__ __forceinline__ T *as_global(T *p)
{
    return (T *)(__attribute__((address_space(1))) T *)p;
}

__device__ __forceinline__ long pack64(uint32_t lo, uint32_t hi)
{
    return static_cast<long>(static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32));
}

// eight consecutive activations of token t starting at column c0, before the RMSNorm scale:
// X_PLAIN x, X_RMSNORM x*gain (the 1/rms factor is applied by the caller)
// Sum of the squares of eight values in one fixed sequence of roundings (explicit fused multiply-adds and additions:
// left to the compiler, each copy of the expression may be contracted differently, and workgroups that look at the
// same row through different copies would disagree in the last bit of 1/rms).
template <typename V4>
__device__ __forceinline__ float sumsq8(const V4 &v0, const V4 &v1)
{
    const float a = __fmaf_rn(v0.x, v0.x, __fmul_rn(v0.y, v0.y)), b = __fmaf_rn(v0.z, v0.z, __fmul_rn(v0.w, v0.w));
    const float c = __fmaf_rn(v1.x, v1.x, __fmul_rn(v1.y, v1.y)), d = __fmaf_rn(v1.z, v1.z, __fmul_rn(v1.w, v1.w));
    return __fadd_rn(__fadd_rn(a, b), __fadd_rn(c, d));
}

__device__ __forceinline__ void load_act8(const float *x, const float *gain, int64_t ldx, bool rmsnorm, int t, int c0, float *f)
{
    const float *xp = x + t * ldx + c0;
    const float4 v0 = *reinterpret_cast<const float4 *>(xp), v1 = *reinterpret_cast<const float4 *>(xp + 4);
    f[0] = v0.x; f[1] = v0.y; f[2] = v0.z; f[3] = v0.w; f[4] = v1.x; f[5] = v1.y; f[6] = v1.z; f[7] = v1.w;
    if (rmsnorm) {
        const float4 g0 = *reinterpret_cast<const float4 *>(gain + c0), g1 = *reinterpret_cast<const float4 *>(gain + c0 + 4);
        const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] *= gg[e];
    }
}

// segment sg and tile-in-segment tis of a tile: (gate, up) pairs sit on tiles 2p, 2p + 1; otherwise the
// segments follow each other, t1 and t2 being the first tiles of segments 1 and 2
__device__ __forceinline__ void tile_segment(bool pairs, int nseg, int t1, int t2, int tile, int &sg, int &tis)
{
    if (pairs) { sg = tile & 1; tis = tile >> 1; return; }
    sg = 0; tis = tile;
    if (nseg > 1 && tile >= t1) { sg = 1; tis = tile - t1; }
    if (nseg > 2 && tile >= t2) { sg = 2; tis = tile - t2; }
}

// position of a wave in its stream of stages: k-th unit (tile, part) the wave took -> chunk of PBS super-blocks
struct Cursor {
    int k, u, c;
    bool valid;
};
constexpr int STATIC_UNITS = NST; // units per wave assigned by position (up to one per ring stage may be
                                  // requested before the counter exists); the rest go to whichever wave asks first
constexpr int FIFO = 8;         // units a wave may have requested and not yet consumed (a power of two > NST)

// ------------------------------------------------------------------------------------------
constexpr int DEFER_MIN_TILES = 6; // several tokens: more tiles per workgroup than this and a second kernel adds the slabs (measured with 6 and 16: at 16 the down projection of a 5120-wide model and the output projection of an 8192-wide one at 8 tokens get 2 and 6 us slower)

struct PPlan {
    int n_tiles, nb, n_wg, ksplit, slab_blocks, n_slabs, units_cap, direct;
    size_t lds_bytes;
    bool ok;
};

// compute units of the device that is current at the first call (the library serves one device per process)
inline int device_cu_count()
{
    static std::atomic<int> cached{0};
    int cus = cached.load(std::memory_order_relaxed);
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
        cached.store(cus, std::memory_order_relaxed);
    }
    return cus;
}

inline size_t fixed_lds(int T, int part_floats)
{
    return RING_BYTES + 32 + static_cast<size_t>(part_floats) * 4 + (16 * T + 2 * T) * 4 + (1 + GEMV_WAVES * FIFO) * 4 + 64;
}

// Decomposition of a launch: slabs of K (as few as the LDS allows), and waves per tile.  Candidates are
// ranked by the longest wave's share of the ideal time; more slabs cost partial-sum traffic.
inline PPlan plan_for(int n_tiles, int nb, int T, int epi)
{
    const int gran = epi == EPI_SWIGLU ? 2 : 1; // tiles that stay together on a workgroup
    const int n_groups = n_tiles / gran;
    PPlan best{};
    best.ok = false;
    double best_score = 0.0;
    const int cus = device_cu_count();
    const int Tq = T == 1 ? 1 : (T + 3) / 4 * 4; // token slots laid out in LDS (several tokens: groups of four)
    const size_t per_block = static_cast<size_t>(Tq) * 8 * (SUB_BYTES + 4);
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
        // The last slab may be shorter.  Every part of a unit must hold at least one chunk in every slab: the kernel's
        // two cursors (requesting and consuming) exchange the units they take through a short queue in LDS, sized for
        // the few units that the ring's stages can span; units without chunks would let the requesting cursor run
        // past the queue's end (wrong sums, and tile numbers read from slots nobody wrote).
        const int chunks_last = (nb - (n_slabs - 1) * p.slab_blocks + PBS - 1) / PBS;
        for (int ks = 1; ks <= 4 * GEMV_WAVES && ks <= chunks && ks <= chunks_last; ks *= 2) {
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


inline int tiles_of(const GemvArgs &ga)
{
    int n = 0;
    for (int i = 0; i < ga.nseg; ++i) n += static_cast<int>((ga.seg[i].n_rows + 15) / 16);
    return n;
}

// scratch in global memory: partial sums of the slabs and the per-tile arrival counters (which must be
// zero before the first launch and are left zero by every launch)
inline size_t part_bytes(const PPlan &p, int T) { return round_up(static_cast<size_t>(p.n_slabs) * p.n_tiles * 16 * T * sizeof(float), 256); }
inline size_t arrivals_bytes(int n_tiles) { return round_up(static_cast<size_t>(n_tiles) * sizeof(unsigned), 256); }


// Arguments and plan of one pass (tokens t0 .. t0+T-1, T <= MAX_T_PASS) of a mat-vec.  ws: scratch whose
// first arrivals_region bytes are the (zero) arrival counters, the slabs' partial sums follow.
inline prima_status build_pass(const GemvArgs &ga, int t0, int T, void *ws, size_t ws_bytes, size_t arrivals_region,
                               PGemvArgs &a, PPlan &p)
{
    if (ga.xmode != X_PLAIN && ga.xmode != X_RMSNORM) return PRIMA_E_SHAPE;
    if (ga.epi == EPI_SWIGLU && (ga.nseg != 2 || ga.seg[0].n_rows != ga.seg[1].n_rows)) return PRIMA_E_SHAPE;
    if (ga.epi != EPI_SWIGLU && ga.epi != EPI_ROWS) return PRIMA_E_SHAPE;
    const int n_tiles = tiles_of(ga);
    p = plan_for(n_tiles, static_cast<int>(ga.n_cols / QK), T, ga.epi);
    if (!p.ok) return PRIMA_E_SHAPE;
    if (static_cast<int64_t>(n_tiles) * (p.n_wg + 1) >= (int64_t{1} << 31)) return PRIMA_E_SHAPE; // the kernel's 32-bit tile arithmetic
    for (int i = 0; i < ga.nseg; ++i) // the kernel's 32-bit row numbers and offsets in 16-byte units (16 rows past the end included)
        if (ga.seg[i].n_rows >= (int64_t{1} << 31) - 16 || (ga.seg[i].n_rows + 16) * (ga.n_cols / QK) * 9 >= (int64_t{1} << 32)) return PRIMA_E_SHAPE;
    // what the kernel's unit queue relies on (plan_for sees to it): every part of a unit has a chunk in every slab
    if (p.ksplit > (p.nb - (p.n_slabs - 1) * p.slab_blocks + PBS - 1) / PBS) return PRIMA_E_SHAPE;
    if (p.ksplit < 1 || (p.ksplit & (p.ksplit - 1))) return PRIMA_E_SHAPE; // the kernel finds a unit's tile and part by shift and mask
    a = PGemvArgs{};
    int tile0 = 0;
    for (int i = 0; i < ga.nseg; ++i) {
        a.seg[i] = ga.seg[i];
        if (a.seg[i].y) a.seg[i].y += t0 * ga.seg[i].ldy;
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
    // Several tokens: a workgroup has many tiles and the slabs finish together, so "whoever arrives last" is
    // one workgroup for nearly all of them (measured: the slowest one adds for 50-70 us while the rest idle);
    // a second small launch does the additions in parallel instead.
    // With few tiles per workgroup (the Q/K/V and output projections of a 5120-wide model: 3 or 4) the arrivals are
    // spread over the workgroups and adding in place is cheaper than the second launch's hand-over.
    const int tiles_per_wg = (p.n_tiles * p.n_slabs + p.n_wg - 1) / p.n_wg;
    a.defer = (p.n_slabs > 1 && T > 1 && tiles_per_wg > DEFER_MIN_TILES) ? 1 : 0;
    a.n_wg = p.n_wg;
    {
        const int gran = ga.epi == EPI_SWIGLU ? 2 : 1, n_groups = n_tiles / gran;
        const int q = p.n_wg / p.n_slabs; // >= 1: plan_for keeps n_wg >= n_slabs
        a.slab_magic = static_cast<uint32_t>(((uint64_t{1} << 32) + p.n_slabs - 1) / p.n_slabs); // exact for w < 2^32 / n_slabs
        if (static_cast<int64_t>(p.n_wg) * p.n_slabs >= (int64_t{1} << 32)) return PRIMA_E_SHAPE;
        a.wg_more = p.n_wg % p.n_slabs;
        a.grp_base[0] = n_groups / (q + 1);
        a.grp_extra[0] = n_groups % (q + 1);
        a.grp_base[1] = n_groups / q;
        a.grp_extra[1] = n_groups % q;
        a.grp_stride[0] = q + 1;
        a.grp_stride[1] = q;
        a.interleave = (p.n_slabs == 1 || a.defer) ? 1 : 0;
    }
    if (p.n_slabs > 1) {
        // the counters sit in a region of fixed size at the start of the scratch, so that launches of
        // different shapes that share the scratch never write partial sums over each other's counters
        if (arrivals_region < arrivals_bytes(n_tiles)) return PRIMA_E_WORKSPACE;
        if (!ws || ws_bytes < arrivals_region + part_bytes(p, T)) return PRIMA_E_WORKSPACE;
        a.arrivals = static_cast<unsigned *>(ws);
        a.part = reinterpret_cast<float *>(static_cast<char *>(ws) + arrivals_region);
    }
    return PRIMA_OK;
}

} // namespace prima
