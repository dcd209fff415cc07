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
// split is done once, not once per row block.  (3) the product: a workgroup of 4 waves owns 256 rows x 64 tokens,
// a wave 64 rows (four B tiles in registers: every A tile read from LDS feeds four MFMAs per part); two workgroups
// share a compute unit, so that one's VALU and LDS phases run under the other's MFMAs.  The super-block is walked
// sub-block by sub-block; global->LDS loads fill a ring of activation slots two positions ahead and, per wave,
// two buffers with half a super-block of its rows' quants each (the comment at the kernel has the details).  Workgroups are numbered so
// that those running on one XCD (one L2) at a time are patches of 4 row blocks x 8 token blocks.  Up to three
// matrices with the same columns share a launch (Q / K / V), and so do a gate and an up matrix, with SwiGLU behind.
// The weights stay exact: dequantised to binary16 (one accumulator for all of K) they would be off by ~1e-3 per
// product, measured in the metric of the tests.
#include <hip/hip_fp16.h>

#include <atomic>
#include <type_traits>

#include "common.h"

namespace prima {
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int GM_THREADS = 256;
constexpr int GM_WAVES = GM_THREADS / 64;       // one wave per SIMD and workgroup
constexpr int GM_RT = 4;                        // 16-row tiles per wave
constexpr int GM_TT = 4;                        // 16-token tiles per workgroup
constexpr int GM_ROWS = 16 * GM_RT * GM_WAVES;  // rows per workgroup
constexpr int GM_TM = 16 * GM_TT;               // tokens per workgroup
constexpr int GM_SLABS = 17;                    // per (token tile, super-block): 8 sub-blocks x (hi, lo), sums
constexpr int GM_TILE_BYTES = GM_SLABS * 1024;
constexpr int GM_NS = 3;                        // ring slots: positions whose activations are in LDS or on their way (a divisor
                                                // of the 9 positions of a super-block: the slot of a position is a constant; 4
                                                // and 5 slots measured the same)
constexpr int GM_SLOT = GM_TT * 2048;                                     // 8 KiB of activations
constexpr int GM_WQ = 2 * 4096;                                           // per wave: the quants of half a super-block, twice
constexpr int GM_LDS_BYTES = GM_NS * GM_SLOT + GM_WAVES * (GM_WQ + 2 * 1024); // 64 KiB: two workgroups per compute unit
constexpr int GM_XCDS = 8;
constexpr int GM_CUS = 256;
// Workgroups that share an XCD at a time: a patch of 4 row blocks x 8 token blocks; with fewer than 8 token blocks all of
// them and more row blocks, with few row blocks per XCD only those.  A workgroup number that falls outside the matrix
// costs its dispatch (about 0.1 us): with one token block and patches of 4 x 8, seven numbers in eight were idle and a
// launch took no less than 260 us whatever its work.
constexpr int GM_PATCH = 32, GM_PATCH_C = 8;
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
    int patch_r, patch_c;       // row blocks x token blocks of a patch
    // K divided among ksplit workgroups per (row block, token block): workgroup blockIdx.y walks its share of the
    // super-blocks and stores its sums to part[split][token][ldp] (column: row block * GM_ROWS + row in the block);
    // gemm_ksplit_reduce_kernel adds the shares in order.  ksplit == 1: the sums go straight to y.
    int ksplit;
    float *part;
    int64_t ldp;
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

// 16 bytes per lane from global memory straight into LDS (as dma16), with the address as a wave-uniform base plus a
// 32-bit lane offset: the bases live in scalar registers and cost no vector register per request in flight
__device__ __forceinline__ void dma16_base(const void *sbase, uint32_t lane_off, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_off), "s"(sbase), "s"(lds_addr) : "memory");
}
// ... and with a per-lane pointer plus a constant byte offset (0 .. 4095) in the instruction.  The instruction adds
// its offset to the LDS address as well as to the global one, so M0 gets the LDS address less the offset.
template <int OFF>
__device__ __forceinline__ void dma16_off(const void *gptr, uint32_t lds_addr)
{
    static_assert(OFF >= 0 && OFF < 4096, "instruction offset");
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off offset:%2" : : "v"(gptr), "s"(lds_addr - OFF), "n"(OFF) : "memory");
}

// Requests a wave makes at the positions p - 3 .. p - 1 behind position p = (b, s) of the product kernel's schedule
// (activations four positions ahead: 2, or 1 where the target is the sums position; at s == 3, 4, 7 of a super-block with
// a successor 4, 1, 4 weight requests).  successor: whether super-block b has one; the one before b always had.
constexpr int GM_AHEAD = GM_NS - 1; // positions between an activation request and its use
constexpr int requests_at(int sk, bool successor) // sk < 0: a position of the super-block before (or the prologue)
{
    const int sp = sk < 0 ? sk + 9 : sk;
    return ((sp + GM_AHEAD) % 9 < 8 ? 2 : 1) + ((sk < 0 || successor) ? (sp == 3 ? 4 : (sp == 4 ? 1 : (sp == 7 ? 4 : 0))) : 0);
}
constexpr int requests_behind(int s, bool successor)
{
    int n = 0;
    for (int k = 1; k < GM_AHEAD; ++k) n += requests_at(s - k, successor);
    return n;
}
static_assert(GM_AHEAD != 4 ||
                  (requests_behind(0, true) == 10 && requests_behind(0, false) == 10 && requests_behind(2, true) == 6 &&
                   requests_behind(4, true) == 10 && requests_behind(4, false) == 6 && requests_behind(5, false) == 5 &&
                   requests_behind(7, true) == 6 && requests_behind(8, true) == 10 && requests_behind(8, false) == 6),
              "request counts of the product kernel's schedule");
static_assert(GM_AHEAD >= 2 && GM_AHEAD <= 4, "the weight requests at s == 3, 4, 7 must be older than the activation requests a wait lets pass");

// workgroup barrier that orders LDS traffic only (__syncthreads() would also wait for every global load in flight,
// that is, for the whole ring of requests below)
__device__ __forceinline__ void gm_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One workgroup: 4 waves, one per SIMD; a wave owns 64 rows (four B tiles) x 64 tokens, i.e. 16 accumulator tiles for the
// super-block in hand and as many running sums; two workgroups share a compute unit (237 registers per wave, 64 KiB of
// LDS per workgroup) and run out of step with each other.  The super-block is walked sub-block by sub-block ("positions"
// 0..7, then position 8: the sums slab and the min term).  Everything comes through LDS by 16-byte global->LDS loads:
//   activations: a ring of NS slots of 8 KiB, [4 token tiles][hi 1 KiB | lo 1 KiB] of a sub-block, shared by the four
//     waves, requested NS - 1 positions ahead (position 8 uses the slot's first 4 KiB for the sums slabs);
//   quants: per wave two buffers of 4 KiB, sub-blocks 0-3 and 4-7 of its 64 rows, each filled by four requests of 64
//     bytes x 16 rows as soon as the B tiles of the half super-block before have been built from it;
//   headers: 64 rows x 16 bytes per wave and super-block, a ring of two.
// Per position: wait until everything this wave requested four positions ago or earlier has landed (requests complete
// in order; the wait names the number of requests made since, which the schedule fixes), barrier (everyone's share of
// the activations is there, and everyone has finished reading the slot of the position before, which is the slot
// requested next), the position's requests, and then, token tile by token tile, the MFMAs of this position with,
// between them, the VALU work that builds the B tiles of the next position.  No global load is left for the compiler
// to wait on.  Measured with parts of the work switched off (8192 x 28672 weights, 1024 tokens): the LDS reads of the
// activations cost 30 % of the time, the requests 12 %, the B tiles 10 %, the barrier 3 %: a wave reads every
// activation of its 64 tokens once per position, whatever the tiling, so LDS bandwidth is met before the MFMA rate.
__global__ void __launch_bounds__(GM_THREADS, 2) q4k_gemm_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int TT = GM_TT;
    constexpr int SLOT = GM_SLOT;
    constexpr int WQ_BASE = GM_NS * SLOT;            // per wave two buffers of 4 KiB: quants of sub-blocks 0-3, of 4-7
    constexpr int HDR_RING = WQ_BASE + GM_WAVES * GM_WQ; // two entries of GM_WAVES KiB
    constexpr int DM = TT / 2, DMS = TT / 4;         // activation requests per wave: a sub-block position, the sums position
    static_assert(TT == 4 && GM_WAVES == 4, "requests per wave and position are counted for 4 tiles and 4 waves");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 15, g = lane >> 4;
    // Consecutive workgroup numbers go to consecutive XCDs.  32 consecutive workgroups of one XCD (one L2) are 4 row
    // blocks x 8 token blocks: per super-block step they fetch 4 x 36 KiB of weights and 8 x 68 KiB of activations
    // between them instead of 32 of either.  An XCD owns the row blocks xcd, xcd + 8, ...  (The shape of the patch
    // makes no measurable difference at 1024 tokens; this one is the best of four at 512.  The host narrows the patch
    // when there are fewer token blocks or row blocks than that, so that few workgroup numbers fall outside.)
    const int xcd = blockIdx.x % GM_XCDS, seq = blockIdx.x / GM_XCDS;
    const int patch_c = a.patch_c, patch_r = a.patch_r;
    const int patch = seq / (patch_r * patch_c), within = seq % (patch_r * patch_c);
    const int patches_tb = (a.n_tb + patch_c - 1) / patch_c;
    const int rb = ((patch / patches_tb) * patch_r + within / patch_c) * GM_XCDS + xcd;
    const int tb = (patch % patches_tb) * patch_c + within % patch_c;
    if (rb >= a.n_rb || tb >= a.n_tb) return; // the whole workgroup, before any barrier
    const int nb = static_cast<int>(a.n_cols >> 8);
    const int sg = a.pair ? 0 : (rb >= a.seg[2].rb0 ? 2 : (rb >= a.seg[1].rb0 ? 1 : 0));
    const GemmSegDev &my = a.seg[sg];
    // first row of this wave: 64 rows of one matrix, or (pair) the same 32 rows of the gate and of the up matrix
    const int64_t row0 = a.pair ? static_cast<int64_t>(rb) * (GM_ROWS / 2) + wave * 32
                                : static_cast<int64_t>(rb - my.rb0) * GM_ROWS + wave * 64;
    // Weight requests of this lane.  Headers: 16 bytes of local row `lane`.  Quants: request k of a half super-block
    // brings 64 bytes (four sub-blocks) of each of the local rows 16k .. 16k+15, this lane the 16 bytes of sub-block
    // (lane & 3) of row 16k + (lane >> 2): 16 runs of 64 bytes per request (16 bytes of each of 64 rows per request cost
    // about 12 % at 1024 tokens and more).  Local row r: row0 + r of the matrix, or (pair) row0 + (r & 31) of the gate
    // (r < 32) or the up matrix; past the end: a valid row, not stored.
    auto row_ptr = [&](int r) __attribute__((always_inline)) -> const uint8_t * {
        const int64_t gr = min<int64_t>(row0 + (a.pair ? (r & 31) : r), my.n_rows - 1);
        return (a.pair ? a.seg[r >> 5].W : my.W) + gr * nb * 144;
    };
    const uint8_t *wsrc = row_ptr(lane);
    const uint8_t *wq[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) wq[k] = row_ptr(16 * k + (lane >> 2)) + 16 + (lane & 3) * 16;
    const int tile0 = tb * TT;
    const uint32_t lds0 = lds_address(smem);
    // this workgroup's share of K: super-blocks [b_lo, b_lo + nbl) (all of them unless K is divided; never empty: the
    // host keeps ksplit <= nb); below, `b` counts from b_lo
    const int b_lo = static_cast<int>(static_cast<int64_t>(blockIdx.y) * nb / a.ksplit);
    const int nbl = static_cast<int>(static_cast<int64_t>(blockIdx.y + 1) * nb / a.ksplit) - b_lo;
    wsrc += static_cast<int64_t>(b_lo) * 144;
#pragma unroll
    for (int k = 0; k < 4; ++k) wq[k] += static_cast<int64_t>(b_lo) * 144;
    const int total = 9 * nbl; // positions (n_cols < 2^32: no overflow)

    // Wave-uniform bases of this wave's activation requests: request jj of a sub-block position is slab (part, tile)
    // with part = wave & 1, tile = 2 jj + (wave >> 1); request jj of a sums position is tile wave + 4 jj.  Past the
    // last tile: a valid one, not stored.
    const uint8_t *abase[DM], *xbase[DMS];
#pragma unroll
    for (int jj = 0; jj < DM; ++jj) {
        const int tg = min(tile0 + 2 * jj + (wave >> 1), a.n_tiles - 1);
        abase[jj] = a.A + ((static_cast<int64_t>(tg) * nb + b_lo) * GM_SLABS + (wave & 1)) * 1024;
    }
#pragma unroll
    for (int jj = 0; jj < DMS; ++jj) {
        const int tg = min(tile0 + wave + GM_WAVES * jj, a.n_tiles - 1);
        xbase[jj] = a.A + ((static_cast<int64_t>(tg) * nb + b_lo) * GM_SLABS + 16) * 1024;
    }
    const uint32_t lane16 = lane * 16;

    // the quants of half `half` (sub-blocks 4 half .. 4 half + 3) of super-block b: four requests; its headers: one
    auto issue_quants = [&](int b, int half) __attribute__((always_inline)) {
        const uint32_t dst = lds0 + WQ_BASE + wave * GM_WQ + half * 4096;
        const int64_t off = static_cast<int64_t>(b) * 144;
        if (half == 0) {
            dma16_off<0>(wq[0] + off, dst);
            dma16_off<0>(wq[1] + off, dst + 1024);
            dma16_off<0>(wq[2] + off, dst + 2048);
            dma16_off<0>(wq[3] + off, dst + 3072);
        } else {
            dma16_off<64>(wq[0] + off, dst);
            dma16_off<64>(wq[1] + off, dst + 1024);
            dma16_off<64>(wq[2] + off, dst + 2048);
            dma16_off<64>(wq[3] + off, dst + 3072);
        }
    };
    auto issue_headers = [&](int b) __attribute__((always_inline)) {
        dma16_off<0>(wsrc + static_cast<int64_t>(b) * 144, lds0 + HDR_RING + ((b & 1) * GM_WAVES + wave) * 1024);
    };
    // the activation requests of position (b, s), into ring slot `slot` (s is a constant wherever this is called)
    auto issue = [&](int b, int s, int slot) __attribute__((always_inline)) {
        const uint32_t base = lds0 + slot * SLOT;
        const int64_t boff = static_cast<int64_t>(b) * (GM_SLABS * 1024);
        if (s < 8) {
#pragma unroll
            for (int jj = 0; jj < DM; ++jj)
                dma16_base(abase[jj] + boff + 2048 * s, lane16, base + (2 * jj + (wave >> 1)) * 2048 + (wave & 1) * 1024);
        } else {
#pragma unroll
            for (int jj = 0; jj < DMS; ++jj) dma16_base(xbase[jj] + boff, lane16, base + (wave + GM_WAVES * jj) * 1024);
        }
    };

    v4f yacc[TT][GM_RT], acch[TT][GM_RT];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
        for (int rt = 0; rt < GM_RT; ++rt) yacc[tt][rt] = acch[tt][rt] = {0.f, 0.f, 0.f, 0.f};

    // Requests complete in the order in which a wave made them, and every wait below names how many of the newest may
    // still be out.  Per position (b, s), behind the barrier: the activations of position p + NS - 1; at s == 3 the first
    // half of super-block b + 1's quants (their buffer was last read for position (b, 3), built during (b, 2)), at
    // s == 4 its headers, at s == 7 the second half (last read during (b, 6)).  The prologue makes its requests in the
    // order a super-block before this one would have: headers, first half, then the activations of the first NS - 1
    // positions with the second half where position (b - 1, 7) would have requested it.
    issue_headers(0);
    issue_quants(0, 0);
#pragma unroll
    for (int q = 0; q < GM_AHEAD; ++q) {
        issue(0, q, q);
        if (q == GM_AHEAD - 2) issue_quants(0, 1); // as position (b - 1, 7) would have
    }

    // B tile `rt` of sub-block s from this wave's quants and its headers of super-block `bb`:
    // sc_s * q as binary16 (exact).  A dword holds the eight weights of lane (n, g); masked in pairs (0,4) (1,5) (2,6)
    // (3,7) into the mantissas of 1024 + q, then one fused multiply-add per pair: (1024 + q) sc - 1024 sc
    auto build_b = [&](half8 &B, int rt, int bb, int s) __attribute__((always_inline)) {
        // request rt of the half brought rows 16 rt .. 16 rt + 15: [row][sub-block of the half][16 bytes]
        const uint32_t w = *reinterpret_cast<const uint32_t *>(smem + WQ_BASE + wave * GM_WQ + (s >> 2) * 4096 + rt * 1024 + n * 64 + (s & 3) * 16 + 4 * g);
        const uint4 hdr = *reinterpret_cast<const uint4 *>(smem + HDR_RING + ((bb & 1) * GM_WAVES + wave) * 1024 + (16 * rt + n) * 16);
        const _Float16 sc = static_cast<_Float16>(static_cast<float>(hdr_field(hdr, s)));
        const half2v sc2 = {sc, sc};
        const _Float16 off = static_cast<_Float16>(-1024.f) * sc; // exact: at most 64512 in magnitude
        const half2v off2 = {off, off};
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
            const uint32_t bits = ((w >> (4 * pr)) & 0x000f000fu) | 0x64006400u;
            const half2v r = __builtin_elementwise_fma(__builtin_bit_cast(half2v, bits), sc2, off2);
            B[2 * pr] = r[0];
            B[2 * pr + 1] = r[1];
        }
    };
    // ... and of the sums position: the m_s as B operand, with d and dmin
    auto build_m = [&](half8 &B, float &d_, float &dm_, int rt, int bb) __attribute__((always_inline)) {
        const uint4 hdr = *reinterpret_cast<const uint4 *>(smem + HDR_RING + ((bb & 1) * GM_WAVES + wave) * 1024 + (16 * rt + n) * 16);
        d_ = hdr_d(hdr);
        dm_ = hdr_dmin(hdr);
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8) B[s8] = static_cast<_Float16>(static_cast<float>(hdr_field(hdr, 8 + s8)));
    };

    // The wave is alone on its SIMD and issues in order: an MFMA occupies the matrix pipe for 16 cycles, during which
    // the same wave can issue three or four other instructions for free, and only then.  So the B tiles of position
    // p + 1 are built (VALU) between the MFMAs of position p, in the order the scheduling groups below prescribe;
    // built in front of their own MFMAs they would cost their full issue time with the matrix pipe idle.  The quants
    // and headers that position p + 1 needs are this wave's own requests; the wait below covers them.
    half8 Bc[GM_RT];     // B tiles of the current position (at the sums position: the m_s)
    float dd[GM_RT], dm[GM_RT];
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(GM_AHEAD * DM + 4) : "memory"); // headers and first half of super-block 0 have landed
#pragma unroll
    for (int rt = 0; rt < GM_RT; ++rt) build_b(Bc[rt], rt, 0, 0);

    for (int b = 0; b < nbl; ++b) {
        // one position; s as a constant of the type system (a loop over s with "#pragma unroll" is refused by the
        // optimizer once its body, which holds every case of s until it is unrolled, passes a size limit)
        auto position = [&](auto s_const) __attribute__((always_inline)) {
            constexpr int s = decltype(s_const)::value;
            constexpr int slot = s % GM_NS; // ring slot of this position
            static_assert(9 % GM_NS == 0, "a position's slot must not depend on the super-block");
            const int p = 9 * b + s;
            // Everything requested at position p - 4 or before has landed (this wave's share of position p's
            // activations; the quants and headers that the B tiles built during this position need are older) once at
            // most the requests of positions p - 3 .. p - 1 are out: their activation requests (DM each, DMS where the
            // target is a sums position) and, where they fall on s == 3, 4, 7 of a super-block that has a successor,
            // 4, 1, 4 weight requests.  The last three positions wait for everything.
            if (p + GM_AHEAD - 1 >= total) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            else if (b + 1 < nbl) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(requests_behind(s, true)) : "memory");
            else asm volatile("s_waitcnt vmcnt(%0)" : : "n"(requests_behind(s, false)) : "memory"); // the last super-block requests no weights
            gm_barrier();
            {
                // position p + NS - 1 goes into the slot that position p - 1 has just left
                const int s_t = (s + GM_NS - 1) % 9;
                const int b_t = b + (s + GM_NS - 1) / 9;
                constexpr int slot_t = (slot + GM_NS - 1) % GM_NS;
                if (b_t < nbl) issue(b_t, s_t, slot_t);
                if (b + 1 < nbl) {
                    if (s == 3) issue_quants(b + 1, 0);
                    if (s == 4) issue_headers(b + 1);
                    if (s == 7) issue_quants(b + 1, 1);
                }
            }
            const uint8_t *base = smem + slot * SLOT + lane * 16;
            const v4f zero = {0.f, 0.f, 0.f, 0.f};
            half8 Bn[GM_RT];
            // Token tile by token tile, each a scheduling region of its own (the scheduler, left alone, hoists all of
            // a position's LDS reads and runs out of registers): the tile's MFMAs, the LDS reads of the next tile, and
            // during the first four tiles one B tile of the next position each.
            if (s < 8) {
                // The hi and the lo parts alternate in one accumulator: 16 fp32 roundings per super-block at the
                // accumulator's magnitude.  Accumulators of their own for the lo parts (whose sums are 2^-11 of the hi
                // sums, so that only 8 roundings count) lower the product's rms error from 2.2e-7 to 1.8e-7 of the
                // output's rms, but need 64 registers more than a wave has with two workgroups on a compute unit.
                // LDS reads run two tiles ahead of their MFMAs (one tile, 8 MFMAs, is shorter than the LDS latency
                // while four waves and the incoming requests share the LDS)
                half8 ah[3], al[3];
                ah[0] = *reinterpret_cast<const half8 *>(base);
                al[0] = *reinterpret_cast<const half8 *>(base + 1024);
                ah[1] = *reinterpret_cast<const half8 *>(base + 2048);
                al[1] = *reinterpret_cast<const half8 *>(base + 2048 + 1024);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    const half8 ch = ah[tt % 3], cl = al[tt % 3];
                    if (tt + 2 < TT) {
                        ah[(tt + 2) % 3] = *reinterpret_cast<const half8 *>(base + (tt + 2) * 2048);
                        al[(tt + 2) % 3] = *reinterpret_cast<const half8 *>(base + (tt + 2) * 2048 + 1024);
                    }
#pragma unroll
                    for (int rt = 0; rt < GM_RT; ++rt) {
                        acch[tt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ch, Bc[rt], s == 0 ? zero : acch[tt][rt], 0, 0, 0);
                        acch[tt][rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(cl, Bc[rt], acch[tt][rt], 0, 0, 0);
                    }
                    if (tt < GM_RT) {
                        if (s < 7) build_b(Bn[tt], tt, b, s + 1);
                        else build_m(Bn[tt], dd[tt], dm[tt], tt, b);
#pragma unroll
                        for (int k = 0; k < 2 * GM_RT; ++k) { // one MFMA, then up to four VALU instructions of the build
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                            __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // the min term: sum_s m_s * xs_s, one MFMA step with the m_s as B operand; then the super-block's term
                // is formed at its own magnitude and added in one step (one rounding per super-block at the magnitude
                // of the running sum)
                half8 ax = *reinterpret_cast<const half8 *>(base);
#pragma unroll
                for (int tt = 0; tt < TT; ++tt) {
                    const half8 cx = ax;
                    if (tt + 1 < TT) ax = *reinterpret_cast<const half8 *>(base + (tt + 1) * 1024);
#pragma unroll
                    for (int rt = 0; rt < GM_RT; ++rt) {
                        const v4f am = __builtin_amdgcn_mfma_f32_16x16x32_f16(cx, Bc[rt], zero, 0, 0, 0);
                        // this lane: row n of row tile rt, tokens 4g .. 4g+3 of the tile
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            yacc[tt][rt][i] += fmaf(dd[rt], acch[tt][rt][i], -(dm[rt] * am[i]));
                    }
                    if (tt < GM_RT) {
                        if (b + 1 < nbl) build_b(Bn[tt], tt, b + 1, 0);
                        else Bn[tt] = Bc[tt];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int rt = 0; rt < GM_RT; ++rt) Bc[rt] = Bn[rt];
        };
        position(std::integral_constant<int, 0>{});
        position(std::integral_constant<int, 1>{});
        position(std::integral_constant<int, 2>{});
        position(std::integral_constant<int, 3>{});
        position(std::integral_constant<int, 4>{});
        position(std::integral_constant<int, 5>{});
        position(std::integral_constant<int, 6>{});
        position(std::integral_constant<int, 7>{});
        position(std::integral_constant<int, 8>{});
    }

    if (a.ksplit > 1) { // this share's sums, scaled back, for gemm_ksplit_reduce_kernel
#pragma unroll
        for (int rt = 0; rt < GM_RT; ++rt) {
            const int64_t out_row = row0 + (a.pair ? 16 * (rt & 1) : 16 * rt) + n;
            if (out_row >= my.n_rows) continue;
            float *dst = a.part + static_cast<int64_t>(rb) * GM_ROWS + wave * 64 + 16 * rt + n;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int t = (tile0 + tt) * 16 + 4 * g + i;
                    if (t < a.T) dst[(static_cast<int64_t>(blockIdx.y) * a.T + t) * a.ldp] = yacc[tt][rt][i] * a.stat[t].y;
                }
        }
        return;
    }
    if (a.pair) { // row tiles 0, 1: rows of the gate matrix; 2, 3: the same rows of the up matrix
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
            const int64_t out_row = row0 + 16 * rt + n;
            if (out_row >= my.n_rows) continue;
#pragma unroll
            for (int tt = 0; tt < TT; ++tt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int t = (tile0 + tt) * 16 + 4 * g + i;
                    if (t < a.T) {
                        const float sc = a.stat[t].y;
                        const float gt = yacc[tt][rt][i] * sc, up = yacc[tt][rt + 2][i] * sc;
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
        for (int tt = 0; tt < TT; ++tt)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int t = (tile0 + tt) * 16 + 4 * g + i;
                if (t < a.T) {
                    float v = yacc[tt][rt][i] * a.stat[t].y;
                    if (a.resid) v += a.resid[t * a.ldr + out_row];
                    my.y[t * my.ldy + out_row] = v;
                }
            }
    }
}

// y = the shares of K added in order (+ resid): one thread per (token, column of the shares)
__global__ void __launch_bounds__(256) gemm_ksplit_reduce_kernel(GemmArgs a)
{
    const int64_t col = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int t = blockIdx.y;
    if (a.pair) {
        // output row `col` of silu(gate) * up: its gate sums sit at column (row block, wave, row in the wave's 32) of the
        // shares, its up sums 32 columns further
        if (col >= a.seg[0].n_rows) return;
        const int64_t gc = (col / (GM_ROWS / 2)) * GM_ROWS + ((col % (GM_ROWS / 2)) / 32) * 64 + col % 32;
        float gt = a.part[static_cast<int64_t>(t) * a.ldp + gc], up = a.part[static_cast<int64_t>(t) * a.ldp + gc + 32];
        for (int ks = 1; ks < a.ksplit; ++ks) {
            gt += a.part[(static_cast<int64_t>(ks) * a.T + t) * a.ldp + gc];
            up += a.part[(static_cast<int64_t>(ks) * a.T + t) * a.ldp + gc + 32];
        }
        a.seg[0].y[t * a.seg[0].ldy + col] = gt / (1.0f + expf(-gt)) * up;
        return;
    }
    if (col >= a.ldp) return;
    const int rb = static_cast<int>(col / GM_ROWS);
    const int sg = rb >= a.seg[2].rb0 ? 2 : (rb >= a.seg[1].rb0 ? 1 : 0);
    const GemmSegDev &my = a.seg[sg];
    const int64_t row = col - static_cast<int64_t>(my.rb0) * GM_ROWS;
    if (row >= my.n_rows) return;
    float v = a.part[static_cast<int64_t>(t) * a.ldp + col];
    for (int ks = 1; ks < a.ksplit; ++ks) v += a.part[(static_cast<int64_t>(ks) * a.T + t) * a.ldp + col];
    if (a.resid) v += a.resid[t * a.ldr + row];
    my.y[t * my.ldy + row] = v;
}

// Into how many shares K is cut: none while the row and token blocks alone give every compute unit a workgroup; else as
// many as fill the workgroup slots of the device (two per compute unit), each share at least GM_MIN_SHARE super-blocks
constexpr int GM_MIN_SHARE = 4, GM_MAX_KSPLIT = 16;
int ksplit_for(int64_t n_rb, int64_t n_tb, int64_t nb)
{
    const int64_t wgs = n_rb * n_tb, slots = 2 * GM_CUS;
    if (wgs <= 0 || wgs * 2 > slots) return 1;
    const int64_t s = std::min<int64_t>({slots / wgs, nb / GM_MIN_SHARE, GM_MAX_KSPLIT});
    return s < 2 ? 1 : static_cast<int>(s);
}
// row blocks of one matrix; of a (gate, up) pair of n_rows each: 128 rows of both per block
int64_t row_blocks(int64_t n_rows, bool pair = false) { return pair ? (n_rows + GM_ROWS / 2 - 1) / (GM_ROWS / 2) : (n_rows + GM_ROWS - 1) / GM_ROWS; }
int token_blocks(int T) { return ((T + 15) / 16 + GM_TT - 1) / GM_TT; }

} // namespace

int gemm_ksplit(int T, const int64_t *n_rows, int n_mats, int64_t n_cols, bool pair)
{
    int64_t n_rb = 0;
    for (int i = 0; i < (pair ? 1 : n_mats); ++i) n_rb += row_blocks(n_rows[i], pair);
    return ksplit_for(n_rb, token_blocks(T), n_cols / QK);
}

size_t gemm_part_bytes(int T, const int64_t *n_rows, int n_mats, int64_t n_cols, bool pair)
{
    const int s = gemm_ksplit(T, n_rows, n_mats, n_cols, pair);
    if (s == 1) return 0;
    int64_t n_rb = 0;
    for (int i = 0; i < (pair ? 1 : n_mats); ++i) n_rb += row_blocks(n_rows[i], pair);
    return static_cast<size_t>(s) * static_cast<size_t>(T) * static_cast<size_t>(n_rb) * GM_ROWS * sizeof(float);
}

size_t gemm_ws_bytes(int T, int64_t n_cols)
{
    const size_t tiles = (static_cast<size_t>(T) + 15) / 16;
    return round_up(static_cast<size_t>(T) * sizeof(float2), GM_STAT_ALIGN) + tiles * static_cast<size_t>(n_cols / QK) * GM_TILE_BYTES;
}

prima_status launch_q4k_gemm_multi(const GemmMat *mats, int n_mats, bool pair, int64_t n_cols, const float *x, int64_t ldx, int T,
                                   const float *gain, float eps, const float *resid, int64_t ldr, void *ws, hipStream_t st, bool split_ready,
                                   void *part, size_t part_bytes)
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
    const int n_tiles = (T + 15) / 16;
    const int n_tb = (n_tiles + GM_TT - 1) / GM_TT;
    const int64_t rb_per_xcd = (n_rb + GM_XCDS - 1) / GM_XCDS;
    const int patch_c = std::min(n_tb, GM_PATCH_C);
    const int patch_r = static_cast<int>(std::min<int64_t>(std::max(1, GM_PATCH / patch_c), rb_per_xcd));
    const int64_t grid = (rb_per_xcd + patch_r - 1) / patch_r * ((n_tb + patch_c - 1) / patch_c) * (patch_r * patch_c) * GM_XCDS;
    if (grid >= (int64_t{1} << 31) || n_tiles > 65535 || nb >= (int64_t{1} << 31)) return PRIMA_E_SHAPE;
    static std::atomic<bool> attr_set{false}; // set twice by two threads at worst: the attribute call is idempotent
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
    a.T = T; a.n_tiles = n_tiles; a.n_rb = static_cast<int>(n_rb); a.n_tb = n_tb; a.patch_r = patch_r; a.patch_c = patch_c;
    // K is divided when that fills the device and the caller's scratch holds the shares
    a.ksplit = part && T <= 65535 ? ksplit_for(n_rb, n_tb, nb) : 1; // (the shares are added by a launch with T as a grid dimension)
    a.ldp = n_rb * GM_ROWS;
    if (a.ksplit > 1 && part_bytes < static_cast<size_t>(a.ksplit) * static_cast<size_t>(T) * static_cast<size_t>(a.ldp) * sizeof(float)) a.ksplit = 1;
    a.part = a.ksplit > 1 ? static_cast<float *>(part) : nullptr;
    hipLaunchKernelGGL(q4k_gemm_kernel, dim3(static_cast<unsigned>(grid), a.ksplit), dim3(GM_THREADS), GM_LDS_BYTES, st, a);
    if (a.ksplit > 1) {
        const prima_status ps = last_launch_status();
        if (ps != PRIMA_OK) return ps;
        hipLaunchKernelGGL(gemm_ksplit_reduce_kernel, dim3(static_cast<unsigned>((a.ldp + 255) / 256), T), dim3(256), 0, st, a);
    }
    return last_launch_status();
}

prima_status launch_q4k_gemm(const uint8_t *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int T,
                             const float *gain, float eps, const float *resid, int64_t ldr, float *y, int64_t ldy,
                             void *ws, hipStream_t st, bool split_ready, void *part, size_t part_bytes)
{
    const GemmMat m{W, y, n_rows, ldy};
    return launch_q4k_gemm_multi(&m, 1, false, n_cols, x, ldx, T, gain, eps, resid, ldr, ws, st, split_ready, part, part_bytes);
}

} // namespace prima
