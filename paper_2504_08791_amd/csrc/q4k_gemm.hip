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
// sub-block by sub-block through a ring of LDS slots that global->LDS loads fill four positions ahead (activations
// and the wave's own weight bytes alike; the comment at the kernel has the details).  Workgroups are numbered so
// that those running on one XCD (one L2) at a time are patches of 4 row blocks x 8 token blocks.  Up to three
// matrices with the same columns share a launch (Q / K / V), and so do a gate and an up matrix, with SwiGLU behind.
// The weights stay exact: dequantised to binary16 (one accumulator for all of K) they would be off by ~1e-3 per
// product, measured in the metric of the tests.
#include <hip/hip_fp16.h>

#include <atomic>

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
constexpr int GM_NS = 5;                        // ring slots: sub-block positions in LDS or on their way
constexpr int GM_SLOT = GM_TT * 2048 + GM_WAVES * 1024;                   // 12 KiB
constexpr int GM_LDS_BYTES = GM_NS * GM_SLOT + 2 * GM_WAVES * 1024;       // 68 KiB: two workgroups per compute unit
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

// workgroup barrier that orders LDS traffic only (__syncthreads() would also wait for every global load in flight,
// that is, for the whole ring of requests below)
__device__ __forceinline__ void gm_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// One workgroup: 4 waves, one per SIMD; a wave owns 64 rows (four B tiles) x 64 tokens, i.e. 16 accumulator tiles for the
// super-block in hand and as many running sums; two workgroups share a compute unit (256 registers per wave, 68 KiB of
// LDS per workgroup) and run out of step with each other.  The super-block is walked sub-block by sub-block ("positions"
// 0..7, then position 8: the sums slab and the min term).  Everything a position needs comes through LDS by 16-byte
// global->LDS loads, NS - 1 positions ahead:
//   slot (12 KiB):  [4 token tiles][hi 1 KiB | lo 1 KiB] activations of the sub-block   (shared by the four waves)
//                   [4 waves][64 rows x 16 bytes] the sub-block's quants              (each wave its own rows)
//   position 8 uses the slot's first 4 KiB for the sums slabs; the headers of a super-block (64 rows x 16 bytes
//   per wave) arrive with its position 0 in a ring of two of their own.
// Per position: wait until all but the newest WAIT_N1 requests of this wave have landed (requests complete in
// order), barrier (everyone's share is there, and everyone has finished reading the slot of the position before,
// which is the slot requested next), request position p + NS - 1, and then, token tile by token tile, the MFMAs of
// this position with, between them, the VALU work that builds the B tiles of the next position (its quants and
// headers are this wave's own requests, which the same wait covers).  No global load is left for the compiler to
// wait on.  Measured with parts of the work switched off (8192 x 28672 weights, 1024 tokens): the LDS reads of the
// activations cost 30 % of the time, the requests 12 %, the B tiles 10 %, the barrier 3 %: a wave reads every
// activation of its 64 tokens once per position, whatever the tiling, so LDS bandwidth is met before the MFMA rate.
__global__ void __launch_bounds__(GM_THREADS, 2) q4k_gemm_kernel(GemmArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int TT = GM_TT;
    constexpr int A_BYTES = TT * 2048, SLOT = GM_SLOT;
    constexpr int HDR_RING = GM_NS * SLOT;           // two entries of GM_WAVES KiB behind the slots
    constexpr int DM = TT / 2, DMS = TT / 4;         // activation requests per wave: a sub-block position, the sums position
    // requests of the NS - 2 positions between the one awaited and now: each at least DM + 1, one of them may be a
    // sums position (DMS)
    constexpr int WAIT_N = (GM_NS - 3) * (DM + 1) + DMS;
    constexpr int WAIT_N1 = (GM_NS - 4) * (DM + 1) + DMS; // the same for the NS - 3 positions behind p + 1
    static_assert(TT == 4 && GM_WAVES == 4, "requests per wave and position are counted for 4 tiles and 4 waves");
    static_assert(WAIT_N <= 63, "vmcnt is a 6-bit counter");
    static_assert(GM_NS >= 4 && GM_NS <= 9, "ring depth: the first NS - 1 positions belong to super-block 0");
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
    // the row whose 16-byte pieces this lane requests: local row `lane` of the wave (past the end: a valid row, not stored)
    const uint8_t *wsrc;
    {
        const int64_t r = min<int64_t>(row0 + (a.pair ? (lane & 31) : lane), my.n_rows - 1);
        wsrc = (a.pair ? a.seg[lane >> 5].W : my.W) + r * nb * 144;
    }
    const int tile0 = tb * TT;
    const uint32_t lds0 = lds_address(smem);
    // this workgroup's share of K: super-blocks [b_lo, b_lo + nbl) (all of them unless K is divided; never empty: the
    // host keeps ksplit <= nb); below, `b` counts from b_lo
    const int b_lo = static_cast<int>(static_cast<int64_t>(blockIdx.y) * nb / a.ksplit);
    const int nbl = static_cast<int>(static_cast<int64_t>(blockIdx.y + 1) * nb / a.ksplit) - b_lo;
    wsrc += static_cast<int64_t>(b_lo) * 144;
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

    // every request of position (b, s), into ring slot `slot` (s is a constant wherever this is called)
    auto issue = [&](int b, int s, int slot) __attribute__((always_inline)) {
        const uint32_t base = lds0 + slot * SLOT;
        const int64_t boff = static_cast<int64_t>(b) * (GM_SLABS * 1024);
        if (s < 8) {
#pragma unroll
            for (int jj = 0; jj < DM; ++jj)
                dma16_base(abase[jj] + boff + 2048 * s, lane16, base + (2 * jj + (wave >> 1)) * 2048 + (wave & 1) * 1024);
            const uint8_t *wp = wsrc + static_cast<int64_t>(b) * 144;
            switch (s) { // the sub-block's 16 bytes of quants of this lane's row
            case 0: dma16_off<16>(wp, base + A_BYTES + wave * 1024); break;
            case 1: dma16_off<32>(wp, base + A_BYTES + wave * 1024); break;
            case 2: dma16_off<48>(wp, base + A_BYTES + wave * 1024); break;
            case 3: dma16_off<64>(wp, base + A_BYTES + wave * 1024); break;
            case 4: dma16_off<80>(wp, base + A_BYTES + wave * 1024); break;
            case 5: dma16_off<96>(wp, base + A_BYTES + wave * 1024); break;
            case 6: dma16_off<112>(wp, base + A_BYTES + wave * 1024); break;
            default: dma16_off<128>(wp, base + A_BYTES + wave * 1024); break;
            }
            if (s == 0) dma16_off<0>(wp, lds0 + HDR_RING + ((b & 1) * GM_WAVES + wave) * 1024);
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

    // positions 0 .. NS-2 (a super-block has 9 > NS - 1 positions, so they all belong to super-block 0)
#pragma unroll
    for (int s = 0; s < GM_NS - 1; ++s) issue(0, s, s);

    // B tile `rt` of a sub-block position from this wave's quants in ring slot `sl` and its headers of super-block `bb`:
    // sc_s * q as binary16 (exact).  A dword holds the eight weights of lane (n, g); masked in pairs (0,4) (1,5) (2,6)
    // (3,7) into the mantissas of 1024 + q, then one fused multiply-add per pair: (1024 + q) sc - 1024 sc
    auto build_b = [&](half8 &B, int rt, int bb, int s, int sl) __attribute__((always_inline)) {
        const uint32_t w = *reinterpret_cast<const uint32_t *>(smem + sl * SLOT + A_BYTES + wave * 1024 + (16 * rt + n) * 16 + 4 * g);
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
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(WAIT_N) : "memory"); // position 0 has landed (this wave's share)
#pragma unroll
    for (int rt = 0; rt < GM_RT; ++rt) build_b(Bc[rt], rt, 0, 0, 0);

    int slot = 0; // ring slot of the current position
    for (int b = 0; b < nbl; ++b) {
#pragma unroll
        for (int s = 0; s < 9; ++s) {
            const int p = 9 * b + s;
            // positions p and p + 1 have landed (this wave's share) once at most the requests of the NS - 3 positions
            // behind them are in flight
            if (p + GM_NS - 2 < total) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(WAIT_N1) : "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // the last positions: nothing is requested behind them any more
            gm_barrier();
            {
                // position p + NS - 1 goes into the slot that position p - 1 has just left
                const int s_t = (s + GM_NS - 1) % 9;
                const int b_t = b + (s + GM_NS - 1) / 9;
                const int slot_t = slot == 0 ? GM_NS - 1 : slot - 1;
                if (b_t < nbl) issue(b_t, s_t, slot_t);
            }
            const uint8_t *base = smem + slot * SLOT + lane * 16;
            const int slot_n = slot + 1 == GM_NS ? 0 : slot + 1;
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
                        if (s < 7) build_b(Bn[tt], tt, b, s + 1, slot_n);
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
                        if (b + 1 < nbl) build_b(Bn[tt], tt, b + 1, 0, slot_n);
                        else Bn[tt] = Bc[tt];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int rt = 0; rt < GM_RT; ++rt) Bc[rt] = Bn[rt];
            slot = slot_n;
        }
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
