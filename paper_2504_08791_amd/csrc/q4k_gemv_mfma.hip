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
//  * several tokens (speculative verification, App. A.12) use the rows of the A operand for
//    (token, digit) pairs instead: 4 tokens x 4 digits, one MFMA per sub-block for all four tokens,
//    lane (j, g) receives the digit sums of token g with row j.  Each weight byte is unpacked once
//    and nothing is multiplied by zeros; at 8 tokens the loop is bound by its instructions
//    (4 multiply-adds per sub-block and token group for the sub-scales), at ~4.8 TB/s of weights.
//
// Data movement.  One 512-thread workgroup per compute unit, persistent; it owns a share of the
// 16-row tiles (with all of K whenever the activations fit in LDS), dealt interleaved with the other
// workgroups' (rank, rank + ranks, ...: the workgroups then read one moving window of the matrix,
// which loads the memory channels evenly) or, where slabs are added in place, as a contiguous run;
// every sum has a fixed order.
// Each wave streams its share of the weights through a private three-stage LDS ring filled by
// 128-bit global->LDS loads (no VGPR staging; at one token with the non-temporal bit: a launch reads
// every weight byte once): a stage is 16 rows x 2 super-blocks, requested as
// runs of 288 contiguous bytes per row, laid out with an odd row stride so that the MFMA-order
// reads (lane (j, g) reads row j) are free of bank conflicts.  Two stages are always in flight
// per wave while the third is consumed; only s_waitcnt orders them, no barrier.  Waves take
// (tile, part) units from an LDS counter.  The activations are transformed (RMSNorm when asked),
// quantised and laid out in LDS by every workgroup for itself.  When the digits of all of K do not
// fit in the LDS left over by the rings, K is cut into slabs and a workgroup handles one slab of a
// (larger) range of tiles, with its own fixed-point scale; the slabs' partial sums meet in global
// memory.  One token: the workgroup that arrives last at a tile adds them in slab order (device-scope
// stores and loads, one relaxed atomic counter per tile, reset for the next launch; no fences).
// Several tokens: a second small kernel adds them (the last arriver would be one workgroup for
// nearly all tiles).  The epilogue adds the residual, or applies SwiGLU to a (gate, up) pair of tiles.
// The body is gemv_body.inc.
#include <atomic>

#include "gemv_common.h"

namespace prima {

// TT tokens per pass.  The kind of activations, the number of matrices and the epilogue are run-time
// arguments: the projections of a layer then share one piece of code, which stays in the instruction
// caches from launch to launch (with one kernel per projection every launch started on cold caches and
// took 3-4 us longer).
template <int TT>
__global__ void __launch_bounds__(GEMV_THREADS) gemv_q4k_persistent_kernel(PGemvArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    const int wg_index = blockIdx.x;
    const float *const arg_x = a.x, *const arg_gain = a.gain;
    const uint8_t *const arg_W0 = a.seg[0].W, *const arg_W1 = a.seg[1].W, *const arg_W2 = a.seg[2].W;
    float *const arg_y0 = a.seg[0].y, *const arg_y1 = a.seg[1].y, *const arg_y2 = a.seg[2].y;
    const float *const arg_r0 = a.seg[0].resid, *const arg_r1 = a.seg[1].resid, *const arg_r2 = a.seg[2].resid;
#include "gemv_body.inc"
}

// Second kernel of a launch with deferred slab addition: one thread per (tile or gate/up pair, token, row) adds
// the slabs' partial sums in slab order and applies the epilogue (residual, or SwiGLU on a pair).
template <int TT>
__global__ void __launch_bounds__(256) gemv_slab_reduce_kernel(PGemvArgs a)
{
    const bool pairs = a.epi == EPI_SWIGLU;
    const int gran = pairs ? 2 : 1;
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t n_out = static_cast<int64_t>(a.n_tiles / gran) * 16 * TT;
    if (idx >= n_out) return;
    const int gl = static_cast<int>(idx / (16 * TT));
    const int rem = static_cast<int>(idx - static_cast<int64_t>(gl) * (16 * TT));
    const int t = rem >> 4, jj = rem & 15;
    const int64_t slab_stride = static_cast<int64_t>(a.n_tiles) * 16 * TT;
    // slab order, eight loads out before the first is added (one at a time every slab costs a trip to memory)
    const int n_slabs = a.n_slabs;
    auto all_slabs = [&](int tile) {
        const float *p = a.part + static_cast<int64_t>(tile) * 16 * TT + rem;
        float v = 0.f;
        for (int s0 = 0; s0 < n_slabs; s0 += 8) {
            float w[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) w[i] = p[min(s0 + i, n_slabs - 1) * slab_stride]; // (past the last slab: a valid address, not added)
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (s0 + i < n_slabs) v += w[i];
        }
        return v;
    };
    if (pairs) {
        const int64_t row = static_cast<int64_t>(gl) * 16 + jj;
        if (row < a.seg[0].n_rows) {
            const float gt = all_slabs(2 * gl), up = all_slabs(2 * gl + 1);
            a.seg[0].y[t * a.seg[0].ldy + row] = gt / (1.0f + expf(-gt)) * up;
        }
    } else {
        int sg, tis;
        tile_segment(false, a.nseg, a.seg_tile0[1], a.seg_tile0[2], gl, sg, tis);
        const GemvSeg &sgm = a.seg[sg];
        const int64_t row = static_cast<int64_t>(tis) * 16 + jj;
        if (row < sgm.n_rows) {
            float v = all_slabs(gl);
            if (sgm.resid) v += sgm.resid[t * sgm.ldr + row];
            sgm.y[t * sgm.ldy + row] = v;
        }
    }
}

size_t gemv_ws_bytes(int64_t n_rows_total, int64_t n_cols, int T)
{
    // any segmentation of the rows into up to three matrices adds at most two tiles; the plan (and with it the number
    // of slabs) can change with every tile more or less, so each possible count is planned
    const int base = static_cast<int>((n_rows_total + 15) / 16);
    const int n_tiles = base + 2;
    size_t worst = 0;
    for (int t0 = 0; t0 < T; t0 += MAX_T_PASS) {
        const int Tp = T - t0 < MAX_T_PASS ? T - t0 : MAX_T_PASS;
        for (int nt = base; nt <= base + 2; ++nt) {
            for (int epi : {EPI_ROWS, EPI_SWIGLU}) {
                if (nt < 1 || (epi == EPI_SWIGLU && (nt & 1))) continue; // gate / up: two matrices of equal height
                PPlan p = plan_for(nt, static_cast<int>(n_cols / QK), Tp, epi);
                if (!p.ok) continue;
                p.n_tiles = n_tiles;
                const size_t b = part_bytes(p, Tp);
                worst = b > worst ? b : worst;
            }
        }
    }
    return arrivals_bytes(n_tiles) + worst;
}

size_t gemv_arrivals_bytes(int64_t n_rows_total) { return arrivals_bytes(static_cast<int>((n_rows_total + 15) / 16) + 2); }

template <int TT>
static hipError_t launch_tt(const PGemvArgs &a, const PPlan &p, hipStream_t st)
{
    static std::atomic<bool> attr_set{false}; // set twice by two threads at worst: the attribute call is idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(gemv_q4k_persistent_kernel<TT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(LDS_BUDGET));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL((gemv_q4k_persistent_kernel<TT>), dim3(p.n_wg), dim3(GEMV_THREADS), p.lds_bytes, st, a);
    if (a.defer) {
        const int64_t n_out = static_cast<int64_t>(a.n_tiles / (a.epi == EPI_SWIGLU ? 2 : 1)) * 16 * TT;
        hipLaunchKernelGGL((gemv_slab_reduce_kernel<TT>), dim3(static_cast<unsigned>((n_out + 255) / 256)), dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

// host only: whether every pass of this launch finds a plan and fits the scratch (nothing is launched; ws is not touched)
prima_status gemv_plan_status(const GemvArgs &ga, void *ws, size_t ws_bytes, size_t arrivals_region)
{
    for (int t0 = 0; t0 < ga.T; t0 += MAX_T_PASS) {
        const int T = ga.T - t0 < MAX_T_PASS ? ga.T - t0 : MAX_T_PASS;
        PPlan p;
        PGemvArgs a;
        const prima_status bs = build_pass(ga, t0, T, ws, ws_bytes, arrivals_region, a, p);
        if (bs != PRIMA_OK) return bs;
    }
    return PRIMA_OK;
}

prima_status launch_gemv_mfma(const GemvArgs &ga, void *ws, size_t ws_bytes, size_t arrivals_region, hipStream_t st)
{
    // up to MAX_T_PASS tokens per pass over the weights
    for (int t0 = 0; t0 < ga.T; t0 += MAX_T_PASS) {
        const int T = ga.T - t0 < MAX_T_PASS ? ga.T - t0 : MAX_T_PASS;
        PPlan p;
        PGemvArgs a;
        const prima_status bs = build_pass(ga, t0, T, ws, ws_bytes, arrivals_region, a, p);
        if (bs != PRIMA_OK) return bs;
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
