// Q4_K dequantisation hook and dequant-fused mat-vec (gfx950).
//
// The projections of a decoder layer are stored in Q4_K and multiplied without ever being
// expanded in memory (arXiv 2504.08791, App. A.9); their bytes are the b of App. A.3's
// device-loading term, which is what bounds decode at small batch (Sec. 4, footnote on
// bandwidth-bound decoding).
#include "common.h"

namespace prima {

// ------------------------------------------------------------------------------------------
// Test hook: bit-exact dequantisation.  One thread per 16-byte quant chunk (one sub-block).
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) dequant_kernel(const uint8_t *__restrict__ W, int64_t n_chunks,
                                                     float *__restrict__ out)
{
    const int64_t c = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; // (block, sub-block)
    if (c >= n_chunks) return;
    const int64_t blk = c >> 3;
    const int s = static_cast<int>(c & 7);
    const uint4 *bp = reinterpret_cast<const uint4 *>(W + blk * BLOCK_BYTES);
    const uint4 hdr = bp[0];
    const uint4 qv = bp[1 + s];
    // d*sc, (d*sc)*q and dmin*m are exact in fp32; the subtraction rounds once (nearest even).
    const float dsc = __fmul_rn(hdr_d(hdr), static_cast<float>(hdr_field(hdr, s)));
    const float mm = __fmul_rn(hdr_dmin(hdr), static_cast<float>(hdr_field(hdr, 8 + s)));
    const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
    float *o = out + blk * QK + s * 32;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float4 lo, hi;
        lo.x = __fsub_rn(__fmul_rn(dsc, static_cast<float>((qw[j] >> 0) & 15u)), mm);
        lo.y = __fsub_rn(__fmul_rn(dsc, static_cast<float>((qw[j] >> 4) & 15u)), mm);
        lo.z = __fsub_rn(__fmul_rn(dsc, static_cast<float>((qw[j] >> 8) & 15u)), mm);
        lo.w = __fsub_rn(__fmul_rn(dsc, static_cast<float>((qw[j] >> 12) & 15u)), mm);
        hi.x = __fsub_rn(__fmul_rn(dsc, static_cast<float>((qw[j] >> 16) & 15u)), mm);
        hi.y = __fsub_rn(__fmul_rn(dsc, static_cast<float>((qw[j] >> 20) & 15u)), mm);
        hi.z = __fsub_rn(__fmul_rn(dsc, static_cast<float>((qw[j] >> 24) & 15u)), mm);
        hi.w = __fsub_rn(__fmul_rn(dsc, static_cast<float>((qw[j] >> 28) & 15u)), mm);
        reinterpret_cast<float4 *>(o)[2 * j] = lo;
        reinterpret_cast<float4 *>(o)[2 * j + 1] = hi;
    }
}

prima_status launch_dequant(const uint8_t *W, int64_t n_rows, int64_t n_cols, float *out, hipStream_t st)
{
    const int64_t n_chunks = n_rows * (n_cols / QK) * 8;
    if (n_chunks == 0) return PRIMA_OK;
    const int64_t grid = (n_chunks + 255) / 256;
    hipLaunchKernelGGL(dequant_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0, st, W, n_chunks, out);
    return last_launch_status();
}

// ------------------------------------------------------------------------------------------
// Reference-grade mat-vec: one wavefront per output row, lanes stride over the row's 16-byte
// chunks with coalesced 128-bit loads, fp32 x read through the caches, wave reduction by
// cross-lane shuffles.  For a sub-block s of a super-block:
//     sum_t w_t x_t = d*sc_s * sum q_t x_t - dmin*m_s * sum x_t.
// ------------------------------------------------------------------------------------------
template <int TT>
__global__ void __launch_bounds__(256) gemv_rowwave_kernel(GemvArgs a)
{
    const int lane = threadIdx.x & 63;
    int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6);
    int sg = 0;
    while (sg < a.nseg && row >= a.seg[sg].n_rows) { row -= a.seg[sg].n_rows; ++sg; }
    if (sg >= a.nseg) return;
    const GemvSeg seg = a.seg[sg];
    const int nb = static_cast<int>(a.n_cols / QK);
    const uint4 *rowp = reinterpret_cast<const uint4 *>(seg.W + row * nb * BLOCK_BYTES);

    float acc[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) acc[t] = 0.f;

    for (int c = lane; c < 9 * nb; c += 64) {
        const int blk = c / 9, part = c - blk * 9;
        if (part == 0) continue; // header chunk: read by the lanes that hold the quants
        const uint4 hdr = rowp[blk * 9];
        const uint4 qv = rowp[c];
        const int s = part - 1;
        const float dsc = hdr_d(hdr) * static_cast<float>(hdr_field(hdr, s));
        const float dm = hdr_dmin(hdr) * static_cast<float>(hdr_field(hdr, 8 + s));
        const uint32_t qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
        for (int t = 0; t < TT; ++t) {
            const float4 *xp = reinterpret_cast<const float4 *>(a.x + t * a.ldx + blk * QK + s * 32);
            float sq = 0.f, sx = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float4 x0 = xp[2 * j], x1 = xp[2 * j + 1];
                sq += static_cast<float>((qw[j] >> 0) & 15u) * x0.x + static_cast<float>((qw[j] >> 4) & 15u) * x0.y +
                      static_cast<float>((qw[j] >> 8) & 15u) * x0.z + static_cast<float>((qw[j] >> 12) & 15u) * x0.w +
                      static_cast<float>((qw[j] >> 16) & 15u) * x1.x + static_cast<float>((qw[j] >> 20) & 15u) * x1.y +
                      static_cast<float>((qw[j] >> 24) & 15u) * x1.z + static_cast<float>((qw[j] >> 28) & 15u) * x1.w;
                sx += (x0.x + x0.y) + (x0.z + x0.w) + (x1.x + x1.y) + (x1.z + x1.w);
            }
            acc[t] += dsc * sq - dm * sx;
        }
    }
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        float v = acc[t];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == 0) {
            if (seg.resid) v += seg.resid[t * seg.ldr + row];
            seg.y[t * seg.ldy + row] = v;
        }
    }
}

bool g_force_rowwave = false;

template <int TT>
static void launch_rowwave(const GemvArgs &a, int64_t rows_total, hipStream_t st)
{
    const int64_t grid = (rows_total + 3) / 4;
    hipLaunchKernelGGL(gemv_rowwave_kernel<TT>, dim3(static_cast<unsigned>(grid)), dim3(256), 0, st, a);
}

size_t gemv_ws_bytes(int64_t n_rows_total, int64_t n_cols, int) { return gemv_t1_ws_bytes(n_rows_total, n_cols); }

prima_status launch_gemv(const GemvArgs &a, void *ws, size_t ws_bytes, hipStream_t st)
{
    int64_t rows_total = 0;
    for (int i = 0; i < a.nseg; ++i) rows_total += a.seg[i].n_rows;
    if (rows_total == 0) return PRIMA_OK;
    if (a.T == 1 && !g_force_rowwave) return launch_gemv_t1(a, ws, ws_bytes, st);
    switch (a.T) {
#define PRIMA_CASE(N) case N: launch_rowwave<N>(a, rows_total, st); break;
        PRIMA_CASE(1) PRIMA_CASE(2) PRIMA_CASE(3) PRIMA_CASE(4) PRIMA_CASE(5) PRIMA_CASE(6) PRIMA_CASE(7) PRIMA_CASE(8)
        PRIMA_CASE(9) PRIMA_CASE(10) PRIMA_CASE(11) PRIMA_CASE(12) PRIMA_CASE(13) PRIMA_CASE(14) PRIMA_CASE(15) PRIMA_CASE(16)
#undef PRIMA_CASE
    default: return PRIMA_E_RANGE;
    }
    return last_launch_status();
}

} // namespace prima
