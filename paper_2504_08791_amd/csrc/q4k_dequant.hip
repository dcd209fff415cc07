// Q4_K dequantisation test hook (gfx950).
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

} // namespace prima
