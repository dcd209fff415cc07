// Load-time conversion of quantised tensors from the block order of GGUF model files into this library's layouts
// (gfx950).
//
// The paper's checkpoints are "Q4K" GGUF files of Llama and Qwen models whose tensors are mostly Q4_K with some in
// other formats (arXiv 2504.08791, Sec. 4, experimental setup; App. A.3, the profiler's format list).  The kernels of
// this library stream their own placements of the same fields (prima.h), chosen for 128-bit loads and one-mask
// unpacking, so a file's tensor is copied to the device as it is and rearranged there once, at HBM speed; values and
// field meanings do not change, only where the bits sit.
//
// One thread per 32-bit word of output (or per binary16 scale); the source is read byte by byte (a file's tensor is
// only guaranteed 2-byte alignment for the 210-byte blocks) and every byte of a block is touched by a few
// neighbouring threads, so the reads are cache hits after the first.
#include "common.h"

namespace prima {

namespace {

// ---- fields of a source block (GGUF order) ----

// six-bit field i of a q4_k / q5_k block's scales[12] (sc12): i < 8 sub-scale sc_i, otherwise sub-min m_{i-8}
__device__ __forceinline__ uint32_t k_field(const uint8_t *sc12, int i)
{
    const int j = i & 7;
    const bool is_min = i >= 8;
    if (j < 4) return sc12[is_min ? j + 4 : j] & 63u;
    const uint32_t lo4 = is_min ? sc12[j + 4] >> 4 : sc12[j + 4] & 15u;
    const uint32_t hi2 = sc12[is_min ? j : j - 4] >> 6;
    return lo4 | (hi2 << 4);
}

// low four bits of weight t: q4_k / q5_k (qs[128]: 64 weights share 32 bytes, the first 32 in the low nibbles)
__device__ __forceinline__ uint32_t k_low4(const uint8_t *qs, int t)
{
    const uint32_t byte = qs[32 * (t >> 6) + (t & 31)];
    return (t & 32) ? byte >> 4 : byte & 15u;
}
// bit 4 of weight t: q5_k (qh[32]: bit 2c + (second half of the 64) of byte t % 32, c = t / 64)
__device__ __forceinline__ uint32_t k5_bit4(const uint8_t *qh, int t)
{
    return (qh[t & 31] >> (2 * (t >> 6) + ((t >> 5) & 1))) & 1u;
}
// q6_k: 128 weights share ql[64] and qh[32]; quarter k of the 128 has its low bits in ql[32 (k & 1) + l], low nibble
// for k < 2, and bits 4..5 at bits 2k of qh[l]
__device__ __forceinline__ uint32_t k6_low4(const uint8_t *ql, int t)
{
    const int h = t >> 7, k = (t >> 5) & 3, l = t & 31;
    const uint32_t byte = ql[64 * h + 32 * (k & 1) + l];
    return k < 2 ? byte & 15u : byte >> 4;
}
__device__ __forceinline__ uint32_t k6_bits45(const uint8_t *qh, int t)
{
    const int h = t >> 7, k = (t >> 5) & 3, l = t & 31;
    return (qh[32 * h + l] >> (2 * k)) & 3u;
}

// word w of the "low four bits" plane of a super-block (prima.h: byte t % 4 of word t / 8, low nibble when t % 8 < 4)
template <typename F> __device__ __forceinline__ uint32_t low_plane_word(F low4_of, int w)
{
    uint32_t v = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) v |= (low4_of(8 * w + j) | (low4_of(8 * w + 4 + j) << 4)) << (8 * j);
    return v;
}

// the header words 1..3 of a q4_k / q5_k super-block: the sixteen fields as a 96-bit little-endian stream
__device__ __forceinline__ uint32_t field_stream_word(const uint8_t *sc12, int w)
{
    uint32_t v = 0;
    for (int i = 0; i < 16; ++i) {
        const int bit = 6 * i - 32 * w; // position of field i relative to this word
        if (bit <= -6 || bit >= 32) continue;
        const uint32_t f = k_field(sc12, i);
        v |= bit >= 0 ? f << bit : f >> -bit;
    }
    return v;
}

__device__ __forceinline__ uint32_t bytes4(const uint8_t *p)
{
    return static_cast<uint32_t>(p[0]) | (static_cast<uint32_t>(p[1]) << 8) | (static_cast<uint32_t>(p[2]) << 16) | (static_cast<uint32_t>(p[3]) << 24);
}

// ---- kernels: thread = (super-block, unit) ----

constexpr int Q4K_UNITS = 36;           // 1 word d/dmin, 3 words of fields, 32 words of quants
constexpr int Q5K_UNITS = 4 + 32 + 8;   // header, low plane, bit-4 plane
constexpr int Q6K_UNITS = 32 + 16 + 4 + 1; // low plane, bits 4..5, sub-scales, d
constexpr int Q80_UNITS = 64 + 8;       // 256 signed bytes, 8 scales

__global__ void __launch_bounds__(256) repack_q4k_kernel(const uint8_t *__restrict__ src, int64_t n, uint8_t *__restrict__ dst)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t blk = idx / Q4K_UNITS;
    const int u = static_cast<int>(idx - blk * Q4K_UNITS);
    if (blk >= n) return;
    const uint8_t *s = src + blk * 144;
    uint32_t v;
    if (u == 0) v = bytes4(s);
    else if (u < 4) v = field_stream_word(s + 4, u - 1);
    else {
        // byte b of the quants holds weights 2b (low nibble) and 2b + 1
        const uint8_t *qs = s + 16;
        v = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int t = 2 * (4 * (u - 4) + j);
            v |= (k_low4(qs, t) | (k_low4(qs, t + 1) << 4)) << (8 * j);
        }
    }
    reinterpret_cast<uint32_t *>(dst + blk * 144)[u] = v;
}

__global__ void __launch_bounds__(256) repack_q5k_kernel(const uint8_t *__restrict__ src, int64_t n, uint8_t *__restrict__ dst)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t blk = idx / Q5K_UNITS;
    const int u = static_cast<int>(idx - blk * Q5K_UNITS);
    if (blk >= n) return;
    const uint8_t *s = src + blk * 176; // d, dmin | scales[12] | qh[32] | qs[128]
    if (u < 4) {
        reinterpret_cast<uint32_t *>(dst + blk * 16)[u] = u == 0 ? bytes4(s) : field_stream_word(s + 4, u - 1);
    } else if (u < 36) {
        const uint8_t *qs = s + 48;
        reinterpret_cast<uint32_t *>(dst + 16 * n + blk * 128)[u - 4] = low_plane_word([&](int t) { return k_low4(qs, t); }, u - 4);
    } else {
        // bit 4: word t / 32, bit (t % 32) / 4 of byte t % 4
        const uint8_t *qh = s + 16;
        const int w = u - 36;
        uint32_t v = 0;
        for (int g = 0; g < 8; ++g)
#pragma unroll
            for (int j = 0; j < 4; ++j) v |= k5_bit4(qh, 32 * w + 4 * g + j) << (8 * j + g);
        reinterpret_cast<uint32_t *>(dst + 144 * n + blk * 32)[w] = v;
    }
}

__global__ void __launch_bounds__(256) repack_q6k_kernel(const uint8_t *__restrict__ src, int64_t n, uint8_t *__restrict__ dst)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t blk = idx / Q6K_UNITS;
    const int u = static_cast<int>(idx - blk * Q6K_UNITS);
    if (blk >= n) return;
    const uint8_t *s = src + blk * 210; // ql[128] | qh[64] | scales[16] | d
    if (u < 32) {
        reinterpret_cast<uint32_t *>(dst + blk * 128)[u] = low_plane_word([&](int t) { return k6_low4(s, t); }, u);
    } else if (u < 48) {
        // bits 4..5: word t / 16, bits 2g and 2g + 1 of byte t % 4, g = (t % 16) / 4
        const int w = u - 32;
        uint32_t v = 0;
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int j = 0; j < 4; ++j) v |= k6_bits45(s + 128, 16 * w + 4 * g + j) << (8 * j + 2 * g);
        reinterpret_cast<uint32_t *>(dst + 128 * n + blk * 64)[w] = v;
    } else if (u < 52) {
        reinterpret_cast<uint32_t *>(dst + 192 * n + blk * 16)[u - 48] = bytes4(s + 192 + 4 * (u - 48));
    } else {
        reinterpret_cast<uint16_t *>(dst + 208 * n)[blk] = static_cast<uint16_t>(s[208] | (s[209] << 8));
    }
}

// n = groups of 256 weights (eight 34-byte source blocks each)
__global__ void __launch_bounds__(256) repack_q80_kernel(const uint8_t *__restrict__ src, int64_t n, uint8_t *__restrict__ dst)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x;
    const int64_t blk = idx / Q80_UNITS;
    const int u = static_cast<int>(idx - blk * Q80_UNITS);
    if (blk >= n) return;
    const uint8_t *s = src + blk * 272;
    if (u < 64) {
        reinterpret_cast<uint32_t *>(dst + blk * 256)[u] = bytes4(s + 34 * (u >> 3) + 2 + 4 * (u & 7));
    } else {
        const uint8_t *p = s + 34 * (u - 64);
        reinterpret_cast<uint16_t *>(dst + 256 * n)[blk * 8 + (u - 64)] = static_cast<uint16_t>(p[0] | (p[1] << 8));
    }
}

} // namespace

size_t gguf_tensor_bytes(int32_t fmt, int64_t n_rows, int64_t n_cols)
{
    if (n_rows < 0 || n_cols < 0 || n_cols % QK) return 0;
    const size_t n = static_cast<size_t>(n_rows) * static_cast<size_t>(n_cols / QK);
    switch (fmt) {
    case PRIMA_FMT_Q4_K: return n * 144;
    case PRIMA_FMT_Q5_K: return n * 176;
    case PRIMA_FMT_Q6_K: return n * 210;
    case PRIMA_FMT_Q8_0: return n * 272;
    case PRIMA_FMT_F16: return n * 512;
    case PRIMA_FMT_F32: return n * 1024;
    }
    return 0;
}

} // namespace prima

using namespace prima;

extern "C" size_t prima_gguf_tensor_bytes(int32_t fmt, int64_t n_rows, int64_t n_cols) { return gguf_tensor_bytes(fmt, n_rows, n_cols); }

extern "C" prima_status prima_repack_gguf(int32_t fmt, const void *src, int64_t n_rows, int64_t n_cols, void *dst, void *hip_stream)
{
    if (fmt < PRIMA_FMT_Q4_K || fmt > PRIMA_FMT_F32 || n_rows < 0 || n_cols < 0 || n_cols % QK) return PRIMA_E_SHAPE;
    const int64_t n = n_rows * (n_cols / QK);
    if (n == 0) return PRIMA_OK;
    if (!src || !dst) return PRIMA_E_NULL;
    if (!aligned(dst, 16)) return PRIMA_E_ALIGN;
    const size_t bytes = gguf_tensor_bytes(fmt, n_rows, n_cols);
    const uint8_t *s = static_cast<const uint8_t *>(src);
    uint8_t *d = static_cast<uint8_t *>(dst);
    if (s < d + bytes && d < s + bytes) return PRIMA_E_RANGE; // the two buffers overlap
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (fmt == PRIMA_FMT_F16 || fmt == PRIMA_FMT_F32)
        return hipMemcpyAsync(d, s, bytes, hipMemcpyDeviceToDevice, st) == hipSuccess ? PRIMA_OK : PRIMA_E_DEVICE;
    const int units = fmt == PRIMA_FMT_Q4_K ? Q4K_UNITS : (fmt == PRIMA_FMT_Q5_K ? Q5K_UNITS : (fmt == PRIMA_FMT_Q6_K ? Q6K_UNITS : Q80_UNITS));
    const int64_t grid = (n * units + 255) / 256;
    if (grid >= (int64_t{1} << 31)) return PRIMA_E_SHAPE;
    const dim3 g(static_cast<unsigned>(grid)), b(256);
    switch (fmt) {
    case PRIMA_FMT_Q4_K: hipLaunchKernelGGL(repack_q4k_kernel, g, b, 0, st, s, n, d); break;
    case PRIMA_FMT_Q5_K: hipLaunchKernelGGL(repack_q5k_kernel, g, b, 0, st, s, n, d); break;
    case PRIMA_FMT_Q6_K: hipLaunchKernelGGL(repack_q6k_kernel, g, b, 0, st, s, n, d); break;
    default: hipLaunchKernelGGL(repack_q80_kernel, g, b, 0, st, s, n, d); break;
    }
    return last_launch_status();
}
