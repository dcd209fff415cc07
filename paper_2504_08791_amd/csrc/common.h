// Shared declarations of the HIP decode path (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stddef.h>
#include <stdint.h>

#include "prima.h"

namespace prima {

constexpr int QK = 256;          // weights per Q4_K super-block
constexpr int BLOCK_BYTES = 144; // bytes per super-block
constexpr int WAVE = 64;

inline prima_status last_launch_status()
{
    return hipGetLastError() == hipSuccess ? PRIMA_OK : PRIMA_E_DEVICE;
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- Q4_K header decoding (layout version 1, see prima.h) ----
// hdr = the first 16 bytes of a super-block as four little-endian dwords:
// hdr.x = d | dmin << 16, hdr.y/z/w = bits 0-31 / 32-63 / 64-95 of the field stream.
__device__ __forceinline__ float hdr_d(const uint4 &hdr)
{
    return __half2float(__ushort_as_half(static_cast<unsigned short>(hdr.x & 0xffffu)));
}
__device__ __forceinline__ float hdr_dmin(const uint4 &hdr)
{
    return __half2float(__ushort_as_half(static_cast<unsigned short>(hdr.x >> 16)));
}
// 6-bit field i (0..15): i < 8 sub-scale sc_i, otherwise sub-min m_{i-8}
__device__ __forceinline__ uint32_t hdr_field(const uint4 &hdr, int i)
{
    const int bit = 6 * i, w = bit >> 5, sh = bit & 31;
    const uint32_t lo = w == 0 ? hdr.y : (w == 1 ? hdr.z : hdr.w);
    const uint32_t hi = w == 0 ? hdr.z : (w == 1 ? hdr.w : 0u);
    const uint64_t two = static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32);
    return static_cast<uint32_t>(two >> sh) & 63u;
}

// ---- launchers implemented in the .hip files (host side, all asynchronous on `st`) ----

struct GemvSeg {
    const uint8_t *W;   // Q4_K matrix of this segment
    float *y;           // fp32 output [T][ldy]
    const float *resid; // optional fp32 [T][ldr] added to the product (may alias y)
    int64_t n_rows, ldy, ldr;
};

// how the mat-vec obtains its activation vector
enum XMode {
    X_PLAIN = 0,  // x as given
    X_RMSNORM = 1 // x * gain / sqrt(mean(x^2) + eps)
};

// what a launch stores
enum Epilogue {
    EPI_ROWS = 0,  // every segment's rows (+ residual) to its own y
    EPI_SWIGLU = 1 // two segments of equal shape (gate, up): silu(gate_r) * up_r to seg[0].y, nothing else
};

// up to three matrices with the same n_cols multiplied with the same activations in one launch
struct GemvArgs {
    GemvSeg seg[3];
    int nseg;
    int64_t n_cols;
    const float *x; // fp32 [T][ldx]
    int64_t ldx;
    int T;
    int xmode;         // XMode
    int epi;           // Epilogue
    const float *gain; // X_RMSNORM: fp32 [n_cols]
    float eps;         // X_RMSNORM
};

// the other weight formats (fmt_gemv.hip)
size_t fmt_tensor_bytes(int fmt, int64_t n_rows, int64_t n_cols);
prima_status launch_fmt_dequant(int fmt, const uint8_t *W, int64_t n_rows, int64_t n_cols, float *out, hipStream_t st);
prima_status launch_fmt_gemv(int fmt, const uint8_t *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int T,
                             const float *gain, float eps, const float *resid, int64_t ldr, float *y, int64_t ldy, hipStream_t st);

prima_status launch_dequant(const uint8_t *W, int64_t n_rows, int64_t n_cols, float *out, hipStream_t st);
// ws: scratch; its first arrivals_region bytes (>= gemv_arrivals_bytes(rows)) are counters that must be
// zero before the first launch (launch_zero_arrivals) and are left zero by every launch; the partial
// sums follow (gemv_ws_bytes() covers both for a region of gemv_arrivals_bytes(rows))
prima_status launch_gemv_mfma(const GemvArgs &a, void *ws, size_t ws_bytes, size_t arrivals_region, hipStream_t st);
size_t gemv_ws_bytes(int64_t n_rows_total, int64_t n_cols, int T);
size_t gemv_arrivals_bytes(int64_t n_rows_total);
prima_status launch_zero_arrivals(void *ws, size_t bytes, hipStream_t st);
// host only: whether every pass of this launch finds a plan and fits the scratch (nothing is launched)
prima_status gemv_plan_status(const GemvArgs &a, void *ws, size_t ws_bytes, size_t arrivals_region);

// many tokens (q4k_gemm.hip): ws holds gemm_ws_bytes(T, n_cols) bytes (per-token scales, the activations split for the matrix cores)
size_t gemm_ws_bytes(int T, int64_t n_cols);
prima_status launch_q4k_gemm(const uint8_t *W, int64_t n_rows, int64_t n_cols, const float *x, int64_t ldx, int T,
                             const float *gain, float eps, const float *resid, int64_t ldr, float *y, int64_t ldy,
                             void *ws, hipStream_t st, bool split_ready = false, void *part = nullptr, size_t part_bytes = 0);
// K divided among workgroups (a launch whose rows and tokens alone would leave most of the device idle): the number of
// shares for T tokens and n_mats matrices of these rows sharing a launch, or (pair) a gate and an up matrix of n_rows[0]
// each (1: none), and the bytes of `part` that hold the shares' sums (0: none).  A launch divides K only if it is given
// that much.
int gemm_ksplit(int T, const int64_t *n_rows, int n_mats, int64_t n_cols, bool pair = false);
size_t gemm_part_bytes(int T, const int64_t *n_rows, int n_mats, int64_t n_cols, bool pair = false);
// up to three matrices with the same columns against the same activations (Q / K / V), or, with pair set, two of equal
// shape (gate, up) with silu(gate) * up stored to mats[0].y; the residual only with one matrix
struct GemmMat {
    const uint8_t *W;
    float *y;
    int64_t n_rows, ldy;
};
prima_status launch_q4k_gemm_multi(const GemmMat *mats, int n_mats, bool pair, int64_t n_cols, const float *x, int64_t ldx, int T,
                                   const float *gain, float eps, const float *resid, int64_t ldr, void *ws, hipStream_t st,
                                   bool split_ready = false, void *part = nullptr, size_t part_bytes = 0);
// RoPE table [T][D/2] of (cos, sin) for the positions n_past .. n_past + T - 1 (any T)
prima_status launch_rope_table(float *tab, int T, int D, int n_past, float theta, hipStream_t st);

prima_status launch_stream_read(const void *src, size_t bytes, void *sink, hipStream_t st, bool nt);
prima_status launch_swiglu(float *a, const float *u, int64_t n, hipStream_t st);
// the RoPE table [T][D/2] of (cos, sin) and up to four regions filled with a word each (null: none) in one launch.
// positions: null (token t sits at n_past + t) or T positions, one per token (a batch of sequences)
prima_status launch_step_init(float *tab, int T, int D, int n_past, float theta, const int *positions,
                              void *const fill_ptr[4], const size_t fill_bytes[4], const unsigned fill_word[4], hipStream_t st);
prima_status launch_fill_words(void *a, size_t a_bytes, unsigned a_word, void *b, size_t b_bytes, unsigned b_word, hipStream_t st);
void attn_ranges(const prima_dims &d, int n_total, int T, bool batch, int &keys_per_split, int &nsplit);
size_t attn_ws_bytes(const prima_dims &d, int kv_cap, int T);
// The attention scratch: attn_counter_bytes() whose first word is the flag a bounded wait raises when it gives up
// (zero before a launch), then the key ranges' records.  A record that has not been written holds ATTN_REC_EMPTY in
// every word: before the first launch the records a launch will use (attn_records_bytes) must be filled with it
// (launch_step_init / launch_fill_words); every launch leaves them so.
size_t attn_counter_bytes(const prima_dims &d, int T);
constexpr unsigned ATTN_REC_EMPTY = 0x7fa5c3e1u; // a NaN pattern that no arithmetic produces
// bytes of records (from the start of the record area) that a launch for T tokens over n_total rows uses
size_t attn_records_bytes(const prima_dims &d, int n_total, int T, bool batch);
// q: [T][Hq][D].  With rope_tab set, q and k_new are un-rotated and the kernel rotates them and
// appends k_new / v_new to the caches; otherwise q is used as is and the caches are complete.
// seq: null, or (a batch of T sequences, one token each) per token its sequence's caches and length; K, V and
// n_past are then not used.
struct AttnSeqs;
prima_status launch_attn(const prima_dims &d, const float *q, float *q_rot_out, const float *k_new, const float *v_new,
                         const float *rope_tab, __half *K, __half *V, int kv_cap, int n_past, int T, float *o,
                         void *ws, hipStream_t st, const AttnSeqs *seq = nullptr);

// a prompt: rotated K / V rows already in the caches, q rotated; n_pieces pieces of PRIMA_MAX_TOK tokens in one launch
prima_status launch_attn_prompt(const prima_dims &d, const float *q, __half *K, __half *V, int kv_cap, int n_past, int n_pieces,
                                float *o, hipStream_t st);
// RoPE on q (in place) and k, and k, v appended to the caches as rows n_past .. n_past + T - 1, for any T; tab from
// launch_rope_table
prima_status launch_rope_append(const prima_dims &d, float *q, const float *k, const float *v, const float *tab,
                                __half *K, __half *V, int kv_cap, int n_past, int T, hipStream_t st);

// Bounded waits inside kernels (a workgroup that waits for records of other workgroups of its launch) raise this
// flag when they give up; it lives in the window scratch and prima_window_check reports it.
constexpr size_t WAIT_FLAG_BYTES = 256; // the flag is the first word

// 16 bytes per lane from global memory straight into LDS: lane l writes bytes [16 l, 16 l + 16) of the
// 1 KiB at LDS byte address lds_addr (wave-uniform, goes through M0).  Written as inline assembly on
// purpose: the compiler then does not know these loads write LDS and leaves the ordering against the
// later LDS reads to the explicit s_waitcnt vmcnt(N) below, which lets newer stages stay in flight
// (with the builtin it waits for *all* outstanding loads before any LDS read).  Loads complete in
// order, so loads the compiler does not know about can only make its own waits stricter.
// NT: the load carries the non-temporal bit: the line is marked to leave the caches first.  For bytes that are read
// once in a launch (the weight stream of a one-token mat-vec, the cache rows of attention) that was measured 7 % faster
// on a 264 MB launch; not for the several-token mat-vec, whose row runs are short and whose lines that straddle two
// stages or two slabs are then fetched from memory twice.
template <bool NT = false>
__device__ __forceinline__ void dma16(const void *gptr, uint32_t lds_addr)
{
    // one wait state is required between the SALU write of M0 and the load that reads it; M0 is a reserved
    // register that nothing else in this file uses
    if (NT) asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" : : "v"(gptr), "s"(lds_addr) : "memory");
    else asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_addr) : "memory");
}

__device__ __forceinline__ uint32_t lds_address(const void *p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(p)); // low half of a flat LDS pointer is the LDS byte address
}

// value of lane (i + n) % 16 of the same 16-lane row
template <int N>
__device__ __forceinline__ float row_ror(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N, 0xf, 0xf, true));
}
__device__ __forceinline__ float row_max16(float v)
{
    v = fmaxf(v, row_ror<8>(v));
    v = fmaxf(v, row_ror<4>(v));
    v = fmaxf(v, row_ror<2>(v));
    return fmaxf(v, row_ror<1>(v));
}
__device__ __forceinline__ float row_sum16(float v)
{
    v += row_ror<8>(v);
    v += row_ror<4>(v);
    v += row_ror<2>(v);
    return v + row_ror<1>(v);
}

// Combining a value across the four 16-lane rows of a wave without LDS permutes: v_permlane16_swap_b32 a, b
// (gfx950) exchanges the odd rows of a with the even rows of b, v_permlane32_swap_b32 the upper half of a with the
// lower half of b.  With the value in both registers the results are (rows r0 r0 r2 r2, rows r1 r1 r3 r3) and
// (lower half twice, upper half twice); combining the two leaves, in every lane, the combination of its own
// value with the one 16 (32) lanes away.  (ds_bpermute, which __shfl_xor uses for these distances, costs an
// LDS round trip each.)  Written as inline assembly, with the wait states the instruction needs after a VALU
// write of its operands and before a VALU read of its results: the compiler's builtin for it was seen to take
// the two results for the same register (x + y compiled to x + x).
__device__ __forceinline__ void swap16_rows(unsigned &a, unsigned &b)
{
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void swap32_halves(unsigned &a, unsigned &b)
{
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float add_across_16(float v)
{
    unsigned a = __builtin_bit_cast(unsigned, v), b = a;
    swap16_rows(a, b);
    return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
}
__device__ __forceinline__ float add_across_32(float v)
{
    unsigned a = __builtin_bit_cast(unsigned, v), b = a;
    swap32_halves(a, b);
    return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
}
__device__ __forceinline__ float max_across_16(float v)
{
    unsigned a = __builtin_bit_cast(unsigned, v), b = a;
    swap16_rows(a, b);
    return fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}
__device__ __forceinline__ float max_across_32(float v)
{
    unsigned a = __builtin_bit_cast(unsigned, v), b = a;
    swap32_halves(a, b);
    return fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}
// over all 64 lanes, the result in every lane: rotations inside the rows, then across them
__device__ __forceinline__ float wave_sum(float v) { return add_across_32(add_across_16(row_sum16(v))); }
__device__ __forceinline__ float wave_max(float v) { return max_across_32(max_across_16(row_max16(v))); }

} // namespace prima
