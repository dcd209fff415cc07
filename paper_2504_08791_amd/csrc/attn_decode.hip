// GQA decode attention over an fp16 KV cache, split over the KV length, partials merged by
// log-sum-exp.  Per layer and step it reads 2(h_k e_k + h_v e_v) n_kv bytes (arXiv 2504.08791,
// App. A.3, device-loading term) and appends 2(h_k e_k + h_v e_v) bytes per token.
//
// The work per launch is small (tens of KB per compute unit), so the kernel is built as one short
// dependency chain: everything a wave needs is requested from memory in its first instructions, and
// nothing is staged through LDS before the matrix multiply.
// One workgroup handles (key range, KV head, group of up to 8 queries that share the head); each of
// its waves takes 16-key tiles of the range.
//  * Q.K^T runs on the matrix cores: the fp16 cache rows are MFMA operands as they lie in memory
//    (lane (n, c) loads 16 bytes of key n), the queries are loaded by every wave straight into the
//    A-operand layout, rotated there (RoPE partners sit in the same lane), pre-scaled by a power of two
//    and split into fp16 high and low parts that occupy rows 0-7 and 8-15 of the A operand, so the
//    logits carry the queries' full fp32 precision with fp32 accumulation.
//  * softmax statistics are kept online per 16-key tile in fp32; reductions over the 16 keys of a
//    tile are row rotations inside the vector ALU (DPP), not LDS permutes.
//  * P.V runs on the vector ALUs in fp32: a lane owns two output columns for all keys of the tile
//    (one 32-bit load per key), so no reduction across lanes is needed; the probabilities reach the
//    lanes as LDS broadcasts.
//  * fused RoPE + KV append: a workgroup whose key range holds new rows builds them from the projection
//    output (rotate k, round k and v to fp16, nearest even), keeps them in LDS for its own tiles and
//    stores them to the cache on the side, so the appended rows cost no store-to-load round trip.
//  * the workgroup that arrives last at a (KV head, query group) merges the key ranges; partial
//    records travel through device-scope stores and loads, ordered by one counter per group.
#include "attn_common.h"

namespace prima {

struct AttnNoSync {
    __device__ __forceinline__ void wait() {}
};

template <int D, int MODE> // head size, RoPE pairing (0: i with i + D/2, 1: 2i with 2i + 1)
__global__ void __launch_bounds__(ATT_THREADS) attn_decode_kernel(AttnArgs a)
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr bool COH = false;
    const int split = blockIdx.x, kvh = blockIdx.y;
    AttnNoSync sync;
    // the view of this workgroup: all T tokens of one sequence, or (batch) the one token of sequence tok0
    const bool batch = a.batch != 0;
    const int gps = (a.Hq / a.Hkv + QG - 1) / QG; // query groups of one token
    const int tok0 = batch ? blockIdx.z / gps : 0;
    const int qgrp = batch ? blockIdx.z - tok0 * gps : blockIdx.z, nqg = batch ? gps : gridDim.z;
    const int arg_T = batch ? 1 : a.T;
    __half *arg_K = a.K, *arg_V = a.V;
    int arg_n_past = a.n_past;
    if (batch) {
        // read by hand from the argument segment: indexing the by-value argument with a run-time index would
        // make the compiler copy all of it to scratch memory
        typedef const __attribute__((address_space(4))) AttnArgs ConstAttnArgs;
        ConstAttnArgs &ka = *(ConstAttnArgs *)__builtin_amdgcn_kernarg_segment_ptr();
        arg_K = ka.seq_K[tok0];
        arg_V = ka.seq_V[tok0];
        arg_n_past = ka.seq_n_past[tok0];
    }
#include "attn_body.inc"
}

int attn_num_splits(const prima_dims &d, int n_total, int T, bool batch)
{
    const int wgs = d.n_kv_heads * (batch ? query_groups_batch(d, T) : query_groups(d, T));
    const int by_len = (n_total + 16 * ATT_WAVES - 1) / (16 * ATT_WAVES); // at least one 16-key tile per wave
    const int by_grid = (256 + wgs - 1) / wgs;                            // about one workgroup per compute unit
    int ns = by_len < by_grid ? by_len : by_grid;
    if (ns < 1) ns = 1;
    if (ns > MAX_SPLITS) ns = MAX_SPLITS;
    return ns;
}

size_t attn_counter_bytes(const prima_dims &d, int T)
{
    return round_up(static_cast<size_t>(d.n_kv_heads) * query_groups_batch(d, T) * sizeof(unsigned), 256); // >= query_groups(d, T)
}

size_t attn_ws_bytes(const prima_dims &d, int, int T)
{
    return attn_counter_bytes(d, T) + round_up(static_cast<size_t>(T) * d.n_q_heads * MAX_SPLITS * (2 + d.head_dim) * sizeof(float), 256);
}

prima_status launch_attn(const prima_dims &d, const float *q, float *q_rot_out, const float *k_new, const float *v_new,
                         const float *rope_tab, __half *K, __half *V, int kv_cap, int n_past, int T, float *o,
                         void *ws, hipStream_t st, const AttnSeqs *seq)
{
    // several tokens of one sequence: both products on the matrix cores (attn_decode_mt.hip)
    if (!seq && T >= 2) return launch_attn_mt(d, q, q_rot_out, k_new, v_new, rope_tab, K, V, kv_cap, n_past, T, o, ws, st);
    const AttnArgs a = build_attn_args(d, q, q_rot_out, k_new, v_new, rope_tab, K, V, kv_cap, n_past, T, o, ws, seq);
    const dim3 grid(a.nsplit, d.n_kv_heads, seq ? query_groups_batch(d, T) : query_groups(d, T)), block(ATT_THREADS);
    if (d.head_dim == 128 && d.rope_mode == 0) hipLaunchKernelGGL((attn_decode_kernel<128, 0>), grid, block, sizeof(AttnLds<128>), st, a);
    else if (d.head_dim == 128 && d.rope_mode == 1) hipLaunchKernelGGL((attn_decode_kernel<128, 1>), grid, block, sizeof(AttnLds<128>), st, a);
    else if (d.head_dim == 64 && d.rope_mode == 0) hipLaunchKernelGGL((attn_decode_kernel<64, 0>), grid, block, sizeof(AttnLds<64>), st, a);
    else if (d.head_dim == 64 && d.rope_mode == 1) hipLaunchKernelGGL((attn_decode_kernel<64, 1>), grid, block, sizeof(AttnLds<64>), st, a);
    else return PRIMA_E_SHAPE;
    return last_launch_status();
}

} // namespace prima
