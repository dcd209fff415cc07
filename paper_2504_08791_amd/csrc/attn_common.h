// Declarations of the attention kernel (the design is described in attn_decode.hip).
#pragma once
#include "common.h"

namespace prima {


typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int QG = 8;        // queries per group in the sizing of the scratch
constexpr int ATT_WAVES = 8; // waves per workgroup
constexpr int ATT_THREADS = ATT_WAVES * 64;
constexpr int MAX_SPLITS = 64;

struct AttnArgs {
    const float *q;       // [T][Hq][D]; rotated already unless rope_tab is set
    float *q_rot_out;     // optional: rotated queries written back (first key range only)
    const float *k_new;   // fused append: un-rotated k [T][Hkv][D], else null
    const float *v_new;   // fused append: v [T][Hkv][D]
    const float2 *rope_tab; // [T][D/2] (cos, sin) or null
    __half *K, *V;        // caches [Hkv][kv_cap][D]
    float *part;          // the key ranges' records [T*Hq][nsplit][4 + D], every word "not written" between launches
    unsigned *err;        // raised when the merging workgroup's bounded wait gives up
    float *o;             // [T][Hq][D]
    int Hq, Hkv, kv_cap, n_past, T, nsplit, keys_per_split;
    // Batch of sequences (continuous batching, App. A.12: one token each): token b is the next token of a
    // sequence of its own, with its own caches and length.  Query group z of the grid then belongs to sequence
    // z / ceil(G / QG), and a workgroup works like a one-token call for that sequence.
    int batch;                       // 0: the T tokens continue one sequence (K, V, n_past above)
    int seq_n_past[PRIMA_MAX_TOK];   // batch: cached rows of sequence b
    __half *seq_K[PRIMA_MAX_TOK], *seq_V[PRIMA_MAX_TOK]; // batch: its caches [Hkv][kv_cap][D]
};

// Rotate the D/8-element slices a lane holds of one head vector: v[x][e] = element 32x + 8c + e.
// mode 0 pairs element i with i + D/2 (the partner is v[x + NA/2][e] of the same lane), mode 1 pairs
// 2i with 2i + 1.  tab = this token's D/2 (cos, sin) pairs.  In two steps, so that the table entries can be
// requested ahead of other loads and used after them: rope_load fetches the lane's D/16 float4 (two (cos, sin)
// pairs each), rope_apply rotates.
template <int D, int MODE>
__device__ __forceinline__ void rope_load(const float2 *tab, int c, float4 (&rt)[D / 16])
{
    constexpr int NA = D / 32;
    if (MODE == 0) {
#pragma unroll
        for (int x = 0; x < NA / 2; ++x) {
            const float4 *tp = reinterpret_cast<const float4 *>(tab + 32 * x + 8 * c);
#pragma unroll
            for (int h = 0; h < 4; ++h) rt[4 * x + h] = tp[h]; // (cos, sin) of pairs 2h, 2h + 1 of this slice
        }
    } else {
#pragma unroll
        for (int x = 0; x < NA; ++x) {
            const float4 *tp = reinterpret_cast<const float4 *>(tab + 16 * x + 4 * c);
#pragma unroll
            for (int h = 0; h < 2; ++h) rt[2 * x + h] = tp[h];
        }
    }
}
template <int D, int MODE>
__device__ __forceinline__ void rope_apply(float (&v)[D / 32][8], const float4 (&rt)[D / 16])
{
    constexpr int NA = D / 32;
    if (MODE == 0) {
#pragma unroll
        for (int x = 0; x < NA / 2; ++x) {
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const float4 cs = rt[4 * x + h];
                const float a0 = v[x][2 * h], b0 = v[x + NA / 2][2 * h], a1 = v[x][2 * h + 1], b1 = v[x + NA / 2][2 * h + 1];
                v[x][2 * h] = a0 * cs.x - b0 * cs.y;
                v[x + NA / 2][2 * h] = a0 * cs.y + b0 * cs.x;
                v[x][2 * h + 1] = a1 * cs.z - b1 * cs.w;
                v[x + NA / 2][2 * h + 1] = a1 * cs.w + b1 * cs.z;
            }
        }
    } else {
#pragma unroll
        for (int x = 0; x < NA; ++x) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float4 cs = rt[2 * x + h];
                const float a0 = v[x][4 * h], b0 = v[x][4 * h + 1], a1 = v[x][4 * h + 2], b1 = v[x][4 * h + 3];
                v[x][4 * h] = a0 * cs.x - b0 * cs.y;
                v[x][4 * h + 1] = a0 * cs.y + b0 * cs.x;
                v[x][4 * h + 2] = a1 * cs.z - b1 * cs.w;
                v[x][4 * h + 3] = a1 * cs.w + b1 * cs.z;
            }
        }
    }
}

template <int D>
__device__ __forceinline__ void load_slices(const float *p, int c, float (&v)[D / 32][8])
{
#pragma unroll
    for (int x = 0; x < D / 32; ++x) {
        const float4 a = *reinterpret_cast<const float4 *>(p + 32 * x + 8 * c), b = *reinterpret_cast<const float4 *>(p + 32 * x + 8 * c + 4);
        v[x][0] = a.x; v[x][1] = a.y; v[x][2] = a.z; v[x][3] = a.w; v[x][4] = b.x; v[x][5] = b.y; v[x][6] = b.z; v[x][7] = b.w;
    }
}

// query groups as the scratch is sized for (groups of QG queries; the kernel's own groups are larger, so fewer)
inline int query_groups(const prima_dims &d, int T)
{
    const int G = d.n_q_heads / d.n_kv_heads;
    return (G * T + QG - 1) / QG;
}
// a batch of T sequences: the groups of one sequence's queries on a KV head, times T
inline int query_groups_batch(const prima_dims &d, int T)
{
    const int G = d.n_q_heads / d.n_kv_heads;
    return (G + QG - 1) / QG * T;
}


// seq (batch): per token its sequence's caches and length (then K, V and n_past are not used)
struct AttnSeqs {
    const int *n_past;
    __half *const *K, *const *V;
};

inline AttnArgs build_attn_args(const prima_dims &d, const float *q, float *q_rot_out, const float *k_new, const float *v_new,
                                const float *rope_tab, __half *K, __half *V, int kv_cap, int n_past, int T, float *o, void *ws,
                                const AttnSeqs *seq = nullptr)
{
    int n_total = n_past + T;
    AttnArgs a{};
    if (seq) {
        a.batch = 1;
        n_total = 0; // the longest sequence sets the key ranges
        for (int b = 0; b < T; ++b) {
            a.seq_n_past[b] = seq->n_past[b];
            a.seq_K[b] = seq->K[b];
            a.seq_V[b] = seq->V[b];
            n_total = seq->n_past[b] + 1 > n_total ? seq->n_past[b] + 1 : n_total;
        }
    }
    a.q = q; a.q_rot_out = q_rot_out; a.k_new = k_new; a.v_new = v_new;
    a.rope_tab = reinterpret_cast<const float2 *>(rope_tab);
    a.K = K; a.V = V;
    a.err = static_cast<unsigned *>(ws);
    a.part = reinterpret_cast<float *>(static_cast<char *>(ws) + attn_counter_bytes(d, T));
    a.o = o;
    a.Hq = d.n_q_heads; a.Hkv = d.n_kv_heads; a.kv_cap = kv_cap; a.n_past = n_past; a.T = T;
    // key ranges are multiples of 16 so that tiles never straddle two workgroups, and none is empty
    attn_ranges(d, n_total, T, seq != nullptr, a.keys_per_split, a.nsplit);
    return a;
}

} // namespace prima
