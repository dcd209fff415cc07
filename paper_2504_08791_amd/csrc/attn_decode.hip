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
#include "common.h"

namespace prima {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int QG = 8;        // queries per workgroup
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
    float *part;          // [T*Hq][nsplit][2 + D]
    unsigned *arrivals;   // [Hkv * query groups], zero between launches
    float *o;             // [T][Hq][D]
    int Hq, Hkv, kv_cap, n_past, T, nsplit, keys_per_split;
};

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

// Rotate the D/8-element slices a lane holds of one head vector: v[x][e] = element 32x + 8c + e.
// mode 0 pairs element i with i + D/2 (the partner is v[x + NA/2][e] of the same lane), mode 1 pairs
// 2i with 2i + 1.  tab = this token's D/2 (cos, sin) pairs.
template <int D, int MODE>
__device__ __forceinline__ void rope_in_lane(float (&v)[D / 32][8], const float2 *tab, int c)
{
    constexpr int NA = D / 32;
    if (MODE == 0) {
#pragma unroll
        for (int x = 0; x < NA / 2; ++x) {
            const float4 *tp = reinterpret_cast<const float4 *>(tab + 32 * x + 8 * c);
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const float4 cs = tp[h]; // (cos, sin) of pairs 2h, 2h + 1 of this slice
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
            const float4 *tp = reinterpret_cast<const float4 *>(tab + 16 * x + 4 * c);
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const float4 cs = tp[h];
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

template <int D, int MODE> // head size, RoPE pairing (0: i with i + D/2, 1: 2i with 2i + 1)
__global__ void __launch_bounds__(ATT_THREADS) attn_decode_kernel(AttnArgs a)
{
    constexpr int NA = D / 32;   // MFMAs (k-steps of 32) per 16-key tile
    constexpr int DL = D / 2;    // lanes per V row (2 columns each)
    constexpr int KSV = 64 / DL; // V rows per wave instruction (1 or 2)
    constexpr int VPT = 16 / KSV; // V loads per lane per 16-key tile
    const int split = blockIdx.x, kvh = blockIdx.y, qgrp = blockIdx.z;
    const int G = a.Hq / a.Hkv, NQ = G * a.T; // queries on this KV head, index = t*G + hg
    const int q0 = qgrp * QG;
    const int nq = min(QG, NQ - q0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_total = a.n_past + a.T;
    const int p_begin = split * a.keys_per_split;
    const int p_end = min(p_begin + a.keys_per_split, n_total);
    const bool fused = a.k_new != nullptr;

    __shared__ __align__(16) float s_p[ATT_WAVES][16][QG]; // probabilities of the current tile [key][query]
    __shared__ __align__(16) float s_corr[ATT_WAVES][QG];
    __shared__ float s_m[ATT_WAVES][QG], s_l[ATT_WAVES][QG];
    __shared__ __align__(16) float s_o[ATT_WAVES][QG][D];
    __shared__ int s_last;
    __shared__ __align__(16) __half s_knew[PRIMA_MAX_TOK][D], s_vnew[PRIMA_MAX_TOK][D]; // the step's new rows (fused append)

    __half *Kh = a.K + static_cast<int64_t>(kvh) * a.kv_cap * D;
    __half *Vh = a.V + static_cast<int64_t>(kvh) * a.kv_cap * D;

    const int mrow = lane & 15, kc = lane >> 4;
    const int dl = lane % DL, ksl = lane / DL; // P.V: columns 2 dl, 2 dl + 1 of keys ksl, ksl + KSV, ...
    const int last_row = n_total - 1;

    // B operand: lane (n, c) holds elements 32x + 8c .. + 8 of key n.  New rows are not read from the
    // cache but from LDS, where the workgroup has put them (below).
    const bool has_new = fused && p_end > a.n_past;
    auto load_k = [&](int k0, half8 *kbuf) {
        const int krow = min(k0 + mrow, last_row);
        const __half *kp = Kh + static_cast<int64_t>(krow) * D + 8 * kc;
#pragma unroll
        for (int x = 0; x < NA; ++x) kbuf[x] = *reinterpret_cast<const half8 *>(kp + 32 * x);
    };
    auto patch_k = [&](int k0, half8 *kbuf) {
        const int krow = min(k0 + mrow, last_row);
        if (has_new && krow >= a.n_past) {
#pragma unroll
            for (int x = 0; x < NA; ++x) kbuf[x] = *reinterpret_cast<const half8 *>(&s_knew[krow - a.n_past][32 * x + 8 * kc]);
        }
    };
    auto load_v = [&](int k0, uint32_t *vbuf) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int vrow = min(k0 + KSV * i + ksl, last_row);
            vbuf[i] = *reinterpret_cast<const uint32_t *>(Vh + static_cast<int64_t>(vrow) * D + 2 * dl);
        }
    };
    auto patch_v = [&](int k0, uint32_t *vbuf) {
        if (has_new && k0 + 16 > a.n_past) {
#pragma unroll
            for (int i = 0; i < VPT; ++i) {
                const int vrow = min(k0 + KSV * i + ksl, last_row);
                if (vrow >= a.n_past) vbuf[i] = *reinterpret_cast<const uint32_t *>(&s_vnew[vrow - a.n_past][2 * dl]);
            }
        }
    };

    half8 kb[NA];
    uint32_t vb[VPT];
    const int tile_stride = ATT_WAVES * 16;
    int key0 = p_begin + wave * 16;

    // ---- queries: A operand row m holds query m % 8, high part for m < 8, low part otherwise ----
    const int qi_l = mrow & 7;
    const bool q_valid = qi_l < nq;
    // fused RoPE + KV append: a workgroup whose key range holds new rows builds them once (rotate k, round
    // k and v to fp16, nearest even), keeps them in LDS for its own tiles and stores them to the cache on
    // the side; its cache reads of those rows are replaced, never waited for.  When several query groups
    // share the range each writes the same values.  The inputs are requested here, behind the tile.
    constexpr int NPT = (PRIMA_MAX_TOK * (D / 2) + ATT_THREADS - 1) / ATT_THREADS; // new (k pair, v pair)s per thread
    float2 n_cs[NPT], n_k[NPT], n_v[NPT];
    half8 qa[NA];
    float fq_own = 0.f; // logit factor 2^-p / sqrt(D) of query qi_l
    {
        float qv[NA][8];
#pragma unroll
        for (int x = 0; x < NA; ++x)
#pragma unroll
            for (int e = 0; e < 8; ++e) qv[x][e] = 0.f;
        if (q_valid) {
            const int qi = q0 + qi_l, t = qi / G, hg = qi - t * G;
            const int64_t qoff = (static_cast<int64_t>(t) * a.Hq + kvh * G + hg) * D;
            load_slices<D>(a.q + qoff, kc, qv);
        }
        // the queries (cache hits) are requested first, the tile right behind them: loads return in order,
        // so the query preparation below runs while the tile is still on its way from HBM
        if (key0 < p_end) {
            load_k(key0, kb);
            load_v(key0, vb);
        }
        if (has_new) {
#pragma unroll
            for (int k = 0; k < NPT; ++k) {
                const int idx = threadIdx.x + k * ATT_THREADS;
                if (idx < a.T * (D / 2)) {
                    const int t = idx / (D / 2), i = idx - t * (D / 2);
                    const int ia = MODE ? 2 * i : i, ib = MODE ? 2 * i + 1 : i + D / 2;
                    const float *kp = a.k_new + (static_cast<int64_t>(t) * a.Hkv + kvh) * D;
                    n_cs[k] = a.rope_tab[t * (D / 2) + i];
                    n_k[k] = make_float2(kp[ia], kp[ib]);
                    n_v[k] = *reinterpret_cast<const float2 *>(a.v_new + (static_cast<int64_t>(t) * a.Hkv + kvh) * D + 2 * i);
                }
            }
        }
        if (q_valid) {
            const int qi = q0 + qi_l, t = qi / G, hg = qi - t * G;
            const int64_t qoff = (static_cast<int64_t>(t) * a.Hq + kvh * G + hg) * D;
            if (a.rope_tab) {
                rope_in_lane<D, MODE>(qv, a.rope_tab + t * (D / 2), kc);
                if (a.q_rot_out && split == 0 && wave == 0 && mrow < 8) {
#pragma unroll
                    for (int x = 0; x < NA; ++x) {
                        float *dst = a.q_rot_out + qoff + 32 * x + 8 * kc;
                        *reinterpret_cast<float4 *>(dst) = make_float4(qv[x][0], qv[x][1], qv[x][2], qv[x][3]);
                        *reinterpret_cast<float4 *>(dst + 4) = make_float4(qv[x][4], qv[x][5], qv[x][6], qv[x][7]);
                    }
                }
            }
        }
        float amax = 0.f;
#pragma unroll
        for (int x = 0; x < NA; ++x)
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(qv[x][e]));
        amax = fmaxf(amax, __shfl_xor(amax, 16, 64)); // the four slices c of the row
        amax = fmaxf(amax, __shfl_xor(amax, 32, 64));
        int ex = 0;
        if (amax > 0.f) frexpf(amax, &ex); // amax < 2^ex
        int p = 12 - ex;                   // scaled |q| < 2^12
        p = p > 100 ? 100 : (p < -100 ? -100 : p);
        const float S = ldexpf(1.0f, p);
        const bool low = mrow >= 8;
#pragma unroll
        for (int x = 0; x < NA; ++x) {
            half8 h;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float sv = qv[x][e] * S;
                const _Float16 hi = static_cast<_Float16>(sv);
                h[e] = low ? static_cast<_Float16>(sv - static_cast<float>(hi)) : hi;
            }
            qa[x] = h;
        }
        fq_own = q_valid ? ldexpf(1.0f, -p) * rsqrtf(static_cast<float>(D)) : 0.f;
    }
    if (has_new) {
#pragma unroll
        for (int k = 0; k < NPT; ++k) {
            const int idx = threadIdx.x + k * ATT_THREADS;
            if (idx < a.T * (D / 2)) {
                const int t = idx / (D / 2), i = idx - t * (D / 2);
                const int row = a.n_past + t;
                const int ia = MODE ? 2 * i : i, ib = MODE ? 2 * i + 1 : i + D / 2;
                const __half ra = __float2half_rn(n_k[k].x * n_cs[k].x - n_k[k].y * n_cs[k].y);
                const __half rb = __float2half_rn(n_k[k].x * n_cs[k].y + n_k[k].y * n_cs[k].x);
                const __half2 hv = __floats2half2_rn(n_v[k].x, n_v[k].y);
                s_knew[t][ia] = ra;
                s_knew[t][ib] = rb;
                *reinterpret_cast<__half2 *>(&s_vnew[t][2 * i]) = hv;
                if (row >= p_begin && row < p_end) { // the range that owns the row stores it
                    Kh[static_cast<int64_t>(row) * D + ia] = ra;
                    Kh[static_cast<int64_t>(row) * D + ib] = rb;
                    *reinterpret_cast<__half2 *>(Vh + static_cast<int64_t>(row) * D + 2 * i) = hv;
                }
            }
        }
        __syncthreads(); // the new rows are in LDS
        if (key0 < p_end) {
            patch_k(key0, kb);
            patch_v(key0, vb);
        }
    }

    // softmax bookkeeping for the 4 queries this lane sees in the MFMA result: m = 4*(kc&1) + r
    const int mq0 = 4 * (kc & 1);
    float fq[4], m_run[4], l_run[4];
    int lim[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        fq[r] = __shfl(fq_own, mq0 + r, 64); // lane mq0 + r holds query mq0 + r
        const int qi = q0 + mq0 + r;
        lim[r] = (mq0 + r < nq) ? a.n_past + qi / G : -1; // last visible cache row
        m_run[r] = -INFINITY;
        l_run[r] = 0.f;
    }
    float o[QG][2];
#pragma unroll
    for (int i = 0; i < QG; ++i) { o[i][0] = 0.f; o[i][1] = 0.f; }

    while (key0 < p_end) {
        const int next = key0 + tile_stride;
        // logits of 16 keys x 16 A rows (8 high + 8 low query parts)
        v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int x = 0; x < NA; ++x) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(qa[x], kb[x], acc, 0, 0, 0);
        // rows 4kc..4kc+3 of column (key) mrow: add the low-part rows held 32 lanes away
        float pr[4], corr[4];
        const int key = key0 + mrow;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float sv = (acc[r] + __shfl_xor(acc[r], 32, 64)) * fq[r];
            if (key >= p_end || key > lim[r]) sv = -INFINITY;
            const float mn = fmaxf(m_run[r], row_max16(sv));
            corr[r] = (mn == -INFINITY) ? 1.f : __expf(m_run[r] - mn); // exp(-inf) = 0 on the first visible key
            pr[r] = (sv == -INFINITY) ? 0.f : __expf(sv - mn);
            l_run[r] = l_run[r] * corr[r] + row_sum16(pr[r]);
            m_run[r] = mn;
        }
        if (next < p_end) {
            load_k(next, kb);
            patch_k(next, kb);
        }
        if (kc < 2) {
            *reinterpret_cast<float4 *>(&s_p[wave][mrow][mq0]) = make_float4(pr[0], pr[1], pr[2], pr[3]);
            if (mrow == 0) *reinterpret_cast<float4 *>(&s_corr[wave][mq0]) = make_float4(corr[0], corr[1], corr[2], corr[3]);
        }
        __builtin_amdgcn_wave_barrier();
        // P.V
        {
            const float4 c0 = *reinterpret_cast<const float4 *>(&s_corr[wave][0]), c1 = *reinterpret_cast<const float4 *>(&s_corr[wave][4]);
            const float cw[QG] = {c0.x, c0.y, c0.z, c0.w, c1.x, c1.y, c1.z, c1.w};
#pragma unroll
            for (int q = 0; q < QG; ++q) { o[q][0] *= cw[q]; o[q][1] *= cw[q]; }
        }
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int kt = KSV * i + ksl;
            const float4 p0 = *reinterpret_cast<const float4 *>(&s_p[wave][kt][0]);
            const float4 p1 = *reinterpret_cast<const float4 *>(&s_p[wave][kt][4]);
            const float pw[QG] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
            const float2 vf = __half22float2(*reinterpret_cast<const __half2 *>(&vb[i]));
#pragma unroll
            for (int q = 0; q < QG; ++q) {
                o[q][0] = fmaf(pw[q], vf.x, o[q][0]);
                o[q][1] = fmaf(pw[q], vf.y, o[q][1]);
            }
            // finish these keys before the next ones' probabilities are read (otherwise all 16 keys' 128
            // values are fetched up front and the kernel spills)
            if ((i & 3) == 3)
                asm volatile("" : "+v"(o[0][0]), "+v"(o[0][1]), "+v"(o[1][0]), "+v"(o[1][1]), "+v"(o[2][0]), "+v"(o[2][1]), "+v"(o[3][0]), "+v"(o[3][1]),
                                  "+v"(o[4][0]), "+v"(o[4][1]), "+v"(o[5][0]), "+v"(o[5][1]), "+v"(o[6][0]), "+v"(o[6][1]), "+v"(o[7][0]), "+v"(o[7][1])
                             :: "memory");
        }
        __builtin_amdgcn_wave_barrier();
        if (next < p_end) {
            load_v(next, vb);
            patch_v(next, vb);
        }
        key0 = next;
    }

    // ---- the waves' results meet in LDS ----
    if (KSV > 1) {
#pragma unroll
        for (int q = 0; q < QG; ++q) {
            o[q][0] += __shfl_xor(o[q][0], 32, 64);
            o[q][1] += __shfl_xor(o[q][1], 32, 64);
        }
    }
    if (ksl == 0) {
#pragma unroll
        for (int q = 0; q < QG; ++q) *reinterpret_cast<float2 *>(&s_o[wave][q][2 * dl]) = make_float2(o[q][0], o[q][1]);
    }
    if (mrow == 0 && kc < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s_m[wave][mq0 + r] = m_run[r];
            s_l[wave][mq0 + r] = l_run[r];
        }
    }
    __syncthreads();
    const int nqg = gridDim.z;
    for (int idx = threadIdx.x; idx < nq * D; idx += ATT_THREADS) {
        const int i = idx / D, e = idx - i * D;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) mm = fmaxf(mm, s_m[w][i]);
        float ll = 0.f, accv = 0.f;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) {
            const float f = (s_m[w][i] == -INFINITY) ? 0.f : __expf(s_m[w][i] - mm);
            ll += s_l[w][i] * f;
            accv += s_o[w][i][e] * f;
        }
        const int qi = q0 + i, t = qi / G, hg = qi - t * G;
        const int64_t head = static_cast<int64_t>(t) * a.Hq + kvh * G + hg;
        if (a.nsplit == 1) { // nothing to merge
            a.o[head * D + e] = accv / ll;
            continue;
        }
        float *rec = a.part + (head * a.nsplit + split) * (2 + D);
        if (e == 0) {
            __hip_atomic_store(rec, mm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(rec + 1, ll, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __hip_atomic_store(rec + 2 + e, accv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (a.nsplit == 1) return;

    // ---- the last workgroup of this (KV head, query group) merges the key ranges ----
    // o[t][h][:] = sum_i part_i.o * exp(m_i - M) / sum_i part_i.l * exp(m_i - M); a key range that held no
    // visible key has (max, sum) = (-inf, 0) and drops out.  The records were written with device-scope
    // stores; vmcnt(0) + barrier makes them complete before the arrival is counted.
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (threadIdx.x == 0) {
        unsigned *ctr = a.arrivals + kvh * nqg + qgrp;
        const unsigned prev = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = prev + 1 == static_cast<unsigned>(a.nsplit);
        if (last) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); // ready for the next launch
        s_last = last ? 1 : 0;
    }
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (!s_last) return;
    // One wave per query, one round trip: lane s requests (max, sum) of key range s, every lane requests
    // its columns of all ranges right behind; the weights come out of wave reductions and reach the
    // lanes as scalar broadcasts.
    static_assert(QG <= ATT_WAVES, "one wave per query of the group");
    if (wave >= nq) return;
    {
        const int qi = q0 + wave, t = qi / G, hg = qi - t * G;
        const int64_t head = static_cast<int64_t>(t) * a.Hq + kvh * G + hg;
        const float *rec0 = a.part + head * a.nsplit * (2 + D);
        // 2 + D is even and the records start 8-byte aligned: (max, sum) is one 64-bit load
        const uint64_t ml = __hip_atomic_load(reinterpret_cast<const uint64_t *>(rec0 + min(lane, a.nsplit - 1) * (2 + D)),
                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        constexpr int CPL = D / 64; // columns per lane
        float acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] = 0.f;
        const float ms = lane < a.nsplit ? __uint_as_float(static_cast<uint32_t>(ml)) : -INFINITY;
        const float ls = lane < a.nsplit ? __uint_as_float(static_cast<uint32_t>(ml >> 32)) : 0.f;
        float wgt = 0.f;
        for (int s0 = 0; s0 < a.nsplit; s0 += 32) {
            float v[32][CPL];
#pragma unroll
            for (int jj = 0; jj < 32; ++jj)
#pragma unroll
                for (int c = 0; c < CPL; ++c)
                    v[jj][c] = __hip_atomic_load(rec0 + min(s0 + jj, a.nsplit - 1) * (2 + D) + 2 + lane + 64 * c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (s0 == 0) {
                float mm = ms;
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) mm = fmaxf(mm, __shfl_xor(mm, off, 64));
                const float w = (ms == -INFINITY) ? 0.f : __expf(ms - mm);
                float ll = ls * w;
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) ll += __shfl_xor(ll, off, 64);
                wgt = w / ll;
            }
#pragma unroll
            for (int jj = 0; jj < 32; ++jj) {
                // lanes past the last range carry weight 0 (and the clamped loads above are then unused)
                const float wj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wgt), jj)); // s0 == 0
                const float wk = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wgt), 32 + jj));
                const float wsel = s0 == 0 ? wj : wk;
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c] = fmaf(v[jj][c], wsel, acc[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < CPL; ++c) a.o[head * D + lane + 64 * c] = acc[c];
    }
}

static int query_groups(const prima_dims &d, int T)
{
    const int G = d.n_q_heads / d.n_kv_heads;
    return (G * T + QG - 1) / QG;
}

int attn_num_splits(const prima_dims &d, int n_total, int T)
{
    const int wgs = d.n_kv_heads * query_groups(d, T);
    const int by_len = (n_total + 16 * ATT_WAVES - 1) / (16 * ATT_WAVES); // at least one 16-key tile per wave
    const int by_grid = (256 + wgs - 1) / wgs;                            // about one workgroup per compute unit
    int ns = by_len < by_grid ? by_len : by_grid;
    if (ns < 1) ns = 1;
    if (ns > MAX_SPLITS) ns = MAX_SPLITS;
    return ns;
}

size_t attn_counter_bytes(const prima_dims &d, int T)
{
    return round_up(static_cast<size_t>(d.n_kv_heads) * query_groups(d, T) * sizeof(unsigned), 256);
}

size_t attn_ws_bytes(const prima_dims &d, int, int T)
{
    return attn_counter_bytes(d, T) + round_up(static_cast<size_t>(T) * d.n_q_heads * MAX_SPLITS * (2 + d.head_dim) * sizeof(float), 256);
}

prima_status launch_attn(const prima_dims &d, const float *q, float *q_rot_out, const float *k_new, const float *v_new,
                         const float *rope_tab, __half *K, __half *V, int kv_cap, int n_past, int T, float *o,
                         void *ws, hipStream_t st)
{
    const int n_total = n_past + T;
    AttnArgs a{};
    a.q = q; a.q_rot_out = q_rot_out; a.k_new = k_new; a.v_new = v_new;
    a.rope_tab = reinterpret_cast<const float2 *>(rope_tab);
    a.K = K; a.V = V;
    a.arrivals = static_cast<unsigned *>(ws);
    a.part = reinterpret_cast<float *>(static_cast<char *>(ws) + attn_counter_bytes(d, T));
    a.o = o;
    a.Hq = d.n_q_heads; a.Hkv = d.n_kv_heads; a.kv_cap = kv_cap; a.n_past = n_past; a.T = T;
    // key ranges are multiples of 16 so that tiles never straddle two workgroups, and none is empty
    const int want = attn_num_splits(d, n_total, T);
    a.keys_per_split = ((n_total + want - 1) / want + 15) / 16 * 16;
    a.nsplit = (n_total + a.keys_per_split - 1) / a.keys_per_split;
    const dim3 grid(a.nsplit, d.n_kv_heads, query_groups(d, T)), block(ATT_THREADS);
    if (d.head_dim == 128 && d.rope_mode == 0) hipLaunchKernelGGL((attn_decode_kernel<128, 0>), grid, block, 0, st, a);
    else if (d.head_dim == 128 && d.rope_mode == 1) hipLaunchKernelGGL((attn_decode_kernel<128, 1>), grid, block, 0, st, a);
    else if (d.head_dim == 64 && d.rope_mode == 0) hipLaunchKernelGGL((attn_decode_kernel<64, 0>), grid, block, 0, st, a);
    else if (d.head_dim == 64 && d.rope_mode == 1) hipLaunchKernelGGL((attn_decode_kernel<64, 1>), grid, block, 0, st, a);
    else return PRIMA_E_SHAPE;
    return last_launch_status();
}

} // namespace prima
