// GQA decode attention over an fp16 KV cache, split over the KV length, partials merged by
// log-sum-exp.  Per layer and step it reads 2(h_k e_k + h_v e_v) n_kv bytes (arXiv 2504.08791,
// App. A.3, device-loading term).
//
// Work decomposition: the queries that share one KV head (G heads x T tokens) are taken in
// groups of up to QG; a block handles one (key range, KV head, query group).  Inside a wave a
// K/V row is spread over D/8 lanes (8 halfs = one 128-bit load per lane), so one wave
// instruction reads 64/(D/8) consecutive rows, fully coalesced.  Every lane group keeps its own
// running (max, sum, output) per query; groups, waves and key ranges are merged at the end.
#include "common.h"

namespace prima {

constexpr int QG = 8;        // queries per block
constexpr int ATT_WAVES = 4; // waves per block
constexpr int MAX_SPLITS = 64;

__device__ __forceinline__ void unpack8(const uint4 &r, float *f)
{
    const __half2 *h = reinterpret_cast<const __half2 *>(&r);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2 v = __half22float2(h[i]);
        f[2 * i] = v.x;
        f[2 * i + 1] = v.y;
    }
}

// partial record per (query, split): [0] = running max, [1] = sum of exp, [2..2+D) = unnormalised output
template <int D>
__global__ void __launch_bounds__(ATT_WAVES * 64)
attn_partial_kernel(const float *__restrict__ q, const __half *__restrict__ K, const __half *__restrict__ V,
                    float *__restrict__ part, int Hq, int Hkv, int kv_cap, int n_past, int T,
                    int nsplit, int keys_per_split)
{
    constexpr int LPK = D / 8;    // lanes per key row
    constexpr int KPW = 64 / LPK; // key rows per wave instruction
    const int split = blockIdx.x, kvh = blockIdx.y, qgrp = blockIdx.z;
    const int G = Hq / Hkv, NQ = G * T; // queries on this KV head, index = t*G + hg
    const int q0 = qgrp * QG;
    const int nq = min(QG, NQ - q0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int dl = lane % LPK, kl = lane / LPK;
    const float scale = rsqrtf(static_cast<float>(D));

    float qr[QG][8], o[QG][8], m[QG], l[QG];
    int limit[QG]; // last visible cache row per query
#pragma unroll
    for (int i = 0; i < QG; ++i) {
        m[i] = -INFINITY;
        l[i] = 0.f;
        limit[i] = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) { o[i][e] = 0.f; qr[i][e] = 0.f; }
        if (i < nq) {
            const int qi = q0 + i, t = qi / G, hg = qi - t * G;
            const float *qp = q + (static_cast<int64_t>(t) * Hq + kvh * G + hg) * D + dl * 8;
            const float4 a = *reinterpret_cast<const float4 *>(qp), b = *reinterpret_cast<const float4 *>(qp + 4);
            qr[i][0] = a.x * scale; qr[i][1] = a.y * scale; qr[i][2] = a.z * scale; qr[i][3] = a.w * scale;
            qr[i][4] = b.x * scale; qr[i][5] = b.y * scale; qr[i][6] = b.z * scale; qr[i][7] = b.w * scale;
            limit[i] = n_past + t;
        }
    }

    const int p_begin = split * keys_per_split;
    const int p_end = min(p_begin + keys_per_split, n_past + T);
    const __half *Kh = K + static_cast<int64_t>(kvh) * kv_cap * D;
    const __half *Vh = V + static_cast<int64_t>(kvh) * kv_cap * D;

    for (int p = p_begin + wave * KPW + kl; p < p_end; p += ATT_WAVES * KPW) {
        const uint4 kraw = *reinterpret_cast<const uint4 *>(Kh + static_cast<int64_t>(p) * D + dl * 8);
        const uint4 vraw = *reinterpret_cast<const uint4 *>(Vh + static_cast<int64_t>(p) * D + dl * 8);
        float kf[8], vf[8];
        unpack8(kraw, kf);
        unpack8(vraw, vf);
#pragma unroll
        for (int i = 0; i < QG; ++i) {
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) s += qr[i][e] * kf[e];
#pragma unroll
            for (int off = LPK / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
            if (p <= limit[i]) {
                const float mn = fmaxf(m[i], s);
                const float corr = __expf(m[i] - mn); // exp(-inf) = 0 on the first key
                const float pw = __expf(s - mn);
                l[i] = l[i] * corr + pw;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[i][e] = o[i][e] * corr + pw * vf[e];
                m[i] = mn;
            }
        }
    }

    // merge the KPW lane groups of the wave, then the waves through LDS
    __shared__ float sm[ATT_WAVES][QG][2 + D];
#pragma unroll
    for (int i = 0; i < QG; ++i) {
        float mm = m[i];
#pragma unroll
        for (int off = LPK; off < 64; off <<= 1) mm = fmaxf(mm, __shfl_xor(mm, off, 64));
        const float w = (m[i] == -INFINITY) ? 0.f : __expf(m[i] - mm);
        float ll = l[i] * w;
#pragma unroll
        for (int off = LPK; off < 64; off <<= 1) ll += __shfl_xor(ll, off, 64);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = o[i][e] * w;
#pragma unroll
            for (int off = LPK; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
            o[i][e] = v;
        }
        if (kl == 0) {
            if (dl == 0) { sm[wave][i][0] = mm; sm[wave][i][1] = ll; }
#pragma unroll
            for (int e = 0; e < 8; ++e) sm[wave][i][2 + dl * 8 + e] = o[i][e];
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < nq * D; idx += blockDim.x) {
        const int i = idx / D, e = idx - i * D;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) mm = fmaxf(mm, sm[w][i][0]);
        float ll = 0.f, acc = 0.f;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) {
            const float f = (sm[w][i][0] == -INFINITY) ? 0.f : __expf(sm[w][i][0] - mm);
            ll += sm[w][i][1] * f;
            acc += sm[w][i][2 + e] * f;
        }
        const int qi = q0 + i, t = qi / G, hg = qi - t * G;
        float *rec = part + ((static_cast<int64_t>(t) * Hq + kvh * G + hg) * nsplit + split) * (2 + D);
        if (e == 0) { rec[0] = mm; rec[1] = ll; }
        rec[2 + e] = acc;
    }
}

// o[t][h][:] = sum_i part_i.o * exp(m_i - M) / sum_i part_i.l * exp(m_i - M); a key range that
// held no visible key has (max, sum) = (-inf, 0) and drops out.
template <int D>
__global__ void __launch_bounds__(D) attn_merge_kernel(const float *__restrict__ part, float *__restrict__ o, int nsplit)
{
    const int64_t qh = blockIdx.x;
    const int e = threadIdx.x;
    const float *rec = part + qh * nsplit * (2 + D);
    float mm = -INFINITY;
    for (int s = 0; s < nsplit; ++s) mm = fmaxf(mm, rec[s * (2 + D)]);
    float ll = 0.f, acc = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float ms = rec[s * (2 + D)];
        const float f = (ms == -INFINITY) ? 0.f : __expf(ms - mm);
        ll += rec[s * (2 + D) + 1] * f;
        acc += rec[s * (2 + D) + 2 + e] * f;
    }
    o[qh * D + e] = acc / ll;
}

int attn_num_splits(const prima_dims &d, int n_total, int T)
{
    const int G = d.n_q_heads / d.n_kv_heads;
    const int nqg = (G * T + QG - 1) / QG;
    const int by_len = (n_total + 63) / 64;                       // at least 64 keys per block
    const int by_grid = (1024 + d.n_kv_heads * nqg - 1) / (d.n_kv_heads * nqg); // about 4 blocks per CU
    int ns = by_len < by_grid ? by_len : by_grid;
    if (ns < 1) ns = 1;
    if (ns > MAX_SPLITS) ns = MAX_SPLITS;
    return ns;
}

size_t attn_ws_bytes(const prima_dims &d, int, int T)
{
    return round_up(static_cast<size_t>(T) * d.n_q_heads * MAX_SPLITS * (2 + d.head_dim) * sizeof(float), 256);
}

prima_status launch_attn(const prima_dims &d, const float *q, const __half *K, const __half *V,
                         int kv_cap, int n_past, int T, float *o, void *ws, hipStream_t st)
{
    const int n_total = n_past + T;
    const int nsplit = attn_num_splits(d, n_total, T);
    const int kps = (n_total + nsplit - 1) / nsplit;
    const int G = d.n_q_heads / d.n_kv_heads;
    const int nqg = (G * T + QG - 1) / QG;
    float *part = static_cast<float *>(ws);
    const dim3 grid(nsplit, d.n_kv_heads, nqg), block(ATT_WAVES * 64);
    if (d.head_dim == 128) {
        hipLaunchKernelGGL(attn_partial_kernel<128>, grid, block, 0, st, q, K, V, part, d.n_q_heads, d.n_kv_heads,
                           kv_cap, n_past, T, nsplit, kps);
        hipLaunchKernelGGL(attn_merge_kernel<128>, dim3(T * d.n_q_heads), dim3(128), 0, st, part, o, nsplit);
    } else if (d.head_dim == 64) {
        hipLaunchKernelGGL(attn_partial_kernel<64>, grid, block, 0, st, q, K, V, part, d.n_q_heads, d.n_kv_heads,
                           kv_cap, n_past, T, nsplit, kps);
        hipLaunchKernelGGL(attn_merge_kernel<64>, dim3(T * d.n_q_heads), dim3(64), 0, st, part, o, nsplit);
    } else {
        return PRIMA_E_SHAPE;
    }
    return last_launch_status();
}

} // namespace prima
