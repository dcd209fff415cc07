// GQA decode attention over an fp16 KV cache, split over the KV length, partials merged by
// log-sum-exp.  Per layer and step it reads 2(h_k e_k + h_v e_v) n_kv bytes (arXiv 2504.08791,
// App. A.3, device-loading term) and appends 2(h_k e_k + h_v e_v) bytes per token.
//
// One workgroup handles (key range, KV head, group of up to 8 queries that share the head).
//  * Q.K^T runs on the matrix cores: the fp16 cache rows are MFMA operands as they lie in memory
//    (lane (n, c) loads 16 bytes of key n), the queries are pre-scaled by a power of two and split
//    into fp16 high and low parts that occupy rows 0-7 and 8-15 of the A operand, so the logits
//    carry the queries' full fp32 precision with fp32 accumulation.
//  * softmax statistics are kept online per 16-key tile in fp32.
//  * P.V runs on the vector ALUs in fp32: lane (dg, ks) owns 8 output columns for the keys
//    congruent to ks mod 4 (one 128-bit load of V per key), combined across lanes at the end.
//  * when asked, the kernel also does the layer's RoPE and KV append: queries are rotated as they
//    are loaded, and the workgroup whose key range holds the new rows rotates k, rounds k and v to
//    fp16 (nearest even) and stores them before reading them back like any other row.
#include "common.h"

namespace prima {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int QG = 8;        // queries per workgroup
constexpr int ATT_WAVES = 4; // waves per workgroup
constexpr int MAX_SPLITS = 64;

struct AttnArgs {
    const float *q;       // [T][Hq][D]; rotated already unless rope_tab is set
    float *q_rot_out;     // optional: rotated queries written back (split 0 only)
    const float *k_new;   // fused append: un-rotated k [T][Hkv][D], else null
    const float *v_new;   // fused append: v [T][Hkv][D]
    const float2 *rope_tab; // [T][D/2] (cos, sin) or null
    __half *K, *V;        // caches [Hkv][kv_cap][D]
    float *part;          // [T*Hq][nsplit][2 + D]
    int Hq, Hkv, kv_cap, n_past, T, nsplit, keys_per_split, rope_mode;
};

__device__ __forceinline__ void rope_pair_index(int i, int half, int mode, int &ia, int &ib)
{
    ia = mode ? 2 * i : i;
    ib = mode ? 2 * i + 1 : i + half;
}

template <int D>
__global__ void __launch_bounds__(ATT_WAVES * 64, 2) attn_partial_kernel(AttnArgs a)
{
    constexpr int NA = D / 32;   // MFMAs (k-steps of 32) per 16-key tile
    constexpr int DG = D / 8;    // lanes per V row (8 columns each)
    constexpr int KS = 64 / DG;  // V rows per wave instruction
    constexpr int VPT = 16 / KS; // V loads per lane per 16-key tile
    const int split = blockIdx.x, kvh = blockIdx.y, qgrp = blockIdx.z;
    const int G = a.Hq / a.Hkv, NQ = G * a.T; // queries on this KV head, index = t*G + hg
    const int q0 = qgrp * QG;
    const int nq = min(QG, NQ - q0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_total = a.n_past + a.T;
    const int p_begin = split * a.keys_per_split;
    const int p_end = min(p_begin + a.keys_per_split, n_total);

    __shared__ __align__(16) _Float16 s_q[16][D + 8];     // rows 0-7 high parts, 8-15 low parts (+8: bank skew)
    __shared__ float s_fq[QG];                            // per-query logit factor 2^e / sqrt(D)
    __shared__ int s_limit[QG];                           // last visible cache row per query
    __shared__ __align__(16) float s_p[ATT_WAVES][16][QG]; // probabilities of the current tile [key][query]
    __shared__ float s_corr[ATT_WAVES][QG];
    __shared__ float s_m[ATT_WAVES][QG], s_l[ATT_WAVES][QG];
    __shared__ __align__(16) float s_o[ATT_WAVES][QG][D];

    __half *Kh = a.K + static_cast<int64_t>(kvh) * a.kv_cap * D;
    __half *Vh = a.V + static_cast<int64_t>(kvh) * a.kv_cap * D;

    // ---- fused KV append: a workgroup whose range contains new rows writes them first (when several
    // query groups share the range each writes the same values) ----
    if (a.k_new && p_end > a.n_past && p_begin < n_total) {
        for (int idx = threadIdx.x; idx < a.T * (D / 2); idx += blockDim.x) {
            const int t = idx / (D / 2), i = idx - t * (D / 2);
            const int row = a.n_past + t;
            if (row < p_begin || row >= p_end) continue;
            int ia, ib;
            rope_pair_index(i, D / 2, a.rope_mode, ia, ib);
            const float2 cs = a.rope_tab[t * (D / 2) + i];
            const float *kp = a.k_new + (static_cast<int64_t>(t) * a.Hkv + kvh) * D;
            const float ka = kp[ia], kb = kp[ib];
            Kh[static_cast<int64_t>(row) * D + ia] = __float2half_rn(ka * cs.x - kb * cs.y);
            Kh[static_cast<int64_t>(row) * D + ib] = __float2half_rn(ka * cs.y + kb * cs.x);
            const float *vp = a.v_new + (static_cast<int64_t>(t) * a.Hkv + kvh) * D;
            Vh[static_cast<int64_t>(row) * D + 2 * i] = __float2half_rn(vp[2 * i]);
            Vh[static_cast<int64_t>(row) * D + 2 * i + 1] = __float2half_rn(vp[2 * i + 1]);
        }
        __threadfence_block();
    }

    // ---- queries: rotate (if asked), scale by a power of two, split into fp16 high + low ----
    for (int i = threadIdx.x; i < 16 * (D + 8); i += blockDim.x) (&s_q[0][0])[i] = static_cast<_Float16>(0.f);
    __syncthreads();
    // appended rows are visible from here on: request the first tile before staging the queries
    const int mrow = lane & 15, kc = lane >> 4;
    // softmax bookkeeping for the 4 queries this lane sees in the MFMA result: m = 4*(kc&1) + r
    const int mq0 = 4 * (kc & 1);
    // P.V ownership: lane (dg, ks): columns 8dg..8dg+7, keys = tile key 4i + ks (D = 128) or 8i + ks (D = 64)
    const int dg = lane % DG, ks = lane / DG;
    float o[QG][8];
#pragma unroll
    for (int i = 0; i < QG; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[i][e] = 0.f;

    const int last_row = n_total - 1;
    auto load_k = [&](int k0, half8 *kbuf) {
        const int krow = min(k0 + mrow, last_row);
        const __half *kp = Kh + static_cast<int64_t>(krow) * D + 8 * kc;
#pragma unroll
        for (int x = 0; x < NA; ++x) kbuf[x] = *reinterpret_cast<const half8 *>(kp + 32 * x);
    };
    auto load_v = [&](int k0, uint4 *vbuf) {
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int vrow = min(k0 + KS * i + ks, last_row);
            vbuf[i] = *reinterpret_cast<const uint4 *>(Vh + static_cast<int64_t>(vrow) * D + 8 * dg);
        }
    };

    // one K and one V buffer per lane: the next tile's K is requested as soon as the MFMAs have
    // consumed the current one, the next V as soon as P.V is done
    half8 kb[NA];
    uint4 vb[VPT];
    const int tile_stride = ATT_WAVES * 16;
    int key0 = p_begin + wave * 16;
    if (key0 < p_end) {
        load_k(key0, kb);
        load_v(key0, vb);
    }
    if (wave < 2) {
        // wave w handles queries 4w..4w+3, 16 lanes per query
        const int qi_l = wave * 4 + (lane >> 4), sub = lane & 15;
        if (qi_l < nq) {
            const int qi = q0 + qi_l, t = qi / G, hg = qi - t * G;
            const int64_t qoff = (static_cast<int64_t>(t) * a.Hq + kvh * G + hg) * D;
            float v[D / 16];
            float amax = 0.f;
#pragma unroll
            for (int c = 0; c < D / 32; ++c) {
                // pair index i = sub + 16c  (i < D/2)
                const int i = sub + 16 * c;
                int ia, ib;
                rope_pair_index(i, D / 2, a.rope_mode, ia, ib);
                float xa = a.q[qoff + ia], xb = a.q[qoff + ib];
                if (a.rope_tab) {
                    const float2 cs = a.rope_tab[t * (D / 2) + i];
                    const float ra = xa * cs.x - xb * cs.y, rb = xa * cs.y + xb * cs.x;
                    xa = ra;
                    xb = rb;
                    if (a.q_rot_out && split == 0) {
                        a.q_rot_out[qoff + ia] = xa;
                        a.q_rot_out[qoff + ib] = xb;
                    }
                }
                v[2 * c] = xa;
                v[2 * c + 1] = xb;
                amax = fmaxf(amax, fmaxf(fabsf(xa), fabsf(xb)));
            }
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off, 64));
            int ex = 0;
            if (amax > 0.f) frexpf(amax, &ex);  // amax < 2^ex
            int p = 12 - ex;                    // scaled |q| < 2^12
            p = p > 100 ? 100 : (p < -100 ? -100 : p);
            const float S = ldexpf(1.0f, p);
#pragma unroll
            for (int c = 0; c < D / 32; ++c) {
                const int i = sub + 16 * c;
                int ia, ib;
                rope_pair_index(i, D / 2, a.rope_mode, ia, ib);
                const float sa = v[2 * c] * S, sb = v[2 * c + 1] * S;
                const _Float16 ha = static_cast<_Float16>(sa), hb = static_cast<_Float16>(sb);
                s_q[qi_l][ia] = ha;
                s_q[qi_l][ib] = hb;
                s_q[8 + qi_l][ia] = static_cast<_Float16>(sa - static_cast<float>(ha));
                s_q[8 + qi_l][ib] = static_cast<_Float16>(sb - static_cast<float>(hb));
            }
            if (sub == 0) {
                s_fq[qi_l] = ldexpf(1.0f, -p) * rsqrtf(static_cast<float>(D));
                s_limit[qi_l] = a.n_past + t;
            }
        } else if (sub == 0 && qi_l < QG) {
            s_fq[qi_l] = 0.f;
            s_limit[qi_l] = -1;
        }
    }
    __syncthreads();


    // A operands: lane (m = lane%16, c = lane/16) holds s_q[m][32a + 8c .. +8] for a = 0..NA-1
    half8 qa[NA];
#pragma unroll
    for (int x = 0; x < NA; ++x) qa[x] = *reinterpret_cast<const half8 *>(&s_q[mrow][32 * x + 8 * kc]);
    float fq[4], m_run[4], l_run[4];
    int lim[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        fq[r] = s_fq[mq0 + r];
        lim[r] = s_limit[mq0 + r];
        m_run[r] = -INFINITY;
        l_run[r] = 0.f;
    }

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
            float mx = sv;
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
            const float mn = fmaxf(m_run[r], mx);
            corr[r] = (mn == -INFINITY) ? 1.f : __expf(m_run[r] - mn); // exp(-inf) = 0 on the first visible key
            pr[r] = (sv == -INFINITY) ? 0.f : __expf(sv - mn);
            float ps = pr[r];
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) ps += __shfl_xor(ps, off, 64);
            l_run[r] = l_run[r] * corr[r] + ps;
            m_run[r] = mn;
        }
        if (next < p_end) load_k(next, kb);
        if (kc < 2) {
            *reinterpret_cast<float4 *>(&s_p[wave][mrow][mq0]) = make_float4(pr[0], pr[1], pr[2], pr[3]);
            if (mrow == 0) *reinterpret_cast<float4 *>(&s_corr[wave][mq0]) = make_float4(corr[0], corr[1], corr[2], corr[3]);
        }
        __builtin_amdgcn_wave_barrier();
        // P.V
#pragma unroll
        for (int q = 0; q < QG; q += 4) {
            const float4 c4 = *reinterpret_cast<const float4 *>(&s_corr[wave][q]);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                o[q][e] *= c4.x; o[q + 1][e] *= c4.y; o[q + 2][e] *= c4.z; o[q + 3][e] *= c4.w;
            }
        }
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
            const int kt = KS * i + ks;
            const float4 p0 = *reinterpret_cast<const float4 *>(&s_p[wave][kt][0]);
            const float4 p1 = *reinterpret_cast<const float4 *>(&s_p[wave][kt][4]);
            const float pw[QG] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
            const __half2 *h = reinterpret_cast<const __half2 *>(&vb[i]);
            float vf[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float2 f2 = __half22float2(h[e]);
                vf[2 * e] = f2.x;
                vf[2 * e + 1] = f2.y;
            }
#pragma unroll
            for (int q = 0; q < QG; ++q)
#pragma unroll
                for (int e = 0; e < 8; ++e) o[q][e] = fmaf(pw[q], vf[e], o[q][e]);
        }
        __builtin_amdgcn_wave_barrier();
        if (next < p_end) load_v(next, vb);
        key0 = next;
    }

    // ---- merge the KS lane groups of the wave, then the waves ----
#pragma unroll
    for (int q = 0; q < QG; ++q)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float v = o[q][e];
#pragma unroll
            for (int off = DG; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
            o[q][e] = v;
        }
    if (ks == 0) {
#pragma unroll
        for (int q = 0; q < QG; ++q) {
            *reinterpret_cast<float4 *>(&s_o[wave][q][8 * dg]) = make_float4(o[q][0], o[q][1], o[q][2], o[q][3]);
            *reinterpret_cast<float4 *>(&s_o[wave][q][8 * dg + 4]) = make_float4(o[q][4], o[q][5], o[q][6], o[q][7]);
        }
    }
    if (mrow == 0 && kc < 2) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            s_m[wave][mq0 + r] = m_run[r];
            s_l[wave][mq0 + r] = l_run[r];
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < nq * D; idx += blockDim.x) {
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
        float *rec = a.part + ((static_cast<int64_t>(t) * a.Hq + kvh * G + hg) * a.nsplit + split) * (2 + D);
        if (e == 0) { rec[0] = mm; rec[1] = ll; }
        rec[2 + e] = accv;
    }
}

// o[t][h][:] = sum_i part_i.o * exp(m_i - M) / sum_i part_i.l * exp(m_i - M); a key range that
// held no visible key has (max, sum) = (-inf, 0) and drops out.  One workgroup per (token, head).
template <int D>
__global__ void __launch_bounds__(256) attn_merge_kernel(const float *__restrict__ part, float *__restrict__ o, int nsplit)
{
    __shared__ float s_w[MAX_SPLITS];
    __shared__ float s_red[4][D];
    __shared__ float s_L;
    const int64_t qh = blockIdx.x;
    const float *rec = part + qh * nsplit * (2 + D);
    if (threadIdx.x < 64) {
        const int s = threadIdx.x;
        const float ms = s < nsplit ? rec[s * (2 + D)] : -INFINITY;
        const float ls = s < nsplit ? rec[s * (2 + D) + 1] : 0.f;
        float mm = ms;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mm = fmaxf(mm, __shfl_xor(mm, off, 64));
        const float w = (ms == -INFINITY) ? 0.f : __expf(ms - mm);
        float ll = ls * w;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ll += __shfl_xor(ll, off, 64);
        s_w[s] = w;
        if (s == 0) s_L = ll;
    }
    __syncthreads();
    // 256 threads: 256/D groups of splits, D columns
    constexpr int NG = 256 / D;
    const int e = threadIdx.x % D, grp = threadIdx.x / D;
    float acc = 0.f;
#pragma unroll 8
    for (int s = grp; s < nsplit; s += NG) acc = fmaf(rec[s * (2 + D) + 2 + e], s_w[s], acc);
    s_red[grp][e] = acc;
    __syncthreads();
    if (grp == 0) {
        float v = s_red[0][e];
#pragma unroll
        for (int g2 = 1; g2 < NG; ++g2) v += s_red[g2][e];
        o[qh * D + e] = v / s_L;
    }
}

int attn_num_splits(const prima_dims &d, int n_total, int T)
{
    const int G = d.n_q_heads / d.n_kv_heads;
    const int nqg = (G * T + QG - 1) / QG;
    const int by_len = (n_total + 63) / 64;                                     // at least one 16-key tile per wave
    const int by_grid = (512 + d.n_kv_heads * nqg - 1) / (d.n_kv_heads * nqg);  // about 2 workgroups per CU
    int ns = by_len < by_grid ? by_len : by_grid;
    if (ns < 1) ns = 1;
    if (ns > MAX_SPLITS) ns = MAX_SPLITS;
    return ns;
}

size_t attn_ws_bytes(const prima_dims &d, int, int T)
{
    return round_up(static_cast<size_t>(T) * d.n_q_heads * MAX_SPLITS * (2 + d.head_dim) * sizeof(float), 256);
}

prima_status launch_attn(const prima_dims &d, const float *q, float *q_rot_out, const float *k_new, const float *v_new,
                         const float *rope_tab, __half *K, __half *V, int kv_cap, int n_past, int T, float *o,
                         void *ws, hipStream_t st)
{
    const int n_total = n_past + T;
    AttnArgs a{};
    a.q = q; a.q_rot_out = q_rot_out; a.k_new = k_new; a.v_new = v_new;
    a.rope_tab = reinterpret_cast<const float2 *>(rope_tab);
    a.K = K; a.V = V; a.part = static_cast<float *>(ws);
    a.Hq = d.n_q_heads; a.Hkv = d.n_kv_heads; a.kv_cap = kv_cap; a.n_past = n_past; a.T = T;
    a.nsplit = attn_num_splits(d, n_total, T);
    // key ranges are multiples of 16 so that tiles never straddle two workgroups
    a.keys_per_split = ((n_total + a.nsplit - 1) / a.nsplit + 15) / 16 * 16;
    a.rope_mode = d.rope_mode;
    const int G = d.n_q_heads / d.n_kv_heads;
    const int nqg = (G * T + QG - 1) / QG;
    const dim3 grid(a.nsplit, d.n_kv_heads, nqg), block(ATT_WAVES * 64);
    if (d.head_dim == 128) {
        hipLaunchKernelGGL(attn_partial_kernel<128>, grid, block, 0, st, a);
        hipLaunchKernelGGL(attn_merge_kernel<128>, dim3(T * d.n_q_heads), dim3(256), 0, st, a.part, o, a.nsplit);
    } else if (d.head_dim == 64) {
        hipLaunchKernelGGL(attn_partial_kernel<64>, grid, block, 0, st, a);
        hipLaunchKernelGGL(attn_merge_kernel<64>, dim3(T * d.n_q_heads), dim3(256), 0, st, a.part, o, a.nsplit);
    } else {
        return PRIMA_E_SHAPE;
    }
    return last_launch_status();
}

} // namespace prima
