// GQA decode attention over an fp16 KV cache, split over the KV length, partials merged by log-sum-exp.
// Per layer and step it reads 2(h_k e_k + h_v e_v) n_kv bytes (arXiv 2504.08791, App. A.3, device-loading term)
// and appends 2(h_k e_k + h_v e_v) bytes per token.  One token, several tokens of one sequence (speculative
// verification, App. A.12: the G*T queries on a KV head share every key and value they may see, so the work per
// byte of cache is T-fold) or a batch of sequences with one token each.  Both products run on the matrix cores.
//  * A workgroup handles (key range, KV head, group of up to 16 queries); each wave takes 16-key tiles.
//  * Logits transposed, S^T = K Q^T: the cache rows are the A operand as they lie in memory, the queries (RoPE
//    applied in-lane, pre-scaled by a power of two, split into fp16 high and low parts: two MFMAs into one
//    accumulator, so the logits carry the queries' fp32 precision) the B operand.  Lane (q, g) then holds the
//    logits of query q with keys 4g..4g+3, which is exactly the A-operand layout of the second product, so
//    the probabilities never leave the registers.
//  * Online softmax per query: four keys in-lane, the other twelve two shuffles away.
//  * P.V: P (fp16 high + low parts, again two MFMAs into one accumulator: fp32-accurate probabilities) times
//    the 16 x D tile of V.  The cache keeps V row-major [key][d] while the B operand wants four keys of one
//    column per lane, so the tile (contiguous 32 D bytes) goes from global memory straight into LDS and the
//    lanes pick their 2-byte elements from there; tiles are double-buffered per wave.
//  * RoPE + KV append fused: a workgroup whose key range holds new rows builds them once from the projection
//    output (rotate k, round k and v to fp16, nearest even), keeps them in LDS (they replace what the tile
//    loads brought from the cache) and stores them to the cache on the side: no store-to-load round trip.
//  * Waves meet in LDS, key ranges in global memory: every workgroup writes its record (max, sum, D columns) per query
//    with device-scope stores, and the workgroup of the first key range merges them.  It does not wait for an
//    arrival count (a store acknowledgement, an atomic and two dependent loads: four trips through global memory):
//    the records say themselves whether they are complete.  Before a launch every word of a record holds a NaN
//    pattern that no arithmetic produces; the merging workgroup requests (max, sum) and the columns of all ranges
//    in one go and repeats the request until no word shows the pattern (the ranges finish together, so the first or
//    second request succeeds), merges, and writes the pattern back for the next launch.  The polling is bounded
//    (error flag in the scratch); the other workgroups wait for nothing, so the launch always drains.
#include <atomic>

#include "attn_common.h"

namespace prima {

constexpr int QGM = 16; // queries per workgroup
constexpr int MERGE_TRIES = 20000; // requests of the merging workgroup before it gives up (each takes a trip through global memory, ~2 us)

size_t attn_counter_bytes(const prima_dims &d, int T)
{
    return round_up(static_cast<size_t>(d.n_kv_heads) * query_groups_batch(d, T) * sizeof(unsigned), 256); // >= query_groups(d, T)
}

// a key range's record for one query: max, sum, two unused words (the columns start 16-byte aligned), D columns
constexpr int REC_HDR = 4;

size_t attn_ws_bytes(const prima_dims &d, int, int T)
{
    return attn_counter_bytes(d, T) + round_up(static_cast<size_t>(T) * d.n_q_heads * MAX_SPLITS * (REC_HDR + d.head_dim) * sizeof(float), 256);
}


typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

template <int D>
struct AttnTileLds {
    union {
        __half vt[ATT_WAVES][2][16][D]; // V tiles of the loop
        float o[ATT_WAVES][QGM][D];     // afterwards: the waves' un-normalised outputs
    };
    float corr[ATT_WAVES][QGM];
    float m[ATT_WAVES][QGM], l[ATT_WAVES][QGM];
    __half knew[PRIMA_MAX_TOK][D], vnew[PRIMA_MAX_TOK][D]; // the step's new rows (fused append)
    int last;
};

template <int D, int MODE> // head size, RoPE pairing (0: i with i + D/2, 1: 2i with 2i + 1)
__global__ void __launch_bounds__(ATT_THREADS, 4) attn_decode_kernel(AttnArgs a) // 4 waves per SIMD (two workgroups per compute unit): at most 128 VGPRs
{
    extern __shared__ __align__(16) uint8_t smem[];
    constexpr int NA = D / 32; // MFMAs (k-steps of 32) per tile of logits and query part
    constexpr int NB = D / 16; // 16-column blocks of the output
    const int split = blockIdx.x, kvh = blockIdx.y;
    const int G = a.Hq / a.Hkv;
    // The view of this workgroup: arg_T tokens that continue one sequence whose caches are arg_K, arg_V with
    // arg_n_past rows; they are tokens tok0 .. tok0 + arg_T - 1 of the call's q, k_new, v_new, rope_tab and o.
    // A call for one sequence: all of its tokens.  A batch of sequences: the one token of sequence tok0, whose
    // caches and length are read by hand from the argument segment (indexing the by-value argument with a
    // run-time index would make the compiler copy all of it to scratch memory).
    // A prompt (batch == 2, caches complete, one key range): piece z / gps of the grid is a call of its own for the
    // tokens 16 piece .. 16 piece + 15, which see the n_past + 16 piece rows before them and, causally, their own.
    const bool batch = a.batch == 1, prompt = a.batch == 2, pieces = batch || prompt;
    const int gps = prompt ? (G * PRIMA_MAX_TOK + QGM - 1) / QGM : (G + QGM - 1) / QGM; // query groups of one token / one piece
    const int piece = pieces ? blockIdx.z / gps : 0;
    const int tok0 = prompt ? piece * PRIMA_MAX_TOK : piece;
    const int qgrp = pieces ? blockIdx.z - piece * gps : blockIdx.z, nqg = pieces ? gps : gridDim.z;
    const int arg_T = batch ? 1 : (prompt ? PRIMA_MAX_TOK : a.T);
    __half *arg_K = a.K, *arg_V = a.V;
    int arg_n_past = a.n_past + (prompt ? tok0 : 0);
    if (batch) {
        typedef const __attribute__((address_space(4))) AttnArgs ConstAttnArgs;
        ConstAttnArgs &ka = *(ConstAttnArgs *)__builtin_amdgcn_kernarg_segment_ptr();
        arg_K = ka.seq_K[tok0];
        arg_V = ka.seq_V[tok0];
        arg_n_past = ka.seq_n_past[tok0];
    }
    const int NQ = G * arg_T; // queries on this KV head, index = t*G + hg
    const int q0 = qgrp * QGM;
    const int nq = min(QGM, NQ - q0);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_total = arg_n_past + arg_T;
    const int p_begin = split * a.keys_per_split;
    const int p_end = min(p_begin + a.keys_per_split, n_total);
    const bool fused = a.k_new != nullptr;

    AttnTileLds<D> &lds = *reinterpret_cast<AttnTileLds<D> *>(smem);
    __half *Kh = arg_K + static_cast<int64_t>(kvh) * a.kv_cap * D;
    __half *Vh = arg_V + static_cast<int64_t>(kvh) * a.kv_cap * D;

    const int col = lane & 15, g = lane >> 4; // MFMA lane coordinates
    const int last_row = n_total - 1;
    const bool has_new = fused && p_end > arg_n_past;

    // A operand of the logits: lane (key, c) holds elements 32x + 8c .. + 8 of the key.  New rows come from LDS.
    auto load_k = [&](int k0, half8 *kbuf) __attribute__((always_inline)) {
        const int krow = min(k0 + col, last_row);
        const __half *kp = Kh + static_cast<int64_t>(krow) * D + 8 * g;
#pragma unroll
        for (int x = 0; x < NA; ++x) kbuf[x] = *reinterpret_cast<const half8 *>(kp + 32 * x);
    };
    auto patch_k = [&](int k0, half8 *kbuf) __attribute__((always_inline)) {
        const int krow = min(k0 + col, last_row);
        if (has_new && krow >= arg_n_past) {
#pragma unroll
            for (int x = 0; x < NA; ++x) kbuf[x] = *reinterpret_cast<const half8 *>(&lds.knew[krow - arg_n_past][32 * x + 8 * g]);
        }
    };
    // the 16 x D tile of V into this wave's LDS buffer `buf`: 1 KiB (1024 / 2D rows) per instruction; rows past
    // the last one re-read it.  Nothing the compiler knows of waits for these loads: s_waitcnt vmcnt(0) below.
    auto request_v = [&](int k0, int buf) __attribute__((always_inline)) {
        constexpr int LPR = D / 8;        // lanes per row
        constexpr int RPI = 64 / LPR;     // rows per instruction
        const uint32_t dst = __builtin_amdgcn_readfirstlane(lds_address(&lds.vt[wave][buf][0][0]));
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); // reads of the buffer being overwritten have returned
#pragma unroll
        for (int i = 0; i < 16 / RPI; ++i) {
            const int vrow = min(k0 + RPI * i + lane / LPR, last_row);
            dma16<true>(Vh + static_cast<int64_t>(vrow) * D + (lane % LPR) * 8, dst + i * 1024);
        }
    };

    half8 kb[NA];
    const int tile_stride = ATT_WAVES * 16;
    int key0 = p_begin + wave * 16;

    // ---- queries: lane (q, c) holds the slices c of query q (B operand of the logits), high and low parts ----
    const bool q_valid = col < nq;
    const int qi = q0 + col, q_t = qi / G, q_hg = qi - q_t * G;
    const int64_t qoff = (static_cast<int64_t>(tok0 + q_t) * a.Hq + kvh * G + q_hg) * D;
    constexpr int NPT = (PRIMA_MAX_TOK * (D / 2) + ATT_THREADS - 1) / ATT_THREADS; // new (k pair, v pair)s per thread
    float2 n_cs[NPT], n_k[NPT], n_v[NPT];
    half8 qh[NA], ql[NA];
    float fq = 0.f; // logit factor 2^-p / sqrt(D) of this lane's query
    {
        float qv[NA][8];
        float4 q_rt[D / 16];
#pragma unroll
        for (int x = 0; x < NA; ++x)
#pragma unroll
            for (int e = 0; e < 8; ++e) qv[x][e] = 0.f;
        if (q_valid) {
            load_slices<D>(a.q + qoff, g, qv);
            if (a.rope_tab) rope_load<D, MODE>(a.rope_tab + (tok0 + q_t) * (D / 2), g, q_rt);
        }
        // the first tile right behind the queries: they are prepared while it is on its way
        if (key0 < p_end) {
            load_k(key0, kb);
            request_v(key0, 0);
        }
        if (has_new) {
#pragma unroll
            for (int k = 0; k < NPT; ++k) {
                const int idx = threadIdx.x + k * ATT_THREADS;
                if (idx < arg_T * (D / 2)) {
                    const int t = idx / (D / 2), i = idx - t * (D / 2);
                    const int ia = MODE ? 2 * i : i, ib = MODE ? 2 * i + 1 : i + D / 2;
                    const float *kp = a.k_new + (static_cast<int64_t>(tok0 + t) * a.Hkv + kvh) * D;
                    n_cs[k] = a.rope_tab[(tok0 + t) * (D / 2) + i];
                    n_k[k] = make_float2(kp[ia], kp[ib]);
                    n_v[k] = *reinterpret_cast<const float2 *>(a.v_new + (static_cast<int64_t>(tok0 + t) * a.Hkv + kvh) * D + 2 * i);
                }
            }
        }
        if (q_valid && a.rope_tab) {
            rope_apply<D, MODE>(qv, q_rt);
            if (a.q_rot_out && split == 0 && wave == 0) {
#pragma unroll
                for (int x = 0; x < NA; ++x) {
                    float *dst = a.q_rot_out + qoff + 32 * x + 8 * g;
                    *reinterpret_cast<float4 *>(dst) = make_float4(qv[x][0], qv[x][1], qv[x][2], qv[x][3]);
                    *reinterpret_cast<float4 *>(dst + 4) = make_float4(qv[x][4], qv[x][5], qv[x][6], qv[x][7]);
                }
            }
        }
        float amax = 0.f;
#pragma unroll
        for (int x = 0; x < NA; ++x)
#pragma unroll
            for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(qv[x][e]));
        amax = max_across_32(max_across_16(amax)); // the four slices of the query
        int ex = 0;
        if (amax > 0.f) frexpf(amax, &ex); // amax < 2^ex
        int p = 12 - ex;                   // scaled |q| < 2^12
        p = p > 100 ? 100 : (p < -100 ? -100 : p);
        const float S = ldexpf(1.0f, p);
#pragma unroll
        for (int x = 0; x < NA; ++x) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float sv = qv[x][e] * S;
                const _Float16 hi = static_cast<_Float16>(sv);
                qh[x][e] = hi;
                ql[x][e] = static_cast<_Float16>(sv - static_cast<float>(hi));
            }
        }
        fq = q_valid ? ldexpf(1.0f, -p) * rsqrtf(static_cast<float>(D)) : 0.f;
    }
    const int lim = q_valid ? arg_n_past + q_t : -1; // last cache row this lane's query may see
    if (has_new) {
        // fused RoPE + KV append: rotate k, round k and v to fp16 (nearest even), keep the rows in LDS for this
        // workgroup's tiles, and the range that owns a row stores it to the cache
#pragma unroll
        for (int k = 0; k < NPT; ++k) {
            const int idx = threadIdx.x + k * ATT_THREADS;
            if (idx < arg_T * (D / 2)) {
                const int t = idx / (D / 2), i = idx - t * (D / 2);
                const int row = arg_n_past + t;
                const int ia = MODE ? 2 * i : i, ib = MODE ? 2 * i + 1 : i + D / 2;
                const __half ra = __float2half_rn(n_k[k].x * n_cs[k].x - n_k[k].y * n_cs[k].y);
                const __half rb = __float2half_rn(n_k[k].x * n_cs[k].y + n_k[k].y * n_cs[k].x);
                const __half2 hv = __floats2half2_rn(n_v[k].x, n_v[k].y);
                lds.knew[t][ia] = ra;
                lds.knew[t][ib] = rb;
                *reinterpret_cast<__half2 *>(&lds.vnew[t][2 * i]) = hv;
                if (row >= p_begin && row < p_end) {
                    Kh[static_cast<int64_t>(row) * D + ia] = ra;
                    Kh[static_cast<int64_t>(row) * D + ib] = rb;
                    *reinterpret_cast<__half2 *>(Vh + static_cast<int64_t>(row) * D + 2 * i) = hv;
                }
            }
        }
        __syncthreads(); // the new rows are in LDS
        if (key0 < p_end) patch_k(key0, kb);
    }

    float m_run = -INFINITY, l_run = 0.f; // of this lane's query (the same in its four lanes)
    v4f oacc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) oacc[nb] = {0.f, 0.f, 0.f, 0.f};
    int buf = 0;

    while (key0 < p_end) {
        const int next = key0 + tile_stride;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); // this tile's V is in LDS (its K is waited for by the compiler)
        if (has_new && key0 + 16 > arg_n_past) {
            // rows of this step in the tile, and the rows past the last one (which repeat it): what the cache
            // held for them is replaced, so that nothing undefined meets a zero probability
            for (int r = max(0, arg_n_past - key0); r < 16; ++r)
                if (lane < D / 2)
                    reinterpret_cast<uint32_t *>(&lds.vt[wave][buf][r][0])[lane] =
                        reinterpret_cast<const uint32_t *>(&lds.vnew[min(key0 + r, last_row) - arg_n_past][0])[lane];
            __builtin_amdgcn_wave_barrier();
        }
        // logits, transposed: rows = keys 4g..4g+3, column = this lane's query
        v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int x = 0; x < NA; ++x) {
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb[x], qh[x], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(kb[x], ql[x], acc, 0, 0, 0);
        }
        float sv[4], tmax = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int key = key0 + 4 * g + r;
            sv[r] = (key >= p_end || key > lim) ? -INFINITY : acc[r] * fq;
            tmax = fmaxf(tmax, sv[r]);
        }
        tmax = max_across_32(max_across_16(tmax));
        const float mn = fmaxf(m_run, tmax);
        const float corr = (mn == -INFINITY) ? 1.f : __expf(m_run - mn); // exp(-inf) = 0 on the first visible key
        float pr[4], ps = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            pr[r] = (sv[r] == -INFINITY) ? 0.f : __expf(sv[r] - mn);
            ps += pr[r];
        }
        ps = add_across_32(add_across_16(ps));
        l_run = l_run * corr + ps;
        m_run = mn;
        // the next tile: its K replaces the one just consumed, its V goes to the other buffer
        if (next < p_end) {
            load_k(next, kb);
            patch_k(next, kb);
            request_v(next, buf ^ 1);
        }
        // rescale what has been accumulated (rows of the accumulators are queries 4g..4g+3: their factors come
        // from the lanes that own those queries, through LDS); skipped when no maximum moved
        if (__ballot(corr != 1.f) != 0) {
            if (g == 0) lds.corr[wave][col] = corr;
            __builtin_amdgcn_wave_barrier();
            const float4 c4 = *reinterpret_cast<const float4 *>(&lds.corr[wave][4 * g]);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                oacc[nb][0] *= c4.x;
                oacc[nb][1] *= c4.y;
                oacc[nb][2] *= c4.z;
                oacc[nb][3] *= c4.w;
            }
            __builtin_amdgcn_wave_barrier();
        }
        // P.V: the probabilities are the A operand as they stand (keys 4g..4g+3 of this lane's query)
        half4 ph, pl;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const _Float16 hi = static_cast<_Float16>(pr[r]);
            ph[r] = hi;
            pl[r] = static_cast<_Float16>(pr[r] - static_cast<float>(hi));
        }
        // B operand: lane (col, g) wants V[key 4g + r][16 nb + col], r = 0..3, out of the row-major tile.  The LDS
        // transpose read does that in one instruction: in each group of 16 lanes, lane i names four consecutive halves
        // (here those of key 4g + i / 4 from column 16 nb + 4 (i % 4)) and receives, of the halves named by lanes
        // i / 4 + 4 r, the one at position i % 4.
        const _Float16 *vt = reinterpret_cast<const _Float16 *>(&lds.vt[wave][buf][4 * g + (col >> 2)][4 * (col & 3)]);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            typedef short v4s __attribute__((ext_vector_type(4)));
            const v4s vraw = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) v4s *)(static_cast<uintptr_t>(lds_address(vt + 16 * nb))));
            const half4 vb = __builtin_bit_cast(half4, vraw);
            oacc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(ph, vb, oacc[nb], 0, 0, 0);
            oacc[nb] = __builtin_amdgcn_mfma_f32_16x16x16f16(pl, vb, oacc[nb], 0, 0, 0);
        }
        buf ^= 1;
        key0 = next;
    }

    // ---- the waves' results meet in LDS (the V tiles are not needed any more) ----
    __syncthreads();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 4; ++r) lds.o[wave][4 * g + r][16 * nb + col] = oacc[nb][r];
    if (g == 0) {
        lds.m[wave][col] = m_run;
        lds.l[wave][col] = l_run;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < nq * D; idx += ATT_THREADS) {
        const int i = idx / D, e = idx - i * D;
        float mm = -INFINITY;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) mm = fmaxf(mm, lds.m[w][i]);
        float ll = 0.f, accv = 0.f;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) {
            const float f = (lds.m[w][i] == -INFINITY) ? 0.f : __expf(lds.m[w][i] - mm);
            ll += lds.l[w][i] * f;
            accv += lds.o[w][i][e] * f;
        }
        const int qj = q0 + i, t = qj / G, hg = qj - t * G;
        const int64_t head = static_cast<int64_t>(tok0 + t) * a.Hq + kvh * G + hg;
        if (a.nsplit == 1) { // nothing to merge
            a.o[head * D + e] = accv / ll;
            continue;
        }
        float *rec = a.part + (head * a.nsplit + split) * (REC_HDR + D);
        if (e == 0) {
            __hip_atomic_store(rec, mm, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(rec + 1, ll, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __hip_atomic_store(rec + REC_HDR + e, accv, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (a.nsplit == 1 || split != 0) return;

    // ---- the workgroup of the first key range merges the ranges of its (KV head, query group) ----
    // o[t][h][:] = sum_i part_i.o * exp(m_i - M) / sum_i part_i.l * exp(m_i - M); a key range that held no
    // visible key has (max, sum) = (-inf, 0) and drops out.  One wave per query at a time: lane s takes (max, sum) of
    // range s; a load instruction brings RPI whole records' columns (16 bytes a lane), MERGE_LD instructions a request.
    constexpr int LPR = D / 4;        // lanes per record
    constexpr int RPI = 64 / LPR;     // records per load instruction
    constexpr int MERGE_LD = 16;      // load instructions per request: 32 (D = 128) or 64 (D = 64) records
    const int sub = lane / LPR, c4 = (lane % LPR) * 4;
    constexpr int REC_BYTES = (REC_HDR + D) * 4;
    constexpr int HALF_LD = MERGE_LD / 2;
    // scalar base of query qq's records
    auto records_of = [&](int qq, int64_t &head) __attribute__((always_inline)) {
        const int qj = q0 + qq, t = qj / G, hg = qj - t * G;
        head = static_cast<int64_t>(tok0 + t) * a.Hq + kvh * G + hg;
        const uint64_t rec_addr = reinterpret_cast<uint64_t>(a.part + head * a.nsplit * (REC_HDR + D));
        // (the builtin returns a signed int: through uint32_t, or the low half's sign would spill into the high half)
        const uint32_t rec_lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(rec_addr))));
        const uint32_t rec_hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(rec_addr >> 32))));
        return reinterpret_cast<const char *>(static_cast<uint64_t>(rec_lo) | (static_cast<uint64_t>(rec_hi) << 32));
    };
    if (nq > ATT_WAVES && a.nsplit <= HALF_LD * RPI) {
        // More queries than waves and few ranges: a request brings the records of TWO queries of the wave (qq and
        // qq + ATT_WAVES; half of its load instructions each), so the second query costs no trip through memory of
        // its own.  Per query the same records are added in the same order as below: the same bits.
        for (int qq = wave; qq < nq; qq += 2 * ATT_WAVES) {
            const bool two = qq + ATT_WAVES < nq;
            int64_t head[2];
            const char *const recA = records_of(qq, head[0]);
            const char *const recB = records_of(two ? qq + ATT_WAVES : qq, head[1]);
            const uint32_t col_off = static_cast<uint32_t>(sub * REC_BYTES + (REC_HDR + c4) * 4);
            const uint32_t ml_off = static_cast<uint32_t>(min(lane, a.nsplit - 1) * REC_BYTES);
            v4f v[MERGE_LD];
            v2f mlA = {0.f, 0.f}, mlB = {0.f, 0.f};
            int tries = 0;
            for (;;) {
                asm volatile("global_load_dwordx2 %0, %1, %2 sc1" : "=&v"(mlA) : "v"(ml_off), "s"(recA) : "memory");
                asm volatile("global_load_dwordx2 %0, %1, %2 sc1" : "=&v"(mlB) : "v"(ml_off), "s"(recB) : "memory");
#pragma unroll
                for (int i = 0; i < HALF_LD; ++i)
                    asm volatile("global_load_dwordx4 %0, %1, %2 sc1" : "=&v"(v[i]) : "v"(col_off), "s"(recA + i * RPI * REC_BYTES) : "memory");
#pragma unroll
                for (int i = 0; i < HALF_LD; ++i)
                    asm volatile("global_load_dwordx4 %0, %1, %2 sc1" : "=&v"(v[HALF_LD + i]) : "v"(col_off), "s"(recB + i * RPI * REC_BYTES) : "memory");
                asm volatile("s_waitcnt vmcnt(0)"
                             : "+v"(mlA), "+v"(mlB), "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                               "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
                             :: "memory");
                bool missing = __float_as_uint(mlA[0]) == ATTN_REC_EMPTY || __float_as_uint(mlA[1]) == ATTN_REC_EMPTY ||
                               __float_as_uint(mlB[0]) == ATTN_REC_EMPTY || __float_as_uint(mlB[1]) == ATTN_REC_EMPTY;
#pragma unroll
                for (int i = 0; i < MERGE_LD; ++i)
                    missing = missing || ((i % HALF_LD) * RPI + sub < a.nsplit &&
                                          (__float_as_uint(v[i][0]) == ATTN_REC_EMPTY || __float_as_uint(v[i][1]) == ATTN_REC_EMPTY ||
                                           __float_as_uint(v[i][2]) == ATTN_REC_EMPTY || __float_as_uint(v[i][3]) == ATTN_REC_EMPTY));
                if (__ballot(missing) == 0ull) break;
                if (++tries > MERGE_TRIES) { // never expected: give up, say so, and go on with what there is
                    if (lane == 0) __hip_atomic_store(a.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                if (x == 1 && !two) break;
                const v2f ml = x ? mlB : mlA;
                const char *const rec0 = x ? recB : recA;
                const float ms = lane < a.nsplit ? ml[0] : -INFINITY;
                const float ls = lane < a.nsplit ? ml[1] : 0.f;
                const float mm = wave_max(ms);
                const float w = (ms == -INFINITY) ? 0.f : __expf(ms - mm);
                const float ll = wave_sum(ls * w);
                const float wgt = w / ll; // lanes past the last range carry weight 0
                if (lane < a.nsplit) // "not written" again, for the next launch
                    *reinterpret_cast<uint2 *>(const_cast<char *>(rec0) + ml_off) = make_uint2(ATTN_REC_EMPTY, ATTN_REC_EMPTY);
                v4f accq = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < HALF_LD; ++i) {
                    const int r = i * RPI + sub;
                    const float ws = __shfl(wgt, min(r, 63), 64);
                    if (r < a.nsplit) {
                        const v4f vv = v[x * HALF_LD + i];
                        accq[0] = fmaf(vv[0], ws, accq[0]);
                        accq[1] = fmaf(vv[1], ws, accq[1]);
                        accq[2] = fmaf(vv[2], ws, accq[2]);
                        accq[3] = fmaf(vv[3], ws, accq[3]);
                        *reinterpret_cast<uint4 *>(const_cast<char *>(rec0) + i * RPI * REC_BYTES + col_off) =
                            make_uint4(ATTN_REC_EMPTY, ATTN_REC_EMPTY, ATTN_REC_EMPTY, ATTN_REC_EMPTY);
                    }
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (RPI == 4) accq[k] = add_across_16(accq[k]);
                    accq[k] = add_across_32(accq[k]);
                }
                if (lane < LPR) *reinterpret_cast<float4 *>(a.o + head[x] * D + c4) = make_float4(accq[0], accq[1], accq[2], accq[3]);
            }
        }
        return;
    }
    for (int qq = wave; qq < nq; qq += ATT_WAVES) {
        // this query's records: a scalar base (the query is the wave's) and one offset per lane, so that the requests
        // of a pass need no address registers of their own.  Records past the last range are read too (they lie
        // inside the scratch, which is sized for MAX_SPLITS ranges per query) and ignored.
        int64_t head;
        const char *const rec0 = records_of(qq, head);
        const uint32_t col_off = static_cast<uint32_t>(sub * REC_BYTES + (REC_HDR + c4) * 4);
        const uint32_t ml_off = static_cast<uint32_t>(min(lane, a.nsplit - 1) * REC_BYTES);
        float mm = 0.f, wgt = 0.f;
        v4f accq = {0.f, 0.f, 0.f, 0.f};
        for (int s0 = 0; s0 < a.nsplit; s0 += MERGE_LD * RPI) {
            const char *const pass0 = rec0 + static_cast<int64_t>(s0) * REC_BYTES;
            v4f v[MERGE_LD];
            v2f ml = {0.f, 0.f};
            int tries = 0;
            for (;;) {
                if (s0 == 0) asm volatile("global_load_dwordx2 %0, %1, %2 sc1" : "=&v"(ml) : "v"(ml_off), "s"(rec0) : "memory");
#pragma unroll
                for (int i = 0; i < MERGE_LD; ++i)
                    asm volatile("global_load_dwordx4 %0, %1, %2 sc1" : "=&v"(v[i]) : "v"(col_off), "s"(pass0 + i * RPI * REC_BYTES) : "memory");
                // the compiler does not know these loads: one wait that names every register
                asm volatile("s_waitcnt vmcnt(0)"
                             : "+v"(ml), "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]),
                               "+v"(v[8]), "+v"(v[9]), "+v"(v[10]), "+v"(v[11]), "+v"(v[12]), "+v"(v[13]), "+v"(v[14]), "+v"(v[15])
                             :: "memory");
                bool missing = s0 == 0 && (__float_as_uint(ml[0]) == ATTN_REC_EMPTY || __float_as_uint(ml[1]) == ATTN_REC_EMPTY);
#pragma unroll
                for (int i = 0; i < MERGE_LD; ++i)
                    missing = missing || (s0 + i * RPI + sub < a.nsplit &&
                                          (__float_as_uint(v[i][0]) == ATTN_REC_EMPTY || __float_as_uint(v[i][1]) == ATTN_REC_EMPTY ||
                                           __float_as_uint(v[i][2]) == ATTN_REC_EMPTY || __float_as_uint(v[i][3]) == ATTN_REC_EMPTY));
                if (__ballot(missing) == 0ull) break;
                if (++tries > MERGE_TRIES) { // never expected: give up, say so, and go on with what there is
                    if (lane == 0) __hip_atomic_store(a.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    break;
                }
            }
            if (s0 == 0) {
                const float ms = lane < a.nsplit ? ml[0] : -INFINITY;
                const float ls = lane < a.nsplit ? ml[1] : 0.f;
                mm = wave_max(ms);
                const float w = (ms == -INFINITY) ? 0.f : __expf(ms - mm);
                const float ll = wave_sum(ls * w);
                wgt = w / ll; // lanes past the last range carry weight 0
                if (lane < a.nsplit) // "not written" again, for the next launch
                    *reinterpret_cast<uint2 *>(const_cast<char *>(rec0) + ml_off) = make_uint2(ATTN_REC_EMPTY, ATTN_REC_EMPTY);
            }
#pragma unroll
            for (int i = 0; i < MERGE_LD; ++i) {
                const int r = s0 + i * RPI + sub;
                const float ws = __shfl(wgt, min(r, 63), 64);
                if (r < a.nsplit) {
                    accq[0] = fmaf(v[i][0], ws, accq[0]);
                    accq[1] = fmaf(v[i][1], ws, accq[1]);
                    accq[2] = fmaf(v[i][2], ws, accq[2]);
                    accq[3] = fmaf(v[i][3], ws, accq[3]);
                    *reinterpret_cast<uint4 *>(const_cast<char *>(pass0) + i * RPI * REC_BYTES + col_off) =
                        make_uint4(ATTN_REC_EMPTY, ATTN_REC_EMPTY, ATTN_REC_EMPTY, ATTN_REC_EMPTY);
                }
            }
        }
        // the RPI groups of lanes hold different ranges' shares of the same columns
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (RPI == 4) accq[k] = add_across_16(accq[k]);
            accq[k] = add_across_32(accq[k]);
        }
        if (lane < LPR) *reinterpret_cast<float4 *>(a.o + head * D + c4) = make_float4(accq[0], accq[1], accq[2], accq[3]);
    }
}

// key ranges for several tokens of one sequence: about one workgroup per compute unit
static int tile_query_groups(const prima_dims &d, int T, bool batch)
{
    const int G = d.n_q_heads / d.n_kv_heads;
    return batch ? (G + QGM - 1) / QGM * T : (G * T + QGM - 1) / QGM;
}

static int tile_num_splits(const prima_dims &d, int n_total, int T, bool batch)
{
    const int wgs = d.n_kv_heads * tile_query_groups(d, T, batch);
    // at least two 16-key tiles per wave: every key range costs a record, an arrival and a share of the merge
    // (4096 rows, one token: 16 ranges 14.8 us, 32 ranges 16.0 us, 8 ranges 16.8 us)
    const int by_len = n_total / (32 * ATT_WAVES); // (rounded down: 4097 rows are 16 ranges of 257, not 16 of 256 and one of 1)
    const int by_grid = (256 + wgs - 1) / wgs; // measured: 128, 192 and 384 workgroups are slower
    int ns = by_len < by_grid ? by_len : by_grid;
    if (ns < 1) ns = 1;
    if (ns > MAX_SPLITS) ns = MAX_SPLITS;
    return ns;
}

static prima_status launch_attn_kernel(const prima_dims &d, dim3 grid, const AttnArgs &a, hipStream_t st);

// key ranges of a launch: multiples of 16 keys, none empty.  (Rounding the range down to whole tiles per wave and
// giving the keys left over a small range of their own, so that no wave has a tile more than the others, was
// measured: no change at 4096 rows and one token, and 28 -> 40 us at 8 tokens behind 8192 rows, where the ninth range
// of each query group no longer fits the compute units in one round.)
void attn_ranges(const prima_dims &d, int n_total, int T, bool batch, int &keys_per_split, int &nsplit)
{
    const int want = tile_num_splits(d, n_total, T, batch);
    keys_per_split = ((n_total + want - 1) / want + 15) / 16 * 16;
    nsplit = (n_total + keys_per_split - 1) / keys_per_split;
}

size_t attn_records_bytes(const prima_dims &d, int n_total, int T, bool batch)
{
    int kps, ns;
    attn_ranges(d, n_total, T, batch, kps, ns);
    return ns == 1 ? 0 : static_cast<size_t>(T) * d.n_q_heads * ns * (REC_HDR + d.head_dim) * sizeof(float);
}

prima_status launch_attn(const prima_dims &d, const float *q, float *q_rot_out, const float *k_new, const float *v_new,
                            const float *rope_tab, __half *K, __half *V, int kv_cap, int n_past, int T, float *o,
                            void *ws, hipStream_t st, const AttnSeqs *seq)
{
    AttnArgs a = build_attn_args(d, q, q_rot_out, k_new, v_new, rope_tab, K, V, kv_cap, n_past, T, o, ws, seq);
    int n_total = n_past + T;
    if (seq) { // the longest sequence sets the key ranges
        n_total = 0;
        for (int b = 0; b < T; ++b) n_total = seq->n_past[b] + 1 > n_total ? seq->n_past[b] + 1 : n_total;
    }
    attn_ranges(d, n_total, T, seq != nullptr, a.keys_per_split, a.nsplit);
    const dim3 grid(a.nsplit, d.n_kv_heads, tile_query_groups(d, T, seq != nullptr));
    return launch_attn_kernel(d, grid, a, st);
}

// Attention for the tokens of a prompt whose rotated K and V rows are in the caches already and whose queries are
// rotated: n_pieces pieces of PRIMA_MAX_TOK tokens in one launch, each piece over the n_past + 16 piece rows before it
// and, causally, its own; one key range per workgroup (there are Hkv * G workgroups per piece), no scratch.
prima_status launch_attn_prompt(const prima_dims &d, const float *q, __half *K, __half *V, int kv_cap, int n_past, int n_pieces,
                                float *o, hipStream_t st)
{
    if (n_pieces < 1) return PRIMA_OK;
    const int G = d.n_q_heads / d.n_kv_heads;
    const int64_t gz = static_cast<int64_t>(n_pieces) * ((G * PRIMA_MAX_TOK + QGM - 1) / QGM);
    if (gz > 65535 || static_cast<int64_t>(n_past) + static_cast<int64_t>(n_pieces) * PRIMA_MAX_TOK > kv_cap) return PRIMA_E_SHAPE;
    AttnArgs a{};
    a.batch = 2;
    a.q = q; a.K = K; a.V = V; a.o = o;
    a.Hq = d.n_q_heads; a.Hkv = d.n_kv_heads; a.kv_cap = kv_cap; a.n_past = n_past; a.T = PRIMA_MAX_TOK;
    a.nsplit = 1;
    a.keys_per_split = (n_past + n_pieces * PRIMA_MAX_TOK + 15) / 16 * 16;
    return launch_attn_kernel(d, dim3(1, d.n_kv_heads, static_cast<unsigned>(gz)), a, st);
}

static prima_status launch_attn_kernel(const prima_dims &d, dim3 grid, const AttnArgs &a, hipStream_t st)
{
    const dim3 block(ATT_THREADS);
    static std::atomic<bool> attr_set{false}; // set twice by two threads at worst: the attribute call is idempotent
    if (!attr_set) {
        const void *fns[] = {reinterpret_cast<const void *>(attn_decode_kernel<128, 0>), reinterpret_cast<const void *>(attn_decode_kernel<128, 1>),
                             reinterpret_cast<const void *>(attn_decode_kernel<64, 0>), reinterpret_cast<const void *>(attn_decode_kernel<64, 1>)};
        const int sizes[] = {static_cast<int>(sizeof(AttnTileLds<128>)), static_cast<int>(sizeof(AttnTileLds<128>)),
                             static_cast<int>(sizeof(AttnTileLds<64>)), static_cast<int>(sizeof(AttnTileLds<64>))};
        for (int i = 0; i < 4; ++i)
            if (hipFuncSetAttribute(fns[i], hipFuncAttributeMaxDynamicSharedMemorySize, sizes[i]) != hipSuccess) return PRIMA_E_DEVICE;
        attr_set = true;
    }
    if (d.head_dim == 128 && d.rope_mode == 0) hipLaunchKernelGGL((attn_decode_kernel<128, 0>), grid, block, sizeof(AttnTileLds<128>), st, a);
    else if (d.head_dim == 128 && d.rope_mode == 1) hipLaunchKernelGGL((attn_decode_kernel<128, 1>), grid, block, sizeof(AttnTileLds<128>), st, a);
    else if (d.head_dim == 64 && d.rope_mode == 0) hipLaunchKernelGGL((attn_decode_kernel<64, 0>), grid, block, sizeof(AttnTileLds<64>), st, a);
    else if (d.head_dim == 64 && d.rope_mode == 1) hipLaunchKernelGGL((attn_decode_kernel<64, 1>), grid, block, sizeof(AttnTileLds<64>), st, a);
    else return PRIMA_E_SHAPE;
    return last_launch_status();
}

} // namespace prima
