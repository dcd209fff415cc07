// A window of decoder layers in one launch (one token per step): the five per-layer kernels of window.hip
// run back to back inside one persistent grid of one 512-thread workgroup per compute unit, separated by
// grid barriers instead of kernel boundaries (arXiv 2504.08791, Sec. 3.1: a device advances its window of
// consecutive layers; App. A.3: the weight bytes of those layers are what the step costs).
//
// What this buys: between two kernels the memory system idles for the whole tail of the first (workgroups
// finish a few percent apart) and the whole prologue of the second (activation fetch, statistics,
// quantisation: ~5 us per mat-vec).  Here a workgroup that has finished its share requests the first ring
// stages of the *next* projection (weights do not depend on the activations still being written), or the
// first K/V tile of the attention, before it waits at the barrier, so the weight stream continues across
// the boundary.
//
// Rules of the launch:
//  * all workgroups must be resident together: the kernel is launched cooperatively with exactly as many
//    workgroups as every phase's plan uses; the host refuses shapes whose plans differ;
//  * everything one phase writes and a later one reads (q, k, v, o, h, the SwiGLU output, the hidden state,
//    partial sums and attention records) is written with device-scope stores and read with device-scope
//    loads: the L2 caches of the XCDs are not coherent with each other inside a launch;
//  * a barrier is an arrival counter: a workgroup adds one after all its stores have completed
//    (s_waitcnt vmcnt(0) + workgroup barrier), thread 0 of each workgroup polls until the count reaches
//    (barriers so far) x (workgroups).  The poll is bounded: after SPIN_LIMIT polls it raises an error flag
//    in the workspace and every later wait returns at once, so the grid always drains; the host reports the
//    flag (prima_window_check).
#include "gemv_common.h"
#include "attn_common.h"

namespace prima {

constexpr int FUSED_MAX_LAYERS = 24; // per launch: the layer table travels in the kernel arguments
constexpr int SPIN_LIMIT = 1 << 20;  // polls of ~1 us each: far beyond any phase, short of a hang

struct FusedArgs {
    PGemvArgs g[4];  // Q/K/V, output, gate/up, down projection: plans, shapes and the buffers that do not change
                     // from layer to layer; weights, gains and the hidden-state pointers are set per layer
    AttnArgs at;     // likewise; the caches are set per layer
    prima_layer layers[FUSED_MAX_LAYERS];
    const float *x_in; // hidden state entering the first layer of the window (global layer 0)
    float *x_out;      // hidden state leaving the last layer of the window
    float *xb0, *xb1;  // ping-pong buffers between layers: global layer i writes xb[i & 1]
    unsigned *bar;     // arrival counter of the grid barriers, zero at launch
    int *err;          // raised when a barrier timed out
    int L;             // layers in this launch
    int first_layer;   // global index of its first layer
    int L_total;       // layers of the whole window
    int n_wg;          // workgroups of the launch
    int attn_wgs;      // workgroups the attention uses: key ranges x KV heads x query groups
    int nqg;           // query groups per KV head
};

struct GridSync {
    unsigned *ctr;
    int *err;
    unsigned target; // arrivals that complete the barrier this phase depends on (0: none)
    bool pending;

    // returns once every workgroup has arrived at the previous barrier; called by all threads of the workgroup
    __device__ __forceinline__ void wait()
    {
        if (!pending) return;
        pending = false;
        if (target != 0u) {
            if (threadIdx.x == 0) {
                int polls = 0;
                while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                    if (__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
                    if (++polls > SPIN_LIMIT) {
                        __hip_atomic_store(err, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        break;
                    }
                    __builtin_amdgcn_s_sleep(4);
                }
            }
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        }
    }
};

// all of this workgroup's device-scope stores have completed before its arrival is counted
__device__ __forceinline__ void grid_arrive(unsigned *ctr)
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (threadIdx.x == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// The arguments are read where they lie, in the kernel-argument segment (constant address space, scalar
// loads, indexable by layer and phase): taking references into the by-value parameter instead makes the
// compiler copy all of it into private memory.
typedef const __attribute__((address_space(4))) FusedArgs ConstFusedArgs;
typedef const __attribute__((address_space(4))) PGemvArgs ConstPGemvArgs;
typedef const __attribute__((address_space(4))) AttnArgs ConstAttnArgs;
typedef const __attribute__((address_space(4))) prima_layer ConstLayer;

template <int D, int MODE>
__global__ void __launch_bounds__(GEMV_THREADS) window_fused_kernel(FusedArgs fa_by_value)
{
    ConstFusedArgs &fa = *(ConstFusedArgs *)__builtin_amdgcn_kernarg_segment_ptr();
    extern __shared__ __align__(16) uint8_t smem[];
    static_assert(ATT_THREADS == GEMV_THREADS, "both bodies run on the same workgroup");
    constexpr int TT = 1;
    constexpr bool COH = true;
    const int wg_index = blockIdx.x;
    unsigned *const bar = as_global(fa.bar);
    GridSync sync{bar, as_global(fa.err), 0u, false};
    unsigned done = 0; // barriers this workgroup has arrived at

    for (int l = 0; l < fa.L; ++l) {
        ConstLayer &Ly = fa.layers[l];
        const int gl = fa.first_layer + l; // global layer index
        const float *cur = as_global(gl == 0 ? fa.x_in : (((gl - 1) & 1) ? fa.xb1 : fa.xb0));
        float *dst = as_global(gl == fa.L_total - 1 ? fa.x_out : ((gl & 1) ? fa.xb1 : fa.xb0));
        for (int ph = 0; ph < 5; ++ph) {
            sync.target = done * static_cast<unsigned>(fa.n_wg);
            sync.pending = true;
            if (ph == 1) {
                // ---- attention: workgroup index -> (key range, KV head, query group) ----
                if (wg_index < fa.attn_wgs) {
                    ConstAttnArgs &a = fa.at;
                    __half *const arg_K = as_global(static_cast<__half *>(Ly.k_cache)), *const arg_V = as_global(static_cast<__half *>(Ly.v_cache));
                    const int split = wg_index % a.nsplit;
                    const int kvh = (wg_index / a.nsplit) % a.Hkv;
                    const int qgrp = wg_index / (a.nsplit * a.Hkv);
                    const int nqg = fa.nqg;
                    constexpr int tok0 = 0; // one sequence
                    const int arg_T = a.T, arg_n_past = a.n_past;
#include "attn_body.inc"
                }
            } else {
                // ---- a projection: the plan and the fixed buffers from the launch arguments, the rest per layer ----
                const int gi = ph == 0 ? 0 : ph - 1;
                ConstPGemvArgs &a = fa.g[gi];
                // phase:                                  Q/K/V        output      gate/up       down
                const float *const arg_x = as_global(gi == 0 ? cur : a.x);
                const float *const arg_gain = as_global(gi == 0 ? Ly.g_attn : (gi == 2 ? Ly.g_ffn : nullptr));
                const uint8_t *const arg_W0 = as_global(static_cast<const uint8_t *>(gi == 0 ? Ly.wq : (gi == 1 ? Ly.wo : (gi == 2 ? Ly.wgate : Ly.wdown))));
                const uint8_t *const arg_W1 = as_global(static_cast<const uint8_t *>(gi == 0 ? Ly.wk : Ly.wup));
                const uint8_t *const arg_W2 = as_global(static_cast<const uint8_t *>(Ly.wv));
                float *const arg_y0 = as_global(gi == 3 ? dst : a.seg[0].y), *const arg_y1 = as_global(a.seg[1].y), *const arg_y2 = as_global(a.seg[2].y);
                const float *const arg_r0 = as_global(gi == 1 ? cur : a.seg[0].resid), *const arg_r1 = nullptr, *const arg_r2 = nullptr;
#include "gemv_body.inc"
            }
            sync.wait(); // a workgroup without work in this phase still has to see the previous one complete
            grid_arrive(bar);
            ++done;
        }
    }
}

// ------------------------------------------------------------------------------------------
size_t fused_sync_bytes() { return 256; } // arrival counter at offset 0, error flag at offset 128

template <int D, int MODE>
static hipError_t launch_fused_inst(const FusedArgs &fa, size_t lds_bytes, hipStream_t st)
{
    static bool attr_set = false;
    const void *fn = reinterpret_cast<const void *>(window_fused_kernel<D, MODE>);
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(LDS_BUDGET));
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    void *params[] = {const_cast<FusedArgs *>(&fa)};
    return hipLaunchCooperativeKernel(fn, dim3(fa.n_wg), dim3(GEMV_THREADS), params, static_cast<unsigned>(lds_bytes), st);
}

// Runs the whole window (one token) as fused launches of up to FUSED_MAX_LAYERS layers.  Returns PRIMA_E_SHAPE
// without launching anything when the shapes do not qualify (the caller then runs the kernels one by one).
// ga[4]: the projections' arguments as for launch_gemv_mfma (weights / gains / hidden-state pointers of any
// layer: they are replaced per layer); the attention's arguments as for launch_attn with the fused append;
// sync: fused_sync_bytes() of zeroed scratch.
prima_status launch_fused_window(const prima_dims &d, const prima_layer *layers, int L, const GemvArgs ga[4],
                                 void *gemv_ws, size_t gemv_ws_bytes, size_t arrivals_region,
                                 const float *q, const float *k_new, const float *v_new, const float *rope_tab,
                                 int kv_cap, int n_past, float *o, void *attn_ws,
                                 const float *x_in, float *x_out, float *xb0, float *xb1, void *sync, hipStream_t st)
{
    if (L < 1) return PRIMA_E_RANGE;
    const AttnArgs at = build_attn_args(d, q, nullptr, k_new, v_new, rope_tab, static_cast<__half *>(layers[0].k_cache),
                                        static_cast<__half *>(layers[0].v_cache), kv_cap, n_past, 1, o, attn_ws);
    if (at.T != 1) return PRIMA_E_SHAPE;
    static_assert(sizeof(FusedArgs) <= 4096, "kernel arguments");
    const int cus = device_cu_count();
    FusedArgs fa{};
    size_t lds = d.head_dim == 128 ? sizeof(AttnLds<128>) : sizeof(AttnLds<64>);
    for (int i = 0; i < 4; ++i) {
        PPlan p;
        const prima_status s = build_pass(ga[i], 0, 1, gemv_ws, gemv_ws_bytes, arrivals_region, fa.g[i], p);
        if (s != PRIMA_OK) return s;
        // every phase on the same grid, every workgroup with at least one tile group, and the activation path
        // that reads with device scope (at most two groups of 8 activations per thread, the whole row for RMSNorm)
        const int gran = ga[i].epi == EPI_SWIGLU ? 2 : 1;
        if (p.n_wg != cus || p.n_tiles / gran < (cus + p.n_slabs - 1) / p.n_slabs) return PRIMA_E_SHAPE;
        if (p.slab_blocks > 32 || (ga[i].xmode == X_RMSNORM && p.n_slabs != 1)) return PRIMA_E_SHAPE;
        lds = p.lds_bytes > lds ? p.lds_bytes : lds;
    }
    fa.at = at;
    fa.nqg = query_groups(d, 1);
    fa.attn_wgs = at.nsplit * d.n_kv_heads * fa.nqg;
    if (fa.attn_wgs > cus) return PRIMA_E_SHAPE;
    fa.x_in = x_in; fa.x_out = x_out; fa.xb0 = xb0; fa.xb1 = xb1;
    fa.bar = static_cast<unsigned *>(sync);
    fa.err = reinterpret_cast<int *>(static_cast<char *>(sync) + 128);
    fa.n_wg = cus;
    fa.L_total = L;
    for (int l0 = 0; l0 < L; l0 += FUSED_MAX_LAYERS) {
        fa.first_layer = l0;
        fa.L = L - l0 < FUSED_MAX_LAYERS ? L - l0 : FUSED_MAX_LAYERS;
        for (int i = 0; i < fa.L; ++i) fa.layers[i] = layers[l0 + i];
        if (l0 > 0) { // a fresh count for every launch (the error flag stays)
            const prima_status zs = launch_zero_arrivals(sync, 128, st);
            if (zs != PRIMA_OK) return zs;
        }
        hipError_t e;
        if (d.head_dim == 128 && d.rope_mode == 0) e = launch_fused_inst<128, 0>(fa, lds, st);
        else if (d.head_dim == 128 && d.rope_mode == 1) e = launch_fused_inst<128, 1>(fa, lds, st);
        else if (d.head_dim == 64 && d.rope_mode == 0) e = launch_fused_inst<64, 0>(fa, lds, st);
        else if (d.head_dim == 64 && d.rope_mode == 1) e = launch_fused_inst<64, 1>(fa, lds, st);
        else return PRIMA_E_SHAPE;
        if (e != hipSuccess) {
            (void)hipGetLastError();
            return l0 == 0 ? PRIMA_E_SHAPE : PRIMA_E_DEVICE; // nothing ran yet: the caller may take the other path
        }
    }
    return PRIMA_OK;
}

} // namespace prima
