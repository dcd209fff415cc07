// RoPE and the fp16 KV append of a Llama/Qwen-style decoder layer (RMSNorm and SwiGLU are fused
// into the mat-vec that consumes them).  The paper does not write these formulas (it names the
// model families); the KV append volume is its 2(h_k e_k + h_v e_v) bytes per layer per token
// (arXiv 2504.08791, App. A.3).
#include "common.h"

namespace prima {

// tab[t][i] = (cos, sin) of (n_past + t) * theta^(-2i/D), evaluated in fp64: at positions of
// several thousand an fp32 angle would already be off by ~1e-4 rad.
__global__ void rope_table_kernel(float2 *tab, int T, int half, int n_past, double theta)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= T * half) return;
    const int t = idx / half, i = idx - t * half;
    const double ang = static_cast<double>(n_past + t) * pow(theta, -static_cast<double>(i) / static_cast<double>(half));
    tab[idx] = make_float2(static_cast<float>(cos(ang)), static_cast<float>(sin(ang)));
}

prima_status launch_rope_table(float *tab, int T, int D, int n_past, float theta, hipStream_t st)
{
    const int n = T * (D / 2);
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 127) / 128), dim3(128), 0, st,
                       reinterpret_cast<float2 *>(tab), T, D / 2, n_past, static_cast<double>(theta));
    return last_launch_status();
}

// grid (T, Hq + 2*Hkv), D/2 threads: q heads rotated in place; k heads rotated and stored as
// fp16; v heads stored as fp16.  fp32 -> fp16 rounds to nearest even.
__global__ void rope_kv_kernel(float *q, const float *k, const float *v, const float2 *tab,
                               __half *Kc, __half *Vc, int Hq, int Hkv, int D, int kv_cap, int n_past, int mode)
{
    const int t = blockIdx.x, hh = blockIdx.y, i = threadIdx.x, half = D / 2;
    const int ia = mode ? 2 * i : i, ib = mode ? 2 * i + 1 : i + half;
    if (hh < Hq + Hkv) {
        const float2 cs = tab[t * half + i];
        if (hh < Hq) {
            float *p = q + (static_cast<int64_t>(t) * Hq + hh) * D;
            const float a = p[ia], b = p[ib];
            p[ia] = a * cs.x - b * cs.y;
            p[ib] = a * cs.y + b * cs.x;
        } else {
            const int h = hh - Hq;
            const float *p = k + (static_cast<int64_t>(t) * Hkv + h) * D;
            __half *dst = Kc + (static_cast<int64_t>(h) * kv_cap + n_past + t) * D;
            const float a = p[ia], b = p[ib];
            dst[ia] = __float2half_rn(a * cs.x - b * cs.y);
            dst[ib] = __float2half_rn(a * cs.y + b * cs.x);
        }
    } else {
        const int h = hh - Hq - Hkv;
        const float *p = v + (static_cast<int64_t>(t) * Hkv + h) * D;
        __half *dst = Vc + (static_cast<int64_t>(h) * kv_cap + n_past + t) * D;
        dst[2 * i] = __float2half_rn(p[2 * i]);
        dst[2 * i + 1] = __float2half_rn(p[2 * i + 1]);
    }
}

prima_status launch_rope_kv_append(const prima_dims &d, float *q, const float *k, const float *v,
                                   const float *rope_tab, __half *k_cache, __half *v_cache,
                                   int kv_cap, int n_past, int T, hipStream_t st)
{
    hipLaunchKernelGGL(rope_kv_kernel, dim3(T, d.n_q_heads + 2 * d.n_kv_heads), dim3(d.head_dim / 2), 0, st,
                       q, k, v, reinterpret_cast<const float2 *>(rope_tab), k_cache, v_cache,
                       d.n_q_heads, d.n_kv_heads, d.head_dim, kv_cap, n_past, d.rope_mode);
    return last_launch_status();
}

} // namespace prima
