// Small per-token operators of a Llama/Qwen-style decoder layer: RMSNorm, RoPE (+ fp16 KV
// append), SwiGLU.  The paper does not write their formulas (it names the model families); the
// KV append volume is its 2(h_k e_k + h_v e_v) bytes per layer per token (App. A.3).
#include "common.h"

namespace prima {

__device__ __forceinline__ float block_sum(float v, float *red /* [16] */)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    const int w = threadIdx.x >> 6, nw = blockDim.x >> 6;
    if ((threadIdx.x & 63) == 0) red[w] = v;
    __syncthreads();
    float s = 0.f;
    for (int i = 0; i < nw; ++i) s += red[i]; // fixed order: deterministic
    __syncthreads();
    return s;
}

// out = x * g / sqrt(mean(x^2) + eps), one block per token
__global__ void __launch_bounds__(1024) rmsnorm_kernel(const float *__restrict__ x, const float *__restrict__ g,
                                                      float *__restrict__ out, int n, float eps)
{
    __shared__ float red[16];
    const float *xt = x + static_cast<int64_t>(blockIdx.x) * n;
    float *ot = out + static_cast<int64_t>(blockIdx.x) * n;
    float ss = 0.f;
    for (int i = threadIdx.x * 4; i < n; i += blockDim.x * 4) {
        const float4 v = *reinterpret_cast<const float4 *>(xt + i);
        ss += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
    }
    ss = block_sum(ss, red);
    const float inv = 1.0f / sqrtf(ss / static_cast<float>(n) + eps);
    for (int i = threadIdx.x * 4; i < n; i += blockDim.x * 4) {
        const float4 v = *reinterpret_cast<const float4 *>(xt + i);
        const float4 gg = *reinterpret_cast<const float4 *>(g + i);
        float4 r;
        r.x = v.x * inv * gg.x; r.y = v.y * inv * gg.y; r.z = v.z * inv * gg.z; r.w = v.w * inv * gg.w;
        *reinterpret_cast<float4 *>(ot + i) = r;
    }
}

prima_status launch_rmsnorm(const float *x, const float *g, float *out, int T, int n, float eps, hipStream_t st)
{
    hipLaunchKernelGGL(rmsnorm_kernel, dim3(T), dim3(1024), 0, st, x, g, out, n, eps);
    return last_launch_status();
}

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

// a = silu(g) * u, silu(z) = z / (1 + exp(-z))
__global__ void __launch_bounds__(256) swiglu_kernel(const float *__restrict__ g, const float *__restrict__ u,
                                                    float *__restrict__ a, int64_t n)
{
    const int64_t i = (static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x) * 4;
    if (i >= n) return;
    const float4 gv = *reinterpret_cast<const float4 *>(g + i);
    const float4 uv = *reinterpret_cast<const float4 *>(u + i);
    float4 r;
    r.x = gv.x / (1.0f + expf(-gv.x)) * uv.x;
    r.y = gv.y / (1.0f + expf(-gv.y)) * uv.y;
    r.z = gv.z / (1.0f + expf(-gv.z)) * uv.z;
    r.w = gv.w / (1.0f + expf(-gv.w)) * uv.w;
    *reinterpret_cast<float4 *>(a + i) = r;
}

prima_status launch_swiglu(const float *g, const float *u, float *a, int64_t n, hipStream_t st)
{
    const int64_t grid = (n / 4 + 255) / 256;
    hipLaunchKernelGGL(swiglu_kernel, dim3(static_cast<unsigned>(grid)), dim3(256), 0, st, g, u, a, n);
    return last_launch_status();
}

} // namespace prima
