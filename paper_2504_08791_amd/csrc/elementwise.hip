// RoPE angle table of a window step.  (RMSNorm and SwiGLU are fused into the mat-vec that consumes
// them; the rotation itself and the fp16 KV append are fused into the attention kernel.)
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

} // namespace prima
