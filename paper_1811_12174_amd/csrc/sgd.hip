// Weight update of the training loop: stochastic gradient descent with (optional) momentum
// and weight decay on a flat fp32 parameter vector, plus the refresh of the bf16 working copy
// the convolution kernels read.  Pure streaming: 12 bytes read and 8 (+2) bytes written per
// parameter, each exactly once, 16-byte accesses when the pointers allow.
#include "common.h"

namespace k3 {

__device__ __forceinline__ void sgd_one(float &w, float &v, float g, float lr, float mu, float wd)
{
    float d = fmaf(wd, w, g);
    v = fmaf(mu, v, d);
    w = fmaf(-lr, v, w);
}

template <bool LP>
__global__ __launch_bounds__(256) void sgd_vec4_kernel(int64_t nq, float4 *__restrict__ w, float4 *__restrict__ v,
                                                       const float4 *__restrict__ g, uint2 *__restrict__ wlp, float lr,
                                                       float mu, float wd)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nq; i += stride) {
        float4 ww = w[i], vv = v[i];
        const float4 gg = g[i];
        sgd_one(ww.x, vv.x, gg.x, lr, mu, wd);
        sgd_one(ww.y, vv.y, gg.y, lr, mu, wd);
        sgd_one(ww.z, vv.z, gg.z, lr, mu, wd);
        sgd_one(ww.w, vv.w, gg.w, lr, mu, wd);
        w[i] = ww;
        v[i] = vv;
        if (LP) wlp[i] = make_uint2(pack2bf(ww.x, ww.y), pack2bf(ww.z, ww.w));
    }
}

// Scalar form for the elements [first, n): misaligned pointers or the ragged tail.
__global__ __launch_bounds__(256) void sgd_scalar_kernel(int64_t first, int64_t n, float *__restrict__ w, float *__restrict__ v,
                                                         const float *__restrict__ g, bf16_t *__restrict__ wlp, float lr,
                                                         float mu, float wd)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        float ww = w[i], vv = v[i];
        sgd_one(ww, vv, g[i], lr, mu, wd);
        w[i] = ww;
        v[i] = vv;
        if (wlp) wlp[i] = f2bf(ww);
    }
}

}  // namespace k3

using namespace k3;

extern "C" int k3_sgd_momentum_step(int64_t n, float *w, float *v, const float *g, float lr, float momentum,
                                    float weight_decay, void *w_bf16, void *stream)
{
    if (n < 0 || (n > 0 && (!w || !v || !g))) return K3_E_BADARG;
    if (!(lr == lr) || !(momentum == momentum) || !(weight_decay == weight_decay)) return K3_E_BADARG;
    if (n == 0) return K3_OK;
    hipStream_t st = (hipStream_t)stream;
    const uintptr_t al = (uintptr_t)w | (uintptr_t)v | (uintptr_t)g;
    const bool vec = (al % 16 == 0) && ((uintptr_t)w_bf16 % 8 == 0);
    const int64_t nq = vec ? n / 4 : 0;
    if (nq > 0) {
        const int64_t want = (nq + 255) / 256;
        const int grid = (int)(want < 4096 ? want : 4096);
        if (w_bf16)
            hipLaunchKernelGGL(sgd_vec4_kernel<true>, dim3(grid), dim3(256), 0, st, nq, (float4 *)w, (float4 *)v,
                               (const float4 *)g, (uint2 *)w_bf16, lr, momentum, weight_decay);
        else
            hipLaunchKernelGGL(sgd_vec4_kernel<false>, dim3(grid), dim3(256), 0, st, nq, (float4 *)w, (float4 *)v,
                               (const float4 *)g, (uint2 *)nullptr, lr, momentum, weight_decay);
        K3_LAUNCH_CHECK();
    }
    const int64_t first = nq * 4;
    if (first < n) {
        const int64_t want = (n - first + 255) / 256;
        const int grid = (int)(want < 4096 ? want : 4096);
        hipLaunchKernelGGL(sgd_scalar_kernel, dim3(grid), dim3(256), 0, st, first, n, w, v, g, (bf16_t *)w_bf16, lr, momentum,
                           weight_decay);
        K3_LAUNCH_CHECK();
    }
    return K3_OK;
}
