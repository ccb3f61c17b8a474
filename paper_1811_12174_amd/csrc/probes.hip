// Measurement aids: the two machine rates the benchmark reports its kernels against, measured on
// the box the benchmark runs on.  Not part of the training path.
//
//  * k3_probe_mfma_bf16: a register-resident loop of v_mfma_f32_32x32x16_bf16 on four independent
//    accumulators per wave, four waves per workgroup, no memory traffic inside the loop: the rate
//    the matrix cores sustain at the clock the chip holds under that load.
//  * k3_probe_copy: a grid-stride 16-byte-per-lane device copy: the HBM rate a plain streaming
//    kernel reaches (bytes read + bytes written).
#include "common.h"

namespace k3 {

__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(float *__restrict__ sink, int64_t iters)
{
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)((threadIdx.x + i) % 3);
        b[i] = (__bf16)(float)((threadIdx.x + 2 * i) % 5);
    }
    f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.f;
    for (int64_t i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += (c0[i] + c1[i]) + (c2[i] + c3[i]);
    sink[(int64_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

}  // namespace k3

using namespace k3;

extern "C" {

int k3_probe_mfma_bf16(int64_t iters, int blocks, float *sink, double *flops, void *stream)
{
    if (iters <= 0 || blocks <= 0 || blocks > (1 << 20) || !sink) return K3_E_BADARG;
    probe_mfma_bf16_kernel<<<dim3((unsigned)blocks), 256, 0, (hipStream_t)stream>>>(sink, iters);
    K3_LAUNCH_CHECK();
    // 4 waves x 4 MFMAs per iteration, 2 * 32 * 32 * 16 FLOP each
    if (flops) *flops = (double)blocks * 4.0 * 4.0 * (double)iters * 2.0 * 32.0 * 32.0 * 16.0;
    return K3_OK;
}

int k3_probe_copy(const void *src, void *dst, size_t bytes, int blocks, void *stream)
{
    if (!src || !dst || bytes == 0 || bytes % 16 != 0 || blocks <= 0 || blocks > (1 << 20)) return K3_E_BADARG;
    if (((uintptr_t)src | (uintptr_t)dst) & 15) return K3_E_BADARG;
    probe_copy_kernel<<<dim3((unsigned)blocks), 256, 0, (hipStream_t)stream>>>((const uint4 *)src, (uint4 *)dst,
                                                                              (int64_t)(bytes / 16));
    K3_LAUNCH_CHECK();
    return K3_OK;
}

}  // extern "C"
