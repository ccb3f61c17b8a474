// Segmentation metric: the 3x3 confusion matrix of predicted class against label, and the
// per-class Dice coefficient that follows from it.  Integer counting only (64-bit integer
// atomics, whose result does not depend on the order); the three quotients are taken in fp64
// and stored as fp32.  Streaming: two bytes read per voxel.
#include "common.h"

namespace k3 {

__global__ void confusion_zero_kernel(unsigned long long *counts)
{
    if (threadIdx.x < 9) counts[threadIdx.x] = 0ull;
}

__device__ __forceinline__ void tally(unsigned p, unsigned t, unsigned &lo, unsigned &hi)
{
    // eight 8-bit counters packed in two words: (t, p) -> slot t * 3 + p; a thread adds at most 16 before it unpacks
    p = p > 2u ? 2u : p;
    t = t > 2u ? 2u : t;
    const unsigned slot = t * 3u + p;
    if (slot < 4u) lo += 1u << (slot * 8u);
    else if (slot < 8u) hi += 1u << ((slot - 4u) * 8u);
    // slot 8 is derived from the total by the caller
}

__global__ __launch_bounds__(256) void confusion_kernel(const uint8_t *__restrict__ cls, const uint8_t *__restrict__ lab,
                                                       int64_t V, unsigned long long *__restrict__ counts)
{
    __shared__ unsigned long long red[9];
    if (threadIdx.x < 9) red[threadIdx.x] = 0ull;
    __syncthreads();
    unsigned long long c[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) c[i] = 0ull;
    const int64_t stride = (int64_t)gridDim.x * 256 * 16;
    const bool aligned = (((uintptr_t)cls | (uintptr_t)lab) & 15u) == 0;
    for (int64_t v0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 16; v0 < V; v0 += stride) {
        unsigned char pb[16], tb[16];
        const int n = (V - v0) < 16 ? (int)(V - v0) : 16;
        if (n == 16 && aligned) {
            *reinterpret_cast<uint4 *>(pb) = *reinterpret_cast<const uint4 *>(cls + v0);
            *reinterpret_cast<uint4 *>(tb) = *reinterpret_cast<const uint4 *>(lab + v0);
        } else {
            for (int i = 0; i < 16; ++i) {
                pb[i] = i < n ? cls[v0 + i] : 0;
                tb[i] = i < n ? lab[v0 + i] : 0;
            }
        }
        unsigned lo = 0u, hi = 0u;
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (i < n) tally(pb[i], tb[i], lo, hi);
        unsigned seen = 0u;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const unsigned a = (lo >> (8 * s)) & 255u, b = (hi >> (8 * s)) & 255u;
            c[s] += a; c[4 + s] += b;
            seen += a + b;
        }
        c[8] += (unsigned)n - seen;
    }
#pragma unroll
    for (int i = 0; i < 9; ++i) {
        unsigned long long v = c[i];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m);
        if ((threadIdx.x & 63) == 0 && v) atomicAdd(&red[i], v);
    }
    __syncthreads();
    if (threadIdx.x < 9 && red[threadIdx.x]) atomicAdd(&counts[threadIdx.x], red[threadIdx.x]);
}

__global__ void dice_kernel(const unsigned long long *__restrict__ counts, float *__restrict__ dice)
{
    const int k = threadIdx.x;
    if (k >= 3) return;
    unsigned long long row = 0ull, col = 0ull;
    for (int j = 0; j < 3; ++j) {
        row += counts[k * 3 + j];   // voxels labelled k
        col += counts[j * 3 + k];   // voxels classified k
    }
    const unsigned long long den = row + col;
    dice[k] = den == 0ull ? 1.f : (float)(2.0 * (double)counts[k * 3 + k] / (double)den);
}

}  // namespace k3

using namespace k3;

extern "C" int k3_dice_coefficients(const uint8_t *classes, const uint8_t *labels, int64_t voxels, uint64_t *counts,
                                    float *dice, void *stream)
{
    if (voxels < 0 || !counts || (voxels > 0 && (!classes || !labels))) return K3_E_BADARG;
    hipStream_t st = (hipStream_t)stream;
    unsigned long long *c = reinterpret_cast<unsigned long long *>(counts);
    hipLaunchKernelGGL(confusion_zero_kernel, dim3(1), dim3(64), 0, st, c);
    K3_LAUNCH_CHECK();
    if (voxels > 0) {
        const int64_t want = (voxels + 256 * 16 - 1) / (256 * 16);
        const int grid = (int)(want < 2048 ? want : 2048);
        hipLaunchKernelGGL(confusion_kernel, dim3(grid), dim3(256), 0, st, classes, labels, voxels, c);
        K3_LAUNCH_CHECK();
    }
    if (dice) {
        hipLaunchKernelGGL(dice_kernel, dim3(1), dim3(64), 0, st, (const unsigned long long *)c, dice);
        K3_LAUNCH_CHECK();
    }
    return K3_OK;
}
