// Shared host/device helpers for the k3 kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "k3.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef unsigned short bf16_t;  // raw bf16 bit pattern in memory

namespace k3 {

void set_hip_error(hipError_t e);

#define K3_HIP(expr)                                   \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) {                       \
            k3::set_hip_error(e__);                    \
            return K3_E_HIP;                           \
        }                                              \
    } while (0)

#define K3_LAUNCH_CHECK() K3_HIP(hipGetLastError())

static inline bool desc_ok(const k3_tensor *t)
{
    return t && t->n > 0 && t->d > 0 && t->h > 0 && t->w > 0 && t->c > 0 &&
           (t->dtype == K3_BF16 || t->dtype == K3_F32) && t->reserved == 0;
}
static inline bool same_space(const k3_tensor *a, const k3_tensor *b)
{
    return a->n == b->n && a->d == b->d && a->h == b->h && a->w == b->w;
}
static inline int64_t voxels(const k3_tensor *t) { return t->n * t->d * t->h * t->w; }
static inline size_t esize(int dtype) { return dtype == K3_BF16 ? 2 : 4; }

// bf16 <-> fp32 (round to nearest even; inputs are finite in this library's use)
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// fp32 -> bf16, round to nearest even, through the hardware conversion (v_cvt_pk_bf16_f32)
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi)
{
    f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ bf16_t f2bf(float f) { return (bf16_t)(pack2bf(f, 0.f) & 0xffffu); }

// Asynchronous copy global -> LDS, 16 bytes per lane (global_load_lds_dwordx4): lane l of the
// wave writes the 16 bytes at its own global address gptr to LDS byte address lds_base + 16*l
// (lds_base is wave-uniform).  Completion is tracked by vmcnt; the compiler does not see the
// LDS write, so the caller waits (s_waitcnt vmcnt) and synchronises before reading the data.
__device__ __forceinline__ void dma16(unsigned lds_base, const void *gptr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}

template <typename T> struct elem;
template <> struct elem<float> {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
};
template <> struct elem<bf16_t> {
    static __device__ __forceinline__ float ld(const bf16_t *p) { return bf2f(*p); }
    static __device__ __forceinline__ void st(bf16_t *p, float v) { *p = f2bf(v); }
};

}  // namespace k3
