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

// One-bit-per-element ReLU masks: word layout is bit i <-> element i of 16 consecutive channels.
// The 16 stored bf16 values arrive as 8 packed pairs d[0..7] (element 2k in the low half of d[k]).
typedef __attribute__((ext_vector_type(2))) short s16x2_t;
typedef __attribute__((ext_vector_type(2))) unsigned short u16x2_t;
// bit 0: the low bf16 half is > 0, bit 16: the high half is (as signed 16-bit integers the positive
// bf16 values are exactly the positive integers; -0.0 and negative values are not)
__device__ __forceinline__ uint32_t bf16_pair_positive(uint32_t d)
{
    s16x2_t h = __builtin_bit_cast(s16x2_t, d);
    const s16x2_t one = {1, 1}, zero = {0, 0};
    h = __builtin_elementwise_max(__builtin_elementwise_min(h, one), zero);
    return __builtin_bit_cast(uint32_t, h);
}
// the same with the two packed instructions pinned (left to itself the compiler expands the
// min/max pair into compares, selects and a byte permute where it knows the halves are >= 0)
__device__ __forceinline__ uint32_t pair_positive_pk(uint32_t d)
{
    uint32_t t;
    asm("v_pk_min_i16 %0, %1, %2" : "=v"(t) : "v"(d), "v"(0x00010001u));
    asm("v_pk_max_i16 %0, %1, 0" : "=v"(t) : "v"(t));
    return t;
}
__device__ __forceinline__ unsigned relu_bits16(const uint32_t (&d)[8])
{
    // even elements gather in bits 0..7, odd ones in bits 16..23, then both bytes are spread to
    // every other bit at once and interleaved
    unsigned z = bf16_pair_positive(d[0]);
#pragma unroll
    for (int k = 1; k < 8; ++k) z |= bf16_pair_positive(d[k]) << k;
    z = (z | (z << 4)) & 0x0F0F0F0Fu;
    z = (z | (z << 2)) & 0x33333333u;
    z = (z | (z << 1)) & 0x55555555u;
    return (z | (z >> 15)) & 0xffffu;
}
// zeroes the bf16 halves of d[0..7] whose bit in m is clear
__device__ __forceinline__ void apply_bits16(uint32_t (&d)[8], unsigned m)
{
    // inverse of the interleave: even bits to 0..7, odd bits to 16..23
    unsigned z = (m | (m << 15)) & 0x55555555u;
    z = (z | (z >> 1)) & 0x33333333u;
    z = (z | (z >> 2)) & 0x0F0F0F0Fu;
    z = (z | (z >> 4)) & 0x00FF00FFu;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const u16x2_t keep = __builtin_bit_cast(u16x2_t, (z >> k) & 0x00010001u);   // 0 or 1 per half
        d[k] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2_t, d[k]) * keep);
    }
}

// Asynchronous copy global -> LDS, 16 bytes per lane (global_load_lds_dwordx4): lane l of the
// wave writes the 16 bytes at its own global address gptr to LDS byte address lds_base + 16*l
// (lds_base is wave-uniform).  Completion is tracked by vmcnt; the compiler does not see the
// LDS write, so the caller waits (s_waitcnt vmcnt) and synchronises before reading the data.
__device__ __forceinline__ void dma16(unsigned lds_base, const void *gptr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}

// Asynchronous copy through a buffer descriptor: lane l writes 16 bytes to LDS byte address
// lds_base + 16 * l from descriptor base + soff + voff.  A lane whose voff lies beyond the
// descriptor's range (0xffffffff is used for "nothing to copy") writes zeros: out-of-volume halo
// items and padding need neither a branch nor a zero block.  Tracked by vmcnt like dma16.
__device__ __forceinline__ void dma16_buf(unsigned lds_base, __amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 ::"s"(__builtin_amdgcn_readfirstlane(lds_base)), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
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
