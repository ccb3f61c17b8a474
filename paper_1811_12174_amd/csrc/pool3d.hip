// 2x2x2 stride-2 max pooling, forward and backward, for gfx950.  Pure streaming kernels:
// one thread handles VEC consecutive channels of one output window (16-byte loads when
// the channel count allows), so every byte of x / y / dx is touched exactly once.
#include "common.h"

namespace k3 {

template <typename T, int VEC> struct vec_io;
template <> struct vec_io<bf16_t, 8> {
    static __device__ __forceinline__ void ld(const bf16_t *p, float *v)
    {
        uint4 u = *reinterpret_cast<const uint4 *>(p);
        uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(w[i] << 16);
            v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void st(bf16_t *p, const float *v)
    {
        uint4 u = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
        *reinterpret_cast<uint4 *>(p) = u;
    }
};
template <> struct vec_io<float, 4> {
    static __device__ __forceinline__ void ld(const float *p, float *v)
    {
        float4 u = *reinterpret_cast<const float4 *>(p);
        v[0] = u.x; v[1] = u.y; v[2] = u.z; v[3] = u.w;
    }
    static __device__ __forceinline__ void st(float *p, const float *v)
    {
        *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <typename T> struct vec_io<T, 1> {
    static __device__ __forceinline__ void ld(const T *p, float *v) { v[0] = elem<T>::ld(p); }
    static __device__ __forceinline__ void st(T *p, const float *v) { elem<T>::st(p, v[0]); }
};

// D, H, W are the OUTPUT sizes; the input is (2D, 2H, 2W).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void pool_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t total,
                                                      int D, int H, int W, int C)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int cv = C / VEC;
    int c = (int)(gid % cv) * VEC;
    int64_t o = gid / cv;
    int w = (int)(o % W);
    int h = (int)((o / W) % H);
    int d = (int)((o / ((int64_t)W * H)) % D);
    int64_t n = o / ((int64_t)W * H * D);
    float m[VEC], v[VEC];
    bool have = false;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                int64_t u = ((n * 2 * D + 2 * d + i) * 2 * H + 2 * h + j) * (2 * (int64_t)W) + 2 * w + k;
                vec_io<T, VEC>::ld(x + u * C + c, v);
#pragma unroll
                for (int e = 0; e < VEC; ++e) m[e] = (!have || v[e] > m[e]) ? v[e] : m[e];
                have = true;
            }
    vec_io<T, VEC>::st(y + o * C + c, m);
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void pool_bwd_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                                      const T *__restrict__ add, int relu_mask, T *__restrict__ dx,
                                                      int64_t total, int D, int H, int W, int C)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int cv = C / VEC;
    int c = (int)(gid % cv) * VEC;
    int64_t o = gid / cv;
    int w = (int)(o % W);
    int h = (int)((o / W) % H);
    int d = (int)((o / ((int64_t)W * H)) % D);
    int64_t n = o / ((int64_t)W * H * D);
    float m[VEC], v[VEC], g[VEC], a[VEC], r[VEC];
    int arg[VEC];
    unsigned pos[VEC];   // bit p: window element p is > 0 (the ReLU mask of x)
#pragma unroll
    for (int e = 0; e < VEC; ++e) pos[e] = 0;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int64_t u = ((n * 2 * D + 2 * d + (p >> 2)) * 2 * H + 2 * h + ((p >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (p & 1);
        vec_io<T, VEC>::ld(x + u * C + c, v);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (p == 0 || v[e] > m[e]) { m[e] = v[e]; arg[e] = p; }  // strict >: the first maximum wins
            pos[e] |= (v[e] > 0.f ? 1u : 0u) << p;
        }
    }
    vec_io<T, VEC>::ld(dy + o * C + c, g);
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int64_t u = ((n * 2 * D + 2 * d + (p >> 2)) * 2 * H + 2 * h + ((p >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (p & 1);
        if (add) vec_io<T, VEC>::ld(add + u * C + c, a);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            r[e] = (arg[e] == p ? g[e] : 0.f) + (add ? a[e] : 0.f);
            if (relu_mask && !((pos[e] >> p) & 1)) r[e] = 0.f;
        }
        vec_io<T, VEC>::st(dx + u * C + c, r);
    }
}

template <typename T, int VEC>
static int pool_launch(bool bwd, const void *x, const void *dy, const void *add, int relu_mask, void *out, int64_t N, int64_t D,
                       int64_t H, int64_t W, int64_t C, hipStream_t st)
{
    int64_t total = N * D * H * W * (C / VEC);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    if (!bwd)
        pool_fwd_kernel<T, VEC><<<dim3((unsigned)blocks), 256, 0, st>>>((const T *)x, (T *)out, total, (int)D, (int)H,
                                                                        (int)W, (int)C);
    else
        pool_bwd_kernel<T, VEC><<<dim3((unsigned)blocks), 256, 0, st>>>((const T *)x, (const T *)dy, (const T *)add, relu_mask,
                                                                        (T *)out, total, (int)D, (int)H, (int)W, (int)C);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

// Forward pooling that also writes the backward pass's routing as one bit per INPUT element, in
// the layout of the ReLU bit masks (a uint16 word per 16 channels of a voxel): the bit is set
// where the element is the first maximum of its window (order i, j, k; strict >, as
// pool_bwd_kernel decides) and greater than zero, i.e. where the pooled gradient arrives AND
// passes the ReLU that produced x.  One thread: 8 channels of one output window, i.e. one byte of
// bits per input voxel; the lanes of a pair (QUAD: of a quad, when C is a multiple of 32) hold
// neighbouring bytes of the same voxel, exchange them across lanes and the first lane stores the
// word (C / 8 is even, and a multiple of 4 with QUAD, so pairs / quads never straddle a voxel or
// the end of the grid).
template <bool QUAD>
__global__ __launch_bounds__(256) void pool_fwd_bits_kernel(const bf16_t *__restrict__ x, bf16_t *__restrict__ y,
                                                           unsigned char *__restrict__ route, int64_t total, int D, int H,
                                                           int W, int C)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int cv = C / 8;
    int c = (int)(gid % cv) * 8;
    int64_t o = gid / cv;
    int w = (int)(o % W);
    int h = (int)((o / W) % H);
    int d = (int)((o / ((int64_t)W * H)) % D);
    int64_t n = o / ((int64_t)W * H * D);
    float m[8], v[8];
    int arg[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int64_t u = ((n * 2 * D + 2 * d + (p >> 2)) * 2 * H + 2 * h + ((p >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (p & 1);
        vec_io<bf16_t, 8>::ld(x + u * C + c, v);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (p == 0 || v[e] > m[e]) { m[e] = v[e]; arg[e] = p; }
    }
    vec_io<bf16_t, 8>::st(y + o * C + c, m);
#pragma unroll
    for (int e = 0; e < 8; ++e)
        if (!(m[e] > 0.f)) arg[e] = 8;   // nothing is routed through a ReLU that was off
    const int sub = threadIdx.x & (QUAD ? 3 : 1);
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int64_t u = ((n * 2 * D + 2 * d + (p >> 2)) * 2 * H + 2 * h + ((p >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (p & 1);
        unsigned b = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) b |= (arg[e] == p ? 1u : 0u) << e;
        b |= (unsigned)__builtin_amdgcn_mov_dpp((int)b, 0xB1, 0xf, 0xf, true) << 8;        // lanes ^ 1
        if (QUAD) {
            b |= (unsigned)__builtin_amdgcn_mov_dpp((int)b, 0x4E, 0xf, 0xf, true) << 16;   // lanes ^ 2
            if (sub == 0) *reinterpret_cast<unsigned *>(route + ((u * C + c) >> 3)) = b;
        } else {
            if (sub == 0) *reinterpret_cast<unsigned short *>(route + ((u * C + c) >> 3)) = (unsigned short)b;
        }
    }
}

// Backward pooling from those bits: dx = the window's dy where the bit is set, zero elsewhere (the
// 16-bit patterns are passed through, nothing is computed).  Reads 1/16 of what pool_bwd_kernel
// reads for x.
__global__ __launch_bounds__(256) void pool_bwd_bits_kernel(const unsigned char *__restrict__ route,
                                                           const bf16_t *__restrict__ dy, bf16_t *__restrict__ dx,
                                                           int64_t total, int D, int H, int W, int C)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int cv = C / 8;
    int c = (int)(gid % cv) * 8;
    int64_t o = gid / cv;
    int w = (int)(o % W);
    int h = (int)((o / W) % H);
    int d = (int)((o / ((int64_t)W * H)) % D);
    int64_t n = o / ((int64_t)W * H * D);
    const uint4 g = *reinterpret_cast<const uint4 *>(dy + o * C + c);
    unsigned b[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int64_t u = ((n * 2 * D + 2 * d + (p >> 2)) * 2 * H + 2 * h + ((p >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (p & 1);
        b[p] = route[(u * C + c) >> 3];
    }
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int64_t u = ((n * 2 * D + 2 * d + (p >> 2)) * 2 * H + 2 * h + ((p >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (p & 1);
        auto keep = [&](unsigned word, int pair) {   // channels 2 pair, 2 pair + 1 of the thread's eight
            const unsigned lo = (b[p] >> (2 * pair)) & 1u, hi = (b[p] >> (2 * pair + 1)) & 1u;
            return word & (((0u - lo) & 0x0000ffffu) | ((0u - hi) & 0xffff0000u));
        };
        *reinterpret_cast<uint4 *>(dx + u * C + c) = make_uint4(keep(g.x, 0), keep(g.y, 1), keep(g.z, 2), keep(g.w, 3));
    }
}

// Nearest-neighbour up-sampling by 2 per axis.  D, H, W are the INPUT sizes; the output is
// (2D, 2H, 2W).  Forward: one thread per VEC channels of one OUTPUT voxel (each input vector is
// read by the eight threads of its block, served by the cache; every store is coalesced).
template <typename T, int VEC>
__global__ __launch_bounds__(256) void upsample_fwd_kernel(const T *__restrict__ x, T *__restrict__ y, int64_t total,
                                                          int D, int H, int W, int C)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int cv = C / VEC;
    int c = (int)(gid % cv) * VEC;
    int64_t o = gid / cv;
    int w = (int)(o % (2 * W));
    int h = (int)((o / (2 * W)) % (2 * H));
    int d = (int)((o / ((int64_t)4 * W * H)) % (2 * D));
    int64_t n = o / ((int64_t)8 * W * H * D);
    int64_t u = ((n * D + (d >> 1)) * H + (h >> 1)) * (int64_t)W + (w >> 1);
    float v[VEC];
    vec_io<T, VEC>::ld(x + u * C + c, v);
    vec_io<T, VEC>::st(y + o * C + c, v);
}

// Backward: the adjoint, dx = sum of dy over the 2x2x2 block in a fixed order (fp32), then the
// ReLU mask of the stored forward input when one is given.  One thread per VEC channels of one
// INPUT voxel.
template <typename T, int VEC>
__global__ __launch_bounds__(256) void upsample_bwd_kernel(const T *__restrict__ dy, const T *__restrict__ xmask,
                                                          T *__restrict__ dx, int64_t total, int D, int H, int W, int C)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int cv = C / VEC;
    int c = (int)(gid % cv) * VEC;
    int64_t o = gid / cv;
    int w = (int)(o % W);
    int h = (int)((o / W) % H);
    int d = (int)((o / ((int64_t)W * H)) % D);
    int64_t n = o / ((int64_t)W * H * D);
    float acc[VEC], v[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
        int64_t u = ((n * 2 * D + 2 * d + (p >> 2)) * 2 * H + 2 * h + ((p >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (p & 1);
        vec_io<T, VEC>::ld(dy + u * C + c, v);
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] += v[e];
    }
    if (xmask) {
        vec_io<T, VEC>::ld(xmask + o * C + c, v);
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            if (!(v[e] > 0.f)) acc[e] = 0.f;
    }
    vec_io<T, VEC>::st(dx + o * C + c, acc);
}

template <typename T, int VEC>
static int upsample_launch(bool bwd, const void *in, const void *xmask, void *out, int64_t N, int64_t D, int64_t H, int64_t W,
                           int64_t C, hipStream_t st)
{
    int64_t total = N * D * H * W * (C / VEC) * (bwd ? 1 : 8);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    if (!bwd)
        upsample_fwd_kernel<T, VEC><<<dim3((unsigned)blocks), 256, 0, st>>>((const T *)in, (T *)out, total, (int)D, (int)H,
                                                                            (int)W, (int)C);
    else
        upsample_bwd_kernel<T, VEC><<<dim3((unsigned)blocks), 256, 0, st>>>((const T *)in, (const T *)xmask, (T *)out, total,
                                                                            (int)D, (int)H, (int)W, (int)C);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

static int upsample_dispatch(bool bwd, int dtype, const void *in, const void *xmask, void *out, int64_t N, int64_t D, int64_t H,
                             int64_t W, int64_t C, hipStream_t st)
{
    if (dtype == K3_BF16) {
        if (C % 8 == 0) return upsample_launch<bf16_t, 8>(bwd, in, xmask, out, N, D, H, W, C, st);
        return upsample_launch<bf16_t, 1>(bwd, in, xmask, out, N, D, H, W, C, st);
    }
    if (C % 4 == 0) return upsample_launch<float, 4>(bwd, in, xmask, out, N, D, H, W, C, st);
    return upsample_launch<float, 1>(bwd, in, xmask, out, N, D, H, W, C, st);
}

static int pool_dispatch(bool bwd, int dtype, const void *x, const void *dy, const void *add, int relu_mask, void *out, int64_t N,
                         int64_t D, int64_t H, int64_t W, int64_t C, hipStream_t st)
{
    if (dtype == K3_BF16) {
        if (C % 8 == 0) return pool_launch<bf16_t, 8>(bwd, x, dy, add, relu_mask, out, N, D, H, W, C, st);
        return pool_launch<bf16_t, 1>(bwd, x, dy, add, relu_mask, out, N, D, H, W, C, st);
    }
    if (C % 4 == 0) return pool_launch<float, 4>(bwd, x, dy, add, relu_mask, out, N, D, H, W, C, st);
    return pool_launch<float, 1>(bwd, x, dy, add, relu_mask, out, N, D, H, W, C, st);
}

static int pool_check(const k3_tensor *xd, const k3_tensor *yd)
{
    if (!desc_ok(xd) || !desc_ok(yd)) return K3_E_BADARG;
    if (xd->d % 2 || xd->h % 2 || xd->w % 2) return K3_E_SHAPE;
    if (yd->n != xd->n || yd->d * 2 != xd->d || yd->h * 2 != xd->h || yd->w * 2 != xd->w || yd->c != xd->c ||
        yd->dtype != xd->dtype)
        return K3_E_SHAPE;
    if (xd->d > 0x3fffffff || xd->h > 0x3fffffff || xd->w > 0x3fffffff || xd->c > 0x3fffffff) return K3_E_UNSUPPORTED;
    return K3_OK;
}

}  // namespace k3

using namespace k3;

extern "C" int k3_pool3d_fwd(const k3_tensor *xd, const void *x, const k3_tensor *yd, void *y, void *stream)
{
    int rc = pool_check(xd, yd);
    if (rc != K3_OK) return rc;
    if (!x || !y) return K3_E_BADARG;
    return pool_dispatch(false, xd->dtype, x, nullptr, nullptr, 0, y, yd->n, yd->d, yd->h, yd->w, yd->c, (hipStream_t)stream);
}

extern "C" int k3_pool3d_bwd(const k3_tensor *xd, const void *x, const k3_tensor *dyd, const void *dy, const void *add,
                             int relu_mask, void *dx, void *stream)
{
    int rc = pool_check(xd, dyd);
    if (rc != K3_OK) return rc;
    if (!x || !dy || !dx) return K3_E_BADARG;
    return pool_dispatch(true, xd->dtype, x, dy, add, relu_mask ? 1 : 0, dx, dyd->n, dyd->d, dyd->h, dyd->w, dyd->c, (hipStream_t)stream);
}

static int pool_bits_check(const k3_tensor *xd, const k3_tensor *yd)
{
    int rc = pool_check(xd, yd);
    if (rc != K3_OK) return rc;
    if (xd->dtype != K3_BF16 || xd->c % 16 != 0) return K3_E_UNSUPPORTED;
    return K3_OK;
}

extern "C" int k3_pool3d_fwd_bits(const k3_tensor *xd, const void *x, const k3_tensor *yd, void *y, void *route_bits,
                                  void *stream)
{
    int rc = pool_bits_check(xd, yd);
    if (rc != K3_OK) return rc;
    if (!x || !y || !route_bits) return K3_E_BADARG;
    const int64_t total = yd->n * yd->d * yd->h * yd->w * (yd->c / 8);
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    if (yd->c % 32 == 0)
        pool_fwd_bits_kernel<true><<<dim3((unsigned)blocks), 256, 0, (hipStream_t)stream>>>(
            (const bf16_t *)x, (bf16_t *)y, (unsigned char *)route_bits, total, (int)yd->d, (int)yd->h, (int)yd->w, (int)yd->c);
    else
        pool_fwd_bits_kernel<false><<<dim3((unsigned)blocks), 256, 0, (hipStream_t)stream>>>(
            (const bf16_t *)x, (bf16_t *)y, (unsigned char *)route_bits, total, (int)yd->d, (int)yd->h, (int)yd->w, (int)yd->c);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

extern "C" int k3_pool3d_bwd_bits(const k3_tensor *xd, const void *route_bits, const k3_tensor *dyd, const void *dy, void *dx,
                                  void *stream)
{
    int rc = pool_bits_check(xd, dyd);
    if (rc != K3_OK) return rc;
    if (!route_bits || !dy || !dx) return K3_E_BADARG;
    const int64_t total = dyd->n * dyd->d * dyd->h * dyd->w * (dyd->c / 8);
    const int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    pool_bwd_bits_kernel<<<dim3((unsigned)blocks), 256, 0, (hipStream_t)stream>>>(
        (const unsigned char *)route_bits, (const bf16_t *)dy, (bf16_t *)dx, total, (int)dyd->d, (int)dyd->h, (int)dyd->w,
        (int)dyd->c);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

// xd: the small tensor (D, H, W); yd: the large one (2D, 2H, 2W): the same relation pool_check tests,
// with the roles of input and output exchanged.
extern "C" int k3_upsample3d_fwd(const k3_tensor *xd, const void *x, const k3_tensor *yd, void *y, void *stream)
{
    int rc = pool_check(yd, xd);
    if (rc != K3_OK) return rc;
    if (!x || !y) return K3_E_BADARG;
    return upsample_dispatch(false, xd->dtype, x, nullptr, y, xd->n, xd->d, xd->h, xd->w, xd->c, (hipStream_t)stream);
}

extern "C" int k3_upsample3d_bwd(const k3_tensor *dyd, const void *dy, const void *x_mask, const k3_tensor *dxd, void *dx,
                                 void *stream)
{
    int rc = pool_check(dyd, dxd);
    if (rc != K3_OK) return rc;
    if (!dy || !dx) return K3_E_BADARG;
    return upsample_dispatch(true, dxd->dtype, dy, x_mask, dx, dxd->n, dxd->d, dxd->h, dxd->w, dxd->c, (hipStream_t)stream);
}
