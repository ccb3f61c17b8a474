// Direct (non-MFMA) 3x3x3 convolution kernels for gfx950: fp32 tensors and bf16 tensors
// whose channel counts do not fit the MFMA tiles (for example the single-channel first
// layer).  One thread per output element, fp32 accumulation, taps visited in (kd,kh,kw)
// order.  These kernels favour generality; the hot shapes go through conv3d_mfma.hip.
#include "common.h"
#include "conv_internal.h"

namespace k3 {

template <typename T>
__global__ __launch_bounds__(256) void conv_fwd_direct_kernel(
    const T *__restrict__ x, const T *__restrict__ x2, int c1, int c2, const T *__restrict__ w,
    const float *__restrict__ bias, int relu, T *__restrict__ y, int64_t N, int D, int H, int W, int cout)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t V = N * D * H * W;
    if (gid >= V * cout) return;
    int co = (int)(gid % cout);
    int64_t v = gid / cout;
    int ww = (int)(v % W);
    int hh = (int)((v / W) % H);
    int dd = (int)((v / ((int64_t)W * H)) % D);
    int64_t n = v / ((int64_t)W * H * D);
    int cin = c1 + c2;
    float acc = bias ? bias[co] : 0.f;
    for (int kd = 0; kd < 3; ++kd) {
        int zd = dd + kd - 1;
        if (zd < 0 || zd >= D) continue;
        for (int kh = 0; kh < 3; ++kh) {
            int zh = hh + kh - 1;
            if (zh < 0 || zh >= H) continue;
            for (int kw = 0; kw < 3; ++kw) {
                int zw = ww + kw - 1;
                if (zw < 0 || zw >= W) continue;
                int64_t u = ((n * D + zd) * H + zh) * (int64_t)W + zw;
                const T *wp = w + ((int64_t)((kd * 3 + kh) * 3 + kw) * cin) * cout + co;
                const T *xp = x + u * c1;
                for (int ci = 0; ci < c1; ++ci) acc += elem<T>::ld(xp + ci) * elem<T>::ld(wp + (int64_t)ci * cout);
                if (c2 > 0) {
                    const T *xq = x2 + u * c2;
                    const T *wq = wp + (int64_t)c1 * cout;
                    for (int ci = 0; ci < c2; ++ci) acc += elem<T>::ld(xq + ci) * elem<T>::ld(wq + (int64_t)ci * cout);
                }
            }
        }
    }
    if (relu) acc = acc > 0.f ? acc : 0.f;
    elem<T>::st(y + gid, acc);
}

template <typename T>
__global__ __launch_bounds__(256) void conv_dgrad_direct_kernel(
    const T *__restrict__ dy, const T *__restrict__ ymask, const T *__restrict__ w,
    T *__restrict__ dx, T *__restrict__ dx2, const T *__restrict__ omask, int c1, int c2, int64_t N, int D, int H, int W,
    int cout)
{
    int cin = c1 + c2;
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int64_t V = N * D * H * W;
    if (gid >= V * cin) return;
    int ci = (int)(gid % cin);
    int64_t v = gid / cin;
    int ww = (int)(v % W);
    int hh = (int)((v / W) % H);
    int dd = (int)((v / ((int64_t)W * H)) % D);
    int64_t n = v / ((int64_t)W * H * D);
    float acc = 0.f;
    for (int kd = 0; kd < 3; ++kd) {
        int zd = dd - kd + 1;
        if (zd < 0 || zd >= D) continue;
        for (int kh = 0; kh < 3; ++kh) {
            int zh = hh - kh + 1;
            if (zh < 0 || zh >= H) continue;
            for (int kw = 0; kw < 3; ++kw) {
                int zw = ww - kw + 1;
                if (zw < 0 || zw >= W) continue;
                int64_t u = ((n * D + zd) * H + zh) * (int64_t)W + zw;
                const T *gp = dy + u * cout;
                const T *mp = ymask ? ymask + u * cout : nullptr;
                const T *wp = w + ((int64_t)((kd * 3 + kh) * 3 + kw) * cin + ci) * cout;
                for (int co = 0; co < cout; ++co) {
                    float g = elem<T>::ld(gp + co);
                    if (mp && !(elem<T>::ld(mp + co) > 0.f)) g = 0.f;
                    acc += g * elem<T>::ld(wp + co);
                }
            }
        }
    }
    if (ci < c1) {
        if (omask && !(elem<T>::ld(omask + v * c1 + ci) > 0.f)) acc = 0.f;
        elem<T>::st(dx + v * c1 + ci, acc);
    } else {
        elem<T>::st(dx2 + v * c2 + (ci - c1), acc);
    }
}

// Weight gradient: block (split s, ci-block b, co-block z) sums its voxel slab.
// Thread t owns output channel z*CB + t % CB and every (256/CB)-th voxel of the slab and
// keeps 27 x CIB accumulators; the threads of one channel are then added in a fixed order.
constexpr int WG_CIB = 4;

template <typename T>
__global__ __launch_bounds__(256) void conv_wgrad_direct_kernel(
    const T *__restrict__ x, const T *__restrict__ x2, int c1, int c2,
    const T *__restrict__ dy, const T *__restrict__ ymask, float *__restrict__ ws,
    int64_t N, int D, int H, int W, int cout, int CB, int64_t slab, int64_t per_split)
{
    __shared__ float red[256];
    int cin = c1 + c2;
    int tid = threadIdx.x;
    int nvs = 256 / CB;
    int cl = tid % CB, vs = tid / CB;
    int co = blockIdx.z * CB + cl;
    bool active = (vs < nvs) && (co < cout);
    int ci0 = blockIdx.y * WG_CIB;
    int64_t V = N * D * H * W;
    int64_t v0 = (int64_t)blockIdx.x * slab;
    int64_t v1 = v0 + slab < V ? v0 + slab : V;
    float acc[27][WG_CIB];
    float accb = 0.f;
#pragma unroll
    for (int t = 0; t < 27; ++t)
#pragma unroll
        for (int c = 0; c < WG_CIB; ++c) acc[t][c] = 0.f;
    if (active) {
        for (int64_t v = v0 + vs; v < v1; v += nvs) {
            float g = elem<T>::ld(dy + v * cout + co);
            if (ymask && !(elem<T>::ld(ymask + v * cout + co) > 0.f)) g = 0.f;
            accb += g;
            int ww = (int)(v % W);
            int hh = (int)((v / W) % H);
            int dd = (int)((v / ((int64_t)W * H)) % D);
            int64_t n = v / ((int64_t)W * H * D);
#pragma unroll
            for (int t = 0; t < 27; ++t) {
                int zd = dd + t / 9 - 1, zh = hh + (t / 3) % 3 - 1, zw = ww + t % 3 - 1;
                if (zd < 0 || zd >= D || zh < 0 || zh >= H || zw < 0 || zw >= W) continue;
                int64_t u = ((n * D + zd) * H + zh) * (int64_t)W + zw;
#pragma unroll
                for (int c = 0; c < WG_CIB; ++c) {
                    int ci = ci0 + c;
                    if (ci < cin) {
                        float xv = ci < c1 ? elem<T>::ld(x + u * c1 + ci) : elem<T>::ld(x2 + u * c2 + (ci - c1));
                        acc[t][c] += xv * g;
                    }
                }
            }
        }
    }
    float *out = ws + (int64_t)blockIdx.x * per_split;
#pragma unroll
    for (int t = 0; t < 27; ++t)
#pragma unroll
        for (int c = 0; c < WG_CIB; ++c) {
            red[tid] = acc[t][c];
            __syncthreads();
            if (active && vs == 0 && ci0 + c < cin) {
                float s = 0.f;
                for (int k = 0; k < nvs; ++k) s += red[k * CB + cl];
                out[((int64_t)t * cin + ci0 + c) * cout + co] = s;
            }
            __syncthreads();
        }
    if (blockIdx.y == 0) {
        red[tid] = accb;
        __syncthreads();
        if (active && vs == 0) {
            float s = 0.f;
            for (int k = 0; k < nvs; ++k) s += red[k * CB + cl];
            out[(int64_t)27 * cin * cout + co] = s;
        }
    }
}

// out[i] = sum_s ws[s*count + i] in a fixed order: a block owns 64 entries; its 4 thread groups
// add the splits g, g+4, g+8, ... in increasing order and the four group sums are then combined
// as ((g0+g1)+g2)+g3.  The first countW entries go to dW, the remaining ones (bias gradient)
// to db when it is not null.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ ws, float *__restrict__ dW,
                                                             float *__restrict__ db, int64_t countW, int64_t count,
                                                             int nsplit)
{
    __shared__ float part[4][64];
    const int e = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + e;
    float s0 = 0.f, s1 = 0.f;
    if (i < count) {
        int k = g;
        for (; k + 4 < nsplit; k += 8) {   // two independent chains, merged below in a fixed order
            s0 += ws[(int64_t)k * count + i];
            s1 += ws[(int64_t)(k + 4) * count + i];
        }
        if (k < nsplit) s0 += ws[(int64_t)k * count + i];
    }
    part[g][e] = s0 + s1;
    __syncthreads();
    if (g == 0 && i < count) {
        float s = ((part[0][e] + part[1][e]) + part[2][e]) + part[3][e];
        if (i < countW) dW[i] = s;
        else if (db) db[i - countW] = s;
    }
}

// Same sum for 16-byte aligned buffers whose element counts are multiples of 4: a thread adds
// float4 quads, 16 quads x 16 groups of splits per block, groups merged in a fixed order.
__global__ __launch_bounds__(256) void reduce_partials_vec4_kernel(const float4 *__restrict__ ws, float4 *__restrict__ dW,
                                                                  float4 *__restrict__ db, int64_t quadsW, int64_t quads,
                                                                  int nsplit)
{
    __shared__ float4 part[16][16];
    const int e = threadIdx.x & 15, g = threadIdx.x >> 4;
    const int64_t i = (int64_t)blockIdx.x * 16 + e;
    float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0;
    if (i < quads) {
        int k = g;
        for (; k + 16 < nsplit; k += 32) {   // two independent chains
            const float4 a = ws[(int64_t)k * quads + i], b = ws[(int64_t)(k + 16) * quads + i];
            s0.x += a.x; s0.y += a.y; s0.z += a.z; s0.w += a.w;
            s1.x += b.x; s1.y += b.y; s1.z += b.z; s1.w += b.w;
        }
        if (k < nsplit) {
            const float4 a = ws[(int64_t)k * quads + i];
            s0.x += a.x; s0.y += a.y; s0.z += a.z; s0.w += a.w;
        }
    }
    part[g][e] = make_float4(s0.x + s1.x, s0.y + s1.y, s0.z + s1.z, s0.w + s1.w);
    __syncthreads();
    if (g == 0 && i < quads) {
        float4 s = part[0][e];
#pragma unroll
        for (int q = 1; q < 16; ++q) {
            const float4 a = part[q][e];
            s.x += a.x; s.y += a.y; s.z += a.z; s.w += a.w;
        }
        if (i < quadsW) dW[i] = s;
        else if (db) db[i - quadsW] = s;
    }
}

int launch_reduce_partials(const float *ws, float *dW, float *db, int64_t countW, int64_t count, int nsplit,
                           hipStream_t st)
{
    const bool vec = count % 4 == 0 && countW % 4 == 0 && ((uintptr_t)ws & 15) == 0 && ((uintptr_t)dW & 15) == 0 &&
                     ((uintptr_t)db & 15) == 0;
    if (vec) {
        const int64_t quads = count / 4;
        reduce_partials_vec4_kernel<<<dim3((unsigned)((quads + 15) / 16)), 256, 0, st>>>(
            (const float4 *)ws, (float4 *)dW, (float4 *)db, countW / 4, quads, nsplit);
        K3_LAUNCH_CHECK();
        return K3_OK;
    }
    int64_t blocks = (count + 63) / 64;
    reduce_partials_kernel<<<dim3((unsigned)blocks), 256, 0, st>>>(ws, dW, db, countW, count, nsplit);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

static int64_t direct_nsplit(int64_t V)
{
    int64_t s = V / 256;
    if (s < 1) s = 1;
    if (s > 1024) s = 1024;
    return s;
}

size_t conv_wgrad_direct_ws_bytes(int64_t V, int64_t cin, int64_t cout)
{
    return (size_t)direct_nsplit(V) * (size_t)(27 * cin * cout + cout) * sizeof(float);
}

template <typename T>
static int fwd_direct_t(const ConvArgs &a, hipStream_t st)
{
    int64_t total = a.V() * a.cout;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    conv_fwd_direct_kernel<T><<<dim3((unsigned)blocks), 256, 0, st>>>(
        (const T *)a.x, (const T *)a.x2, (int)a.c1, (int)a.c2, (const T *)a.w, a.bias, a.relu, (T *)a.y, a.N,
        (int)a.D, (int)a.H, (int)a.W, (int)a.cout);
    K3_LAUNCH_CHECK();
    return K3_OK;
}
// ---- one-bit-per-element ReLU masks, generic passes (the MFMA kernels produce / consume the
// bits themselves; these serve the kernels that do not)
template <typename T>
__global__ __launch_bounds__(256) void relu_bits_kernel(const T *__restrict__ y, unsigned short *__restrict__ bits, int64_t nwords)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nwords; i += stride) {
        unsigned m = 0u;
#pragma unroll
        for (int e = 0; e < 16; ++e) m |= (elem<T>::ld(y + i * 16 + e) > 0.f ? 1u : 0u) << e;
        bits[i] = (unsigned short)m;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void apply_relu_bits_kernel(T *__restrict__ t, const unsigned short *__restrict__ bits,
                                                             int64_t nwords)
{
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < nwords; i += stride) {
        const unsigned m = bits[i];
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (!((m >> e) & 1u)) elem<T>::st(t + i * 16 + e, 0.f);
    }
}

int launch_relu_bits(int dtype, const void *y, void *bits, int64_t nwords, hipStream_t st)
{
    const int64_t want = (nwords + 255) / 256;
    const unsigned grid = (unsigned)(want < 8192 ? (want > 0 ? want : 1) : 8192);
    if (dtype == K3_F32) relu_bits_kernel<float><<<dim3(grid), 256, 0, st>>>((const float *)y, (unsigned short *)bits, nwords);
    else relu_bits_kernel<bf16_t><<<dim3(grid), 256, 0, st>>>((const bf16_t *)y, (unsigned short *)bits, nwords);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

int launch_apply_relu_bits(int dtype, void *t, const void *bits, int64_t nwords, hipStream_t st)
{
    const int64_t want = (nwords + 255) / 256;
    const unsigned grid = (unsigned)(want < 8192 ? (want > 0 ? want : 1) : 8192);
    if (dtype == K3_F32) apply_relu_bits_kernel<float><<<dim3(grid), 256, 0, st>>>((float *)t, (const unsigned short *)bits, nwords);
    else apply_relu_bits_kernel<bf16_t><<<dim3(grid), 256, 0, st>>>((bf16_t *)t, (const unsigned short *)bits, nwords);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

int conv_fwd_direct(const ConvArgs &a, hipStream_t st)
{
    return a.dtype == K3_F32 ? fwd_direct_t<float>(a, st) : fwd_direct_t<bf16_t>(a, st);
}

template <typename T>
static int dgrad_direct_t(const ConvArgs &a, hipStream_t st)
{
    int64_t total = a.V() * (a.c1 + a.c2);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    conv_dgrad_direct_kernel<T><<<dim3((unsigned)blocks), 256, 0, st>>>(
        (const T *)a.dy, (const T *)a.ymask, (const T *)a.w, (T *)a.dx, (T *)a.dx2, (const T *)a.omask, (int)a.c1, (int)a.c2, a.N,
        (int)a.D, (int)a.H, (int)a.W, (int)a.cout);
    K3_LAUNCH_CHECK();
    return K3_OK;
}
int conv_dgrad_direct(const ConvArgs &a, hipStream_t st)
{
    return a.dtype == K3_F32 ? dgrad_direct_t<float>(a, st) : dgrad_direct_t<bf16_t>(a, st);
}

template <typename T>
static int wgrad_direct_t(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st)
{
    int64_t V = a.V();
    int64_t cin = a.c1 + a.c2;
    int64_t nsplit = direct_nsplit(V);
    int64_t slab = (V + nsplit - 1) / nsplit;
    int CB = a.cout < 256 ? (int)a.cout : 256;
    int64_t per_split = 27 * cin * a.cout + a.cout;
    dim3 grid((unsigned)nsplit, (unsigned)((cin + WG_CIB - 1) / WG_CIB), (unsigned)((a.cout + CB - 1) / CB));
    if (grid.y > 65535 || grid.z > 65535) return K3_E_UNSUPPORTED;
    conv_wgrad_direct_kernel<T><<<grid, 256, 0, st>>>((const T *)a.x, (const T *)a.x2, (int)a.c1, (int)a.c2,
                                                      (const T *)a.dy, (const T *)a.ymask, ws, a.N, (int)a.D,
                                                      (int)a.H, (int)a.W, (int)a.cout, CB, slab, per_split);
    K3_LAUNCH_CHECK();
    return launch_reduce_partials(ws, dW, db, 27 * cin * a.cout, per_split, (int)nsplit, st);
}
int conv_wgrad_direct(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st)
{
    return a.dtype == K3_F32 ? wgrad_direct_t<float>(a, dW, db, ws, st) : wgrad_direct_t<bf16_t>(a, dW, db, ws, st);
}

}  // namespace k3
