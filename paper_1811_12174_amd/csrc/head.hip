// 1x1x1 head (C -> 3 classes) fused with softmax cross-entropy, forward and backward in a
// single pass over the activations, for gfx950.  HBM-bound: reads a and the labels once,
// writes da (and optionally the logits) once.
//
// A workgroup walks batches of 256 voxels.  The batch's activation rows are copied into LDS
// with coalesced loads; thread v then owns voxel v (logits, softmax, loss term, dz, and the
// da row, which it writes into a second LDS tile so the store to memory is coalesced too);
// afterwards thread (c, group) accumulates dWh[c][0..2] over a quarter of the batch.  Each
// workgroup writes its partial sums (dWh, dbh, loss); a one-block kernel adds the partials
// in block order, so the result is run-to-run identical.
#include "common.h"

namespace k3 {

constexpr int HB = 256;       // voxels per batch
constexpr int HEAD_K = 3;

// da may be a itself: a workgroup reads the rows of a batch into LDS before it writes that batch's
// rows of da, and no other workgroup touches them (hence no __restrict__ on the two).
template <typename T>
__global__ __launch_bounds__(256) void head_kernel(const T *a, const float *__restrict__ wh,
                                                  const float *__restrict__ bh, const uint8_t *__restrict__ labels,
                                                  T *da, float *__restrict__ logits,
                                                  float *__restrict__ partial, int64_t V, int C, float invV, int relu_mask,
                                                  const float *__restrict__ cw)
{
    const float cw0 = cw ? cw[0] : 1.f, cw1 = cw ? cw[1] : 1.f, cw2 = cw ? cw[2] : 1.f;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int rowb = C * (int)sizeof(T) + 4;  // padded row: consecutive voxels start in consecutive banks
    unsigned char *as = smem;
    unsigned char *ds = smem + HB * rowb;
    float *dzs = reinterpret_cast<float *>(smem + 2 * HB * rowb);  // [HB][4]
    float *red = dzs + HB * 4;                                       // [256]
    const int tid = threadIdx.x;
    const int ngrp = 256 / C;
    const int c2 = tid % C, grp = tid / C;
    const bool acc_thread = grp < ngrp;
    float accw0 = 0.f, accw1 = 0.f, accw2 = 0.f;
    float lossacc = 0.f, db0 = 0.f, db1 = 0.f, db2 = 0.f;
    const int64_t nbatch = (V + HB - 1) / HB;
    const int rowwords = C * (int)sizeof(T) / 4;  // 4-byte words per row (C*sizeof(T) is a multiple of 4)

    for (int64_t b = blockIdx.x; b < nbatch; b += gridDim.x) {
        const int64_t v0 = b * HB;
        const int nv = (int)((V - v0) < HB ? (V - v0) : HB);
        __syncthreads();
        {   // coalesced copy of nv rows into the padded LDS tile
            const uint32_t *src = reinterpret_cast<const uint32_t *>(a + v0 * C);
            for (int i = tid; i < nv * rowwords; i += 256) {
                int r = i / rowwords, q = i - r * rowwords;
                *reinterpret_cast<uint32_t *>(as + r * rowb + q * 4) = src[i];
            }
        }
        __syncthreads();
        if (tid < nv) {
            const T *row = reinterpret_cast<const T *>(as + tid * rowb);
            float z0 = bh ? bh[0] : 0.f, z1 = bh ? bh[1] : 0.f, z2 = bh ? bh[2] : 0.f;
            for (int c = 0; c < C; ++c) {
                float av = elem<T>::ld(row + c);
                z0 += av * wh[c * 3 + 0];
                z1 += av * wh[c * 3 + 1];
                z2 += av * wh[c * 3 + 2];
            }
            if (logits) {
                float *lp = logits + (v0 + tid) * 3;
                lp[0] = z0; lp[1] = z1; lp[2] = z2;
            }
            float m = fmaxf(z0, fmaxf(z1, z2));
            float e0 = expf(z0 - m), e1 = expf(z1 - m), e2 = expf(z2 - m);
            float den = e0 + e1 + e2;
            float inv = 1.f / den;
            int lab = labels[v0 + tid];
            float zl = lab == 0 ? z0 : (lab == 1 ? z1 : z2);
            const float wl = lab == 0 ? cw0 : (lab == 1 ? cw1 : cw2);   // class weight of this voxel
            const float sc = invV * wl;
            lossacc += wl * ((m - zl) + logf(den));
            float d0 = (e0 * inv - (lab == 0 ? 1.f : 0.f)) * sc;
            float d1 = (e1 * inv - (lab == 1 ? 1.f : 0.f)) * sc;
            float d2 = (e2 * inv - (lab == 2 ? 1.f : 0.f)) * sc;
            db0 += d0; db1 += d1; db2 += d2;
            dzs[tid * 4 + 0] = d0; dzs[tid * 4 + 1] = d1; dzs[tid * 4 + 2] = d2;
            T *drow = reinterpret_cast<T *>(ds + tid * rowb);
            for (int c = 0; c < C; ++c) {
                float gv = d0 * wh[c * 3 + 0] + d1 * wh[c * 3 + 1] + d2 * wh[c * 3 + 2];
                if (relu_mask && !(elem<T>::ld(row + c) > 0.f)) gv = 0.f;
                elem<T>::st(drow + c, gv);
            }
        }
        __syncthreads();
        {   // coalesced store of the da rows
            uint32_t *dst = reinterpret_cast<uint32_t *>(da + v0 * C);
            for (int i = tid; i < nv * rowwords; i += 256) {
                int r = i / rowwords, q = i - r * rowwords;
                dst[i] = *reinterpret_cast<const uint32_t *>(ds + r * rowb + q * 4);
            }
        }
        if (acc_thread) {
            for (int v = grp; v < nv; v += ngrp) {
                float av = elem<T>::ld(reinterpret_cast<const T *>(as + v * rowb) + c2);
                accw0 += av * dzs[v * 4 + 0];
                accw1 += av * dzs[v * 4 + 1];
                accw2 += av * dzs[v * 4 + 2];
            }
        }
    }
    // block partials: [C*3 dWh][3 dbh][1 loss]
    float *out = partial + (int64_t)blockIdx.x * (C * 3 + 4);
    float accw[3] = {accw0, accw1, accw2};
    for (int k = 0; k < 3; ++k) {
        __syncthreads();
        red[tid] = acc_thread ? accw[k] : 0.f;
        __syncthreads();
        if (tid < C) {
            float s = 0.f;
            for (int g = 0; g < ngrp; ++g) s += red[g * C + tid];
            out[tid * 3 + k] = s;
        }
    }
    float sc[4] = {db0, db1, db2, lossacc};
    for (int k = 0; k < 4; ++k) {
        __syncthreads();
        red[tid] = sc[k];
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) red[tid] += red[tid + s];
            __syncthreads();
        }
        if (tid == 0) out[C * 3 + k] = red[0];
    }
}

// Streaming variant for bf16 activations whose channel count is a multiple of 16 (the U-Net
// levels): LPV = C / 16 neighbouring lanes share a voxel, 16 channels (32 bytes) each, so a wave
// reads and writes whole contiguous 2 KB runs and nothing goes through LDS.  The lanes of a
// voxel add their partial logits with xor-shuffles, every lane then forms the softmax terms,
// its 16 values of da, and its share of dWh in 48 register accumulators.  Workgroup partials
// are merged in a fixed order.  da may be a itself: a lane writes the 32 bytes it has read, after
// reading them, and nobody else's (the clamped loads of lanes beyond the last voxel are not used).
template <int LPV>
__global__ __launch_bounds__(256) void head_stream_kernel(const bf16_t *a, const float *__restrict__ wh,
                                                         const float *__restrict__ bh,
                                                         const uint8_t *__restrict__ labels, bf16_t *da,
                                                         float *__restrict__ logits, float *__restrict__ partial,
                                                         int64_t V, float invV, int relu_mask, const float *__restrict__ cw)
{
    constexpr int C = 16 * LPV;
    const float cw0 = cw ? cw[0] : 1.f, cw1 = cw ? cw[1] : 1.f, cw2 = cw ? cw[2] : 1.f;
    constexpr int VPB = 256 / LPV;   // voxels per workgroup and step
    __shared__ float red[256 * 49];
    const int tid = threadIdx.x, sub = tid % LPV;
    float w0[16], w1[16], w2[16], g0[16], g1[16], g2[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        w0[i] = wh[(sub * 16 + i) * 3 + 0];
        w1[i] = wh[(sub * 16 + i) * 3 + 1];
        w2[i] = wh[(sub * 16 + i) * 3 + 2];
        g0[i] = g1[i] = g2[i] = 0.f;
    }
    const float b0 = bh ? bh[0] : 0.f, b1 = bh ? bh[1] : 0.f, b2 = bh ? bh[2] : 0.f;
    float lossacc = 0.f, db0 = 0.f, db1 = 0.f, db2 = 0.f;
    const int64_t nstep = (V + VPB - 1) / VPB;
    // The loads of the next step are requested before this step is computed: one 32-byte load
    // per thread and iteration leaves too few bytes in flight to cover the memory latency.
    auto voxel_of = [&](int64_t st) __attribute__((always_inline)) {
        const int64_t v = st * VPB + tid / LPV;
        return v < V ? v : V - 1;
    };
    uint4 n0 = make_uint4(0u, 0u, 0u, 0u), n1 = n0;
    int nlab = 0;
    if ((int64_t)blockIdx.x < nstep) {
        const int64_t vv = voxel_of(blockIdx.x);
        const uint4 *src = reinterpret_cast<const uint4 *>(a + vv * C + sub * 16);
        n0 = src[0];
        n1 = src[1];
        nlab = labels[vv];
    }
    for (int64_t st = blockIdx.x; st < nstep; st += gridDim.x) {
        const int64_t v = st * VPB + tid / LPV;
        const bool on = v < V;
        const uint4 r0 = n0, r1 = n1;
        const int lab = nlab;
        if (st + gridDim.x < nstep) {
            const int64_t vn = voxel_of(st + gridDim.x);
            const uint4 *src = reinterpret_cast<const uint4 *>(a + vn * C + sub * 16);
            n0 = src[0];
            n1 = src[1];
            nlab = labels[vn];
        }
        const uint32_t raw[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
        float av[16];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            av[2 * i] = __uint_as_float(raw[i] << 16);
            av[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
        }
        float z0 = 0.f, z1 = 0.f, z2 = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            z0 += av[i] * w0[i];
            z1 += av[i] * w1[i];
            z2 += av[i] * w2[i];
        }
#pragma unroll
        for (int m = 1; m < LPV; m <<= 1) {   // fixed pairing: the same sum in every lane of the voxel
            z0 += __shfl_xor(z0, m);
            z1 += __shfl_xor(z1, m);
            z2 += __shfl_xor(z2, m);
        }
        z0 += b0; z1 += b1; z2 += b2;
        const float mx = fmaxf(z0, fmaxf(z1, z2));
        const float e0 = expf(z0 - mx), e1 = expf(z1 - mx), e2 = expf(z2 - mx);
        const float den = e0 + e1 + e2, inv = 1.f / den;
        const float zl = lab == 0 ? z0 : (lab == 1 ? z1 : z2);
        const float wl = lab == 0 ? cw0 : (lab == 1 ? cw1 : cw2);   // class weight of this voxel
        const float sc = invV * wl;
        float d0 = (e0 * inv - (lab == 0 ? 1.f : 0.f)) * sc;
        float d1 = (e1 * inv - (lab == 1 ? 1.f : 0.f)) * sc;
        float d2 = (e2 * inv - (lab == 2 ? 1.f : 0.f)) * sc;
        if (!on) d0 = d1 = d2 = 0.f;
        if (on && sub == 0) {
            lossacc += wl * ((mx - zl) + logf(den));
            db0 += d0; db1 += d1; db2 += d2;
            if (logits) {
                float *lp = logits + v * 3;
                lp[0] = z0; lp[1] = z1; lp[2] = z2;
            }
        }
        uint32_t o[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float x0 = d0 * w0[2 * i] + d1 * w1[2 * i] + d2 * w2[2 * i];
            float x1 = d0 * w0[2 * i + 1] + d1 * w1[2 * i + 1] + d2 * w2[2 * i + 1];
            if (relu_mask && !(av[2 * i] > 0.f)) x0 = 0.f;
            if (relu_mask && !(av[2 * i + 1] > 0.f)) x1 = 0.f;
            o[i] = pack2bf(x0, x1);
        }
        if (on) {
            uint4 *dst = reinterpret_cast<uint4 *>(da + v * C + sub * 16);
            dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
            dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            g0[i] += av[i] * d0;
            g1[i] += av[i] * d1;
            g2[i] += av[i] * d2;
        }
    }
    // workgroup partials [C*3 dWh][3 dbh][1 loss]: thread values to LDS, then fixed-order column sums
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        red[tid * 49 + i * 3 + 0] = g0[i];
        red[tid * 49 + i * 3 + 1] = g1[i];
        red[tid * 49 + i * 3 + 2] = g2[i];
    }
    red[tid * 49 + 48] = 0.f;
    __syncthreads();
    float *out = partial + (int64_t)blockIdx.x * (C * 3 + 4);
    for (int e = tid; e < C * 3; e += 256) {
        const int c = e / 3, k = e - c * 3, sb = c / 16, i = c - sb * 16;
        float s = 0.f;
        for (int t = sb; t < 256; t += LPV) s += red[t * 49 + i * 3 + k];
        out[e] = s;
    }
    const float sc[4] = {db0, db1, db2, lossacc};
    for (int k = 0; k < 4; ++k) {
        __syncthreads();
        red[tid] = sc[k];
        __syncthreads();
        if (tid == 0) {
            float s = 0.f;
            for (int t = 0; t < 256; ++t) s += red[t];
            out[C * 3 + k] = s;
        }
    }
}

// One block per output element (C*3 weight gradients, 3 bias gradients, the loss): its 256
// threads add the workgroup partials in a fixed strided order, then a fixed tree.
__global__ __launch_bounds__(256) void head_reduce_kernel(const float *__restrict__ partial, int nblocks, int C,
                                                         float invV, float *__restrict__ dWh, float *__restrict__ dbh,
                                                         float *__restrict__ loss)
{
    __shared__ float red[256];
    const int cnt = C * 3 + 4, i = blockIdx.x, tid = threadIdx.x;
    float s = 0.f;
    for (int b = tid; b < nblocks; b += 256) s += partial[(int64_t)b * cnt + i];
    red[tid] = s;
    __syncthreads();
    for (int h = 128; h > 0; h >>= 1) {
        if (tid < h) red[tid] += red[tid + h];
        __syncthreads();
    }
    if (tid == 0) {
        const float r = red[0];
        if (i < C * 3) { if (dWh) dWh[i] = r; }
        else if (i < C * 3 + 3) { if (dbh) dbh[i - C * 3] = r; }
        else *loss = r * invV;
    }
}

static int head_blocks(int64_t V)
{
    int64_t nb = (V + HB - 1) / HB;
    return (int)(nb < 1024 ? nb : 1024);
}

}  // namespace k3

using namespace k3;

extern "C" int k3_head_workspace_bytes(const k3_tensor *ad, size_t *bytes)
{
    if (!desc_ok(ad) || !bytes) return K3_E_BADARG;
    *bytes = (size_t)head_blocks(voxels(ad)) * (size_t)(ad->c * 3 + 4) * sizeof(float);
    return K3_OK;
}

static int head_run(const k3_tensor *ad, const void *a, const float *wh, const float *bh, const uint8_t *labels,
                    const float *cw, float *loss, void *da, int relu_mask, float *dWh, float *dbh, float *logits, void *ws,
                    size_t ws_bytes, void *stream)
{
    size_t need = 0;
    int rc = k3_head_workspace_bytes(ad, &need);
    if (rc != K3_OK) return rc;
    if (!a || !wh || !labels || !loss || !da || !ws) return K3_E_BADARG;
    if (ws_bytes < need) return K3_E_WORKSPACE;
    int C = (int)ad->c;
    if (ad->c > 256 || (ad->dtype == K3_BF16 && C % 2 != 0)) return K3_E_UNSUPPORTED;
    int64_t V = voxels(ad);
    int nb = head_blocks(V);
    float invV = (float)(1.0 / (double)V);
    hipStream_t st = (hipStream_t)stream;
    size_t es = esize(ad->dtype);
    size_t lds = 2 * (size_t)HB * (C * es + 4) + HB * 4 * sizeof(float) + 256 * sizeof(float);
    if (lds > 160 * 1024) return K3_E_UNSUPPORTED;
    if (ad->dtype == K3_BF16 && (C == 16 || C == 32 || C == 64 || C == 128 || C == 256)) {
        const bf16_t *ap = (const bf16_t *)a;
        bf16_t *dp = (bf16_t *)da;
        float *pw = (float *)ws;
        const int rm = relu_mask ? 1 : 0;
        switch (C / 16) {
        case 1: head_stream_kernel<1><<<nb, 256, 0, st>>>(ap, wh, bh, labels, dp, logits, pw, V, invV, rm, cw); break;
        case 2: head_stream_kernel<2><<<nb, 256, 0, st>>>(ap, wh, bh, labels, dp, logits, pw, V, invV, rm, cw); break;
        case 4: head_stream_kernel<4><<<nb, 256, 0, st>>>(ap, wh, bh, labels, dp, logits, pw, V, invV, rm, cw); break;
        case 8: head_stream_kernel<8><<<nb, 256, 0, st>>>(ap, wh, bh, labels, dp, logits, pw, V, invV, rm, cw); break;
        default: head_stream_kernel<16><<<nb, 256, 0, st>>>(ap, wh, bh, labels, dp, logits, pw, V, invV, rm, cw); break;
        }
    } else if (ad->dtype == K3_BF16) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&head_kernel<bf16_t>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        head_kernel<bf16_t><<<nb, 256, lds, st>>>((const bf16_t *)a, wh, bh, labels, (bf16_t *)da, logits, (float *)ws, V, C, invV, relu_mask ? 1 : 0, cw);
    } else {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&head_kernel<float>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        head_kernel<float><<<nb, 256, lds, st>>>((const float *)a, wh, bh, labels, (float *)da, logits, (float *)ws, V, C, invV, relu_mask ? 1 : 0, cw);
    }
    K3_LAUNCH_CHECK();
    head_reduce_kernel<<<C * 3 + 4, 256, 0, st>>>((const float *)ws, nb, C, invV, dWh, dbh, loss);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

extern "C" int k3_head_softmax_ce_fwd_bwd(const k3_tensor *ad, const void *a, const float *wh, const float *bh,
                                          const uint8_t *labels, float *loss, void *da, int relu_mask, float *dWh,
                                          float *dbh, float *logits, void *ws, size_t ws_bytes, void *stream)
{
    return head_run(ad, a, wh, bh, labels, nullptr, loss, da, relu_mask, dWh, dbh, logits, ws, ws_bytes, stream);
}

extern "C" int k3_head_softmax_wce_fwd_bwd(const k3_tensor *ad, const void *a, const float *wh, const float *bh,
                                           const uint8_t *labels, const float *class_w, float *loss, void *da,
                                           int relu_mask, float *dWh, float *dbh, float *logits, void *ws,
                                           size_t ws_bytes, void *stream)
{
    if (!class_w) return K3_E_BADARG;
    return head_run(ad, a, wh, bh, labels, class_w, loss, da, relu_mask, dWh, dbh, logits, ws, ws_bytes, stream);
}

namespace k3 {

// Inference read-out: logits of the 1x1x1 head and the most likely class (lowest index on ties).
// LPV lanes share a voxel (16 channels each, 32-byte loads), as in head_stream_kernel.
template <int LPV>
__global__ __launch_bounds__(256) void head_classify_stream_kernel(const bf16_t *__restrict__ a, const float *__restrict__ wh,
                                                                  const float *__restrict__ bh, uint8_t *__restrict__ cls,
                                                                  float *__restrict__ logits, int64_t V)
{
    constexpr int C = 16 * LPV;
    constexpr int VPB = 256 / LPV;
    const int tid = threadIdx.x, sub = tid % LPV;
    float w0[16], w1[16], w2[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        w0[i] = wh[(sub * 16 + i) * 3 + 0];
        w1[i] = wh[(sub * 16 + i) * 3 + 1];
        w2[i] = wh[(sub * 16 + i) * 3 + 2];
    }
    const float b0 = bh ? bh[0] : 0.f, b1 = bh ? bh[1] : 0.f, b2 = bh ? bh[2] : 0.f;
    const int64_t nstep = (V + VPB - 1) / VPB;
    // The loads of the next step are requested before this step is computed: one 32-byte load
    // per thread and iteration leaves too few bytes in flight to cover the memory latency.
    auto voxel_of = [&](int64_t st) __attribute__((always_inline)) {
        const int64_t v = st * VPB + tid / LPV;
        return v < V ? v : V - 1;
    };
    uint4 n0 = make_uint4(0u, 0u, 0u, 0u), n1 = n0;
    if ((int64_t)blockIdx.x < nstep) {
        const int64_t vv = voxel_of(blockIdx.x);
        const uint4 *src = reinterpret_cast<const uint4 *>(a + vv * C + sub * 16);
        n0 = src[0];
        n1 = src[1];
    }
    for (int64_t st = blockIdx.x; st < nstep; st += gridDim.x) {
        const int64_t v = st * VPB + tid / LPV;
        const bool on = v < V;
        const uint4 r0 = n0, r1 = n1;
        if (st + gridDim.x < nstep) {
            const int64_t vn = voxel_of(st + gridDim.x);
            const uint4 *src = reinterpret_cast<const uint4 *>(a + vn * C + sub * 16);
            n0 = src[0];
            n1 = src[1];
        }
        const uint32_t raw[8] = {r0.x, r0.y, r0.z, r0.w, r1.x, r1.y, r1.z, r1.w};
        float z0 = 0.f, z1 = 0.f, z2 = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float lo = __uint_as_float(raw[i] << 16), hi = __uint_as_float(raw[i] & 0xffff0000u);
            z0 += lo * w0[2 * i]; z1 += lo * w1[2 * i]; z2 += lo * w2[2 * i];
            z0 += hi * w0[2 * i + 1]; z1 += hi * w1[2 * i + 1]; z2 += hi * w2[2 * i + 1];
        }
#pragma unroll
        for (int m = 1; m < LPV; m <<= 1) {
            z0 += __shfl_xor(z0, m);
            z1 += __shfl_xor(z1, m);
            z2 += __shfl_xor(z2, m);
        }
        z0 += b0; z1 += b1; z2 += b2;
        if (on && sub == 0) {
            cls[v] = (uint8_t)(z1 > z0 ? (z2 > z1 ? 2 : 1) : (z2 > z0 ? 2 : 0));
            if (logits) {
                float *lp = logits + v * 3;
                lp[0] = z0; lp[1] = z1; lp[2] = z2;
            }
        }
    }
}

// Any dtype / channel count: one thread per voxel.
template <typename T>
__global__ __launch_bounds__(256) void head_classify_kernel(const T *__restrict__ a, const float *__restrict__ wh,
                                                           const float *__restrict__ bh, uint8_t *__restrict__ cls,
                                                           float *__restrict__ logits, int64_t V, int C)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; v < V; v += stride) {
        const T *row = a + v * C;
        float z0 = bh ? bh[0] : 0.f, z1 = bh ? bh[1] : 0.f, z2 = bh ? bh[2] : 0.f;
        for (int c = 0; c < C; ++c) {
            const float av = elem<T>::ld(row + c);
            z0 += av * wh[c * 3 + 0];
            z1 += av * wh[c * 3 + 1];
            z2 += av * wh[c * 3 + 2];
        }
        cls[v] = (uint8_t)(z1 > z0 ? (z2 > z1 ? 2 : 1) : (z2 > z0 ? 2 : 0));
        if (logits) {
            float *lp = logits + v * 3;
            lp[0] = z0; lp[1] = z1; lp[2] = z2;
        }
    }
}

}  // namespace k3

extern "C" int k3_head_classify(const k3_tensor *ad, const void *a, const float *wh, const float *bh, uint8_t *classes,
                                float *logits, void *stream)
{
    if (!desc_ok(ad)) return K3_E_BADARG;
    if (!a || !wh || !classes) return K3_E_BADARG;
    const int C = (int)ad->c;
    if (ad->c > 4096) return K3_E_UNSUPPORTED;
    const int64_t V = voxels(ad);
    hipStream_t st = (hipStream_t)stream;
    if (ad->dtype == K3_BF16 && (C == 16 || C == 32 || C == 64 || C == 128 || C == 256)) {
        const int lpv = C / 16;
        const int64_t want = (V + 256 / lpv - 1) / (256 / lpv);
        const int nb = (int)(want < 4096 ? want : 4096);
        const bf16_t *ap = (const bf16_t *)a;
        switch (lpv) {
        case 1: head_classify_stream_kernel<1><<<nb, 256, 0, st>>>(ap, wh, bh, classes, logits, V); break;
        case 2: head_classify_stream_kernel<2><<<nb, 256, 0, st>>>(ap, wh, bh, classes, logits, V); break;
        case 4: head_classify_stream_kernel<4><<<nb, 256, 0, st>>>(ap, wh, bh, classes, logits, V); break;
        case 8: head_classify_stream_kernel<8><<<nb, 256, 0, st>>>(ap, wh, bh, classes, logits, V); break;
        default: head_classify_stream_kernel<16><<<nb, 256, 0, st>>>(ap, wh, bh, classes, logits, V); break;
        }
    } else {
        const int64_t want = (V + 255) / 256;
        const int nb = (int)(want < 4096 ? want : 4096);
        if (ad->dtype == K3_BF16)
            head_classify_kernel<bf16_t><<<nb, 256, 0, st>>>((const bf16_t *)a, wh, bh, classes, logits, V, C);
        else
            head_classify_kernel<float><<<nb, 256, 0, st>>>((const float *)a, wh, bh, classes, logits, V, C);
    }
    K3_LAUNCH_CHECK();
    return K3_OK;
}
