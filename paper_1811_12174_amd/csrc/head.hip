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

template <typename T>
__global__ __launch_bounds__(256) void head_kernel(const T *__restrict__ a, const float *__restrict__ wh,
                                                  const float *__restrict__ bh, const uint8_t *__restrict__ labels,
                                                  T *__restrict__ da, float *__restrict__ logits,
                                                  float *__restrict__ partial, int64_t V, int C, float invV, int relu_mask)
{
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
            lossacc += (m - zl) + logf(den);
            float d0 = (e0 * inv - (lab == 0 ? 1.f : 0.f)) * invV;
            float d1 = (e1 * inv - (lab == 1 ? 1.f : 0.f)) * invV;
            float d2 = (e2 * inv - (lab == 2 ? 1.f : 0.f)) * invV;
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

__global__ __launch_bounds__(256) void head_reduce_kernel(const float *__restrict__ partial, int nblocks, int C,
                                                         float invV, float *__restrict__ dWh, float *__restrict__ dbh,
                                                         float *__restrict__ loss)
{
    int cnt = C * 3 + 4;
    for (int i = threadIdx.x; i < cnt; i += 256) {
        float s = 0.f;
        for (int b = 0; b < nblocks; ++b) s += partial[(int64_t)b * cnt + i];
        if (i < C * 3) { if (dWh) dWh[i] = s; }
        else if (i < C * 3 + 3) { if (dbh) dbh[i - C * 3] = s; }
        else *loss = s * invV;
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

extern "C" int k3_head_softmax_ce_fwd_bwd(const k3_tensor *ad, const void *a, const float *wh, const float *bh,
                                          const uint8_t *labels, float *loss, void *da, int relu_mask, float *dWh,
                                          float *dbh, float *logits, void *ws, size_t ws_bytes, void *stream)
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
    if (ad->dtype == K3_BF16) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&head_kernel<bf16_t>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        head_kernel<bf16_t><<<nb, 256, lds, st>>>((const bf16_t *)a, wh, bh, labels, (bf16_t *)da, logits, (float *)ws, V, C, invV, relu_mask ? 1 : 0);
    } else {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&head_kernel<float>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        head_kernel<float><<<nb, 256, lds, st>>>((const float *)a, wh, bh, labels, (float *)da, logits, (float *)ws, V, C, invV, relu_mask ? 1 : 0);
    }
    K3_LAUNCH_CHECK();
    head_reduce_kernel<<<1, 256, 0, st>>>((const float *)ws, nb, C, invV, dWh, dbh, loss);
    K3_LAUNCH_CHECK();
    return K3_OK;
}
