// Single-input-channel 3x3x3 convolution (the network's first layer) for gfx950, bf16:
// forward (+bias+ReLU) and backward-weight.  With C_in = 1 the contraction is only 27 long,
// so both passes are HBM-bound streams over the C_out-channel tensor (y, or dy and its ReLU
// mask); the input volume is tiny by comparison.
//
// A block stages the halo tile of the input in LDS; a thread owns 4 consecutive output channels
// and a strided set of the tile's voxels.  Forward keeps its 27 x 4 weights in registers;
// backward-weight keeps 27 x 4 accumulators over many tiles (persistent blocks), which are then
// added across the threads of a block through LDS in a fixed order and written as one partial
// per block (summed by the split-K reduction kernel).
#include "common.h"
#include "conv_internal.h"

namespace k3 {

namespace first {
constexpr int TD = 4, TH = 8, TW = 16;            // output voxels per tile
constexpr int HD = TD + 2, HH = TH + 2, HW = TW + 2;
constexpr int NHALO = HD * HH * HW;               // 1080 input voxels, kept as floats in LDS
constexpr int NVOX = TD * TH * TW;                // 512
constexpr int CPT = 4;                            // channels per thread
}  // namespace first

__device__ __forceinline__ void load4(const bf16_t *p, float *v)
{
    uint2 u = *reinterpret_cast<const uint2 *>(p);
    v[0] = __uint_as_float(u.x << 16);
    v[1] = __uint_as_float(u.x & 0xffff0000u);
    v[2] = __uint_as_float(u.y << 16);
    v[3] = __uint_as_float(u.y & 0xffff0000u);
}

struct FirstTile {
    int n, d0, h0, w0;
};
__device__ __forceinline__ FirstTile first_tile(int64_t tile, int ntd, int nth, int ntw)
{
    FirstTile t;
    t.w0 = (int)(tile % ntw) * first::TW;
    tile /= ntw;
    t.h0 = (int)(tile % nth) * first::TH;
    tile /= nth;
    t.d0 = (int)(tile % ntd) * first::TD;
    t.n = (int)(tile / ntd);
    return t;
}

// Stages the halo tile of the single-channel input in LDS as floats (zero outside the volume).
__device__ __forceinline__ void stage_x(const bf16_t *__restrict__ x, float *xs, const FirstTile &t, int D, int H, int W)
{
    using namespace first;
    for (int i = threadIdx.x; i < NHALO; i += 256) {
        int lw = i % HW, lh = (i / HW) % HH, ld = i / (HW * HH);
        int gd = t.d0 + ld - 1, gh = t.h0 + lh - 1, gw = t.w0 + lw - 1;
        float v = 0.f;
        if (gd >= 0 && gd < D && gh >= 0 && gh < H && gw >= 0 && gw < W)
            v = bf2f(x[(((int64_t)t.n * D + gd) * H + gh) * W + gw]);
        xs[i] = v;
    }
}

__global__ __launch_bounds__(256) void conv_first_fwd_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w,
                                                            const float *__restrict__ bias, int relu,
                                                            bf16_t *__restrict__ y, int D, int H, int W, int cout,
                                                            int ntd, int nth, int ntw)
{
    using namespace first;
    __shared__ float xs[NHALO];
    const int ng = cout / CPT;   // channel groups; divides 256
    const int cg = threadIdx.x % ng, vl = threadIdx.x / ng, nvl = 256 / ng;
    float wr[27][CPT], b[CPT];
#pragma unroll
    for (int t = 0; t < 27; ++t) load4(w + (int64_t)t * cout + cg * CPT, wr[t]);
#pragma unroll
    for (int i = 0; i < CPT; ++i) b[i] = bias ? bias[cg * CPT + i] : 0.f;
    const FirstTile t = first_tile(blockIdx.x, ntd, nth, ntw);
    stage_x(x, xs, t, D, H, W);
    __syncthreads();
    for (int v = vl; v < NVOX; v += nvl) {
        int lw = v % TW, lh = (v / TW) % TH, ld = v / (TW * TH);
        int gd = t.d0 + ld, gh = t.h0 + lh, gw = t.w0 + lw;
        if (gd >= D || gh >= H || gw >= W) continue;
        const float *c = xs + (ld * HH + lh) * HW + lw;
        float acc[CPT];
#pragma unroll
        for (int i = 0; i < CPT; ++i) acc[i] = b[i];
#pragma unroll
        for (int tp = 0; tp < 27; ++tp) {
            float xv = c[((tp / 9) * HH + (tp / 3) % 3) * HW + tp % 3];
#pragma unroll
            for (int i = 0; i < CPT; ++i) acc[i] += xv * wr[tp][i];
        }
        if (relu) {
#pragma unroll
            for (int i = 0; i < CPT; ++i) acc[i] = acc[i] > 0.f ? acc[i] : 0.f;
        }
        int64_t vox = (((int64_t)t.n * D + gd) * H + gh) * W + gw;
        *reinterpret_cast<uint2 *>(y + vox * cout + cg * CPT) = make_uint2(pack2bf(acc[0], acc[1]), pack2bf(acc[2], acc[3]));
    }
}

// Persistent blocks: block s walks tiles s, s + gridDim.x, ... and keeps 27 x CPT (+ CPT bias) sums.
__global__ __launch_bounds__(256) void conv_first_wgrad_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy,
                                                              const bf16_t *__restrict__ mask, float *__restrict__ ws,
                                                              int64_t per_split, int D, int H, int W, int cout, int ntd,
                                                              int nth, int ntw, int64_t ntiles)
{
    using namespace first;
    __shared__ float xs[NHALO];
    __shared__ float red[256][CPT + 1];
    const int ng = cout / CPT;
    const int cg = threadIdx.x % ng, vl = threadIdx.x / ng, nvl = 256 / ng;
    float acc[27][CPT], accb[CPT];
#pragma unroll
    for (int t = 0; t < 27; ++t)
#pragma unroll
        for (int i = 0; i < CPT; ++i) acc[t][i] = 0.f;
#pragma unroll
    for (int i = 0; i < CPT; ++i) accb[i] = 0.f;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const FirstTile t = first_tile(tile, ntd, nth, ntw);
        __syncthreads();
        stage_x(x, xs, t, D, H, W);
        __syncthreads();
        for (int v = vl; v < NVOX; v += nvl) {
            int lw = v % TW, lh = (v / TW) % TH, ld = v / (TW * TH);
            int gd = t.d0 + ld, gh = t.h0 + lh, gw = t.w0 + lw;
            if (gd >= D || gh >= H || gw >= W) continue;
            int64_t vox = (((int64_t)t.n * D + gd) * H + gh) * W + gw;
            float g[CPT];
            load4(dy + vox * cout + cg * CPT, g);
            if (mask) {
                float m[CPT];
                load4(mask + vox * cout + cg * CPT, m);
#pragma unroll
                for (int i = 0; i < CPT; ++i) g[i] = m[i] > 0.f ? g[i] : 0.f;
            }
            const float *c = xs + (ld * HH + lh) * HW + lw;
#pragma unroll
            for (int i = 0; i < CPT; ++i) accb[i] += g[i];
#pragma unroll
            for (int tp = 0; tp < 27; ++tp) {
                float xv = c[((tp / 9) * HH + (tp / 3) % 3) * HW + tp % 3];
#pragma unroll
                for (int i = 0; i < CPT; ++i) acc[tp][i] += xv * g[i];
            }
        }
    }
    // add the nvl voxel lanes of each channel group in lane order; thread co writes channel co
    float *out = ws + (int64_t)blockIdx.x * per_split;
#pragma unroll
    for (int t = 0; t < 28; ++t) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < CPT; ++i) red[threadIdx.x][i] = t < 27 ? acc[t < 27 ? t : 0][i] : accb[i];
        __syncthreads();
        if (threadIdx.x < cout) {
            int g2 = threadIdx.x / CPT, i = threadIdx.x % CPT;
            float s = 0.f;
            for (int k = 0; k < nvl; ++k) s += red[k * ng + g2][i];
            out[(int64_t)t * cout + threadIdx.x] = s;   // t == 27 is the bias-gradient row
        }
    }
}

bool conv_first_ok(int dtype, int64_t c1, int64_t c2, int64_t cout)
{
    return dtype == K3_BF16 && c1 == 1 && c2 == 0 && cout % first::CPT == 0 && cout <= 256 &&
           256 % (cout / first::CPT) == 0;
}

static int64_t first_tiles(const ConvArgs &a, int *ntd, int *nth, int *ntw)
{
    *ntd = (int)((a.D + first::TD - 1) / first::TD);
    *nth = (int)((a.H + first::TH - 1) / first::TH);
    *ntw = (int)((a.W + first::TW - 1) / first::TW);
    return a.N * *ntd * *nth * *ntw;
}

int conv_first_fwd(const ConvArgs &a, hipStream_t st)
{
    int ntd, nth, ntw;
    int64_t ntiles = first_tiles(a, &ntd, &nth, &ntw);
    if (ntiles > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    conv_first_fwd_kernel<<<dim3((unsigned)ntiles), 256, 0, st>>>((const bf16_t *)a.x, (const bf16_t *)a.w, a.bias, a.relu,
                                                                  (bf16_t *)a.y, (int)a.D, (int)a.H, (int)a.W, (int)a.cout,
                                                                  ntd, nth, ntw);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

static int64_t first_nsplit(int64_t ntiles) { return ntiles < 2048 ? ntiles : 2048; }

size_t conv_first_wgrad_ws_bytes(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cout)
{
    int64_t ntiles = N * ((D + first::TD - 1) / first::TD) * ((H + first::TH - 1) / first::TH) *
                     ((W + first::TW - 1) / first::TW);
    return (size_t)first_nsplit(ntiles) * 28 * cout * sizeof(float);
}

int conv_first_wgrad(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st)
{
    int ntd, nth, ntw;
    int64_t ntiles = first_tiles(a, &ntd, &nth, &ntw);
    int64_t nsplit = first_nsplit(ntiles);
    int64_t per = 28 * a.cout;   // 27 tap rows + the bias row: canonical [27][1][cout] followed by db
    conv_first_wgrad_kernel<<<dim3((unsigned)nsplit), 256, 0, st>>>((const bf16_t *)a.x, (const bf16_t *)a.dy,
                                                                    (const bf16_t *)a.ymask, ws, per, (int)a.D, (int)a.H,
                                                                    (int)a.W, (int)a.cout, ntd, nth, ntw, ntiles);
    K3_LAUNCH_CHECK();
    return launch_reduce_partials(ws, dW, db, 27 * a.cout, per, (int)nsplit, st);
}

}  // namespace k3
