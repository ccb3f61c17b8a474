// bf16 MFMA kernel for the 3x3x3 convolution backward-weight pass on gfx950.
//
// GEMM view: dW[tap][ci][co] = sum_v X[ci][v + off_tap] * G[v][co], so the contraction runs
// over voxels while both tensors are stored channel-fastest.  The tiles are staged in LDS
// exactly as they lie in memory ([voxel][channel]) and the MFMA operands (8 consecutive
// voxels of one channel per lane) are produced by the transposing LDS read
// ds_read_b64_tr_b16: within 16 lanes, lane j supplies the address of 4 channels of voxel
// j/4 (channel group j%4) and lane i receives channel i of the 4 voxels.
//
// A workgroup owns one 32-channel block of x, 32*COBN channels of g and a strided set of
// 4x8x8-voxel tiles; its 4 waves split the 27 taps (7,7,7,6) and the last wave also
// multiplies g by a vector of ones, which yields the bias gradient.  Each workgroup
// writes its partial sums to the workspace; a second kernel adds the partials in a fixed
// order (no atomics, run-to-run identical).
#include "common.h"
#include "conv_internal.h"

namespace k3 {

struct WgradParams {
    const bf16_t *x1, *x2;
    int c1, c2;
    const bf16_t *dy, *mask;
    int cout;
    float *ws;
    int64_t per_split;  // floats per split: 27*cin*cout + cout
    int N, D, H, W;
    int ntd, nth, ntw;
    int64_t ntiles;
    int nsplit;
};

namespace wg {
constexpr int TD = 4, TH = 8, TW = 8;
constexpr int HD = TD + 2, HH = TH + 2, HW = TW + 2;
constexpr int NHALO = HD * HH * HW;   // 600
constexpr int NVOX = TD * TH * TW;    // 256
constexpr int XS_BYTES = NHALO * 64;  // 32 channels, unpadded: 4 consecutive voxels span all 64 banks
constexpr int GS_PLANE = NVOX * 64;
}  // namespace wg

__device__ __forceinline__ bf16x8 tr_pair(const unsigned char *base, int off0, int off1)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(base + off0));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(base + off1));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ uint32_t wg_mask_pair(uint32_t v, uint32_t m)
{
    uint32_t lo = ((m & 0x8000u) == 0 && (m & 0x7fffu) != 0) ? 0x0000ffffu : 0u;
    uint32_t hi = ((m & 0x80000000u) == 0 && (m & 0x7fff0000u) != 0) ? 0xffff0000u : 0u;
    return v & (lo | hi);
}

template <int COBN>
__global__ __launch_bounds__(256) void conv_wgrad_mfma_kernel(WgradParams p)
{
    using namespace wg;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *xs = smem;
    unsigned char *gs = smem + XS_BYTES;  // [COBN][NVOX][32 ch]
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int hb = lane >> 5, blk = lane >> 4, j = lane & 15;
    const int cib = blockIdx.y, cob0 = blockIdx.z * COBN;
    const int cin = p.c1 + p.c2;
    const bool first = cib * 32 < p.c1;
    const bf16_t *xsrc = first ? p.x1 : p.x2;
    const int Cx = first ? p.c1 : p.c2;
    const int chx = first ? cib * 32 : cib * 32 - p.c1;

    // lane-constant parts of the transposing-read addresses
    const int lane_x = (hb * HW + (j >> 2)) * 64 + (blk & 1) * 32 + (j & 3) * 8;
    const int lane_g = (hb * TW + (j >> 2)) * 64 + (blk & 1) * 32 + (j & 3) * 8;
    int xoff[7];
#pragma unroll
    for (int t = 0; t < 7; ++t) {
        int tap = wv * 7 + t;
        if (tap > 26) tap = 26;  // slot of the ones-vector (bias) product; address unused
        xoff[t] = lane_x + (((tap / 9) * HH + (tap / 3) % 3) * HW + tap % 3) * 64;
    }

    f32x16 acc[7][COBN];
#pragma unroll
    for (int t = 0; t < 7; ++t)
#pragma unroll
        for (int c = 0; c < COBN; ++c)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][c][i] = 0.f;

    bf16x8 ones;
#pragma unroll
    for (int i = 0; i < 8; ++i) ones[i] = (__bf16)1.0f;

    for (int64_t tile = blockIdx.x; tile < p.ntiles; tile += p.nsplit) {
        int64_t q = tile;
        const int twi = (int)(q % p.ntw);
        q /= p.ntw;
        const int thi = (int)(q % p.nth);
        q /= p.nth;
        const int tdi = (int)(q % p.ntd);
        const int n = (int)(q / p.ntd);
        const int d0 = tdi * TD, h0 = thi * TH, w0 = twi * TW;
        __syncthreads();
        for (int i = tid; i < NHALO * 4; i += 256) {
            int vox = i >> 2, part = i & 3;
            int lw = vox % HW, lh = (vox / HW) % HH, ld = vox / (HW * HH);
            int gd = d0 + ld - 1, gh = h0 + lh - 1, gw = w0 + lw - 1;
            uint4 val = make_uint4(0, 0, 0, 0);
            if (gd >= 0 && gd < p.D && gh >= 0 && gh < p.H && gw >= 0 && gw < p.W) {
                int64_t g = ((((int64_t)n * p.D + gd) * p.H + gh) * p.W + gw) * Cx + chx + part * 8;
                val = *reinterpret_cast<const uint4 *>(xsrc + g);
            }
            *reinterpret_cast<uint4 *>(xs + vox * 64 + part * 16) = val;
        }
        for (int i = tid; i < NVOX * COBN * 4; i += 256) {
            int part = i & 3, cb = (i >> 2) % COBN, vox = i / (4 * COBN);
            int lw = vox % TW, lh = (vox / TW) % TH, ld = vox / (TW * TH);
            int gd = d0 + ld, gh = h0 + lh, gw = w0 + lw;
            uint4 val = make_uint4(0, 0, 0, 0);
            if (gd < p.D && gh < p.H && gw < p.W) {
                int64_t g = ((((int64_t)n * p.D + gd) * p.H + gh) * p.W + gw) * p.cout + (cob0 + cb) * 32 + part * 8;
                val = *reinterpret_cast<const uint4 *>(p.dy + g);
                if (p.mask) {
                    uint4 m = *reinterpret_cast<const uint4 *>(p.mask + g);
                    val.x = wg_mask_pair(val.x, m.x);
                    val.y = wg_mask_pair(val.y, m.y);
                    val.z = wg_mask_pair(val.z, m.z);
                    val.w = wg_mask_pair(val.w, m.w);
                }
            }
            *reinterpret_cast<uint4 *>(gs + cb * GS_PLANE + vox * 64 + part * 16) = val;
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < NVOX / 16; ++s) {
            // K-step s: voxels (d = s/4, h = 2*(s%4) + hb, w = 0..7); k-slot e of read r is w = 4r + e
            const int sx = (((s >> 2) * HH + 2 * (s & 3)) * HW) * 64;
            const int sg = (((s >> 2) * TH + 2 * (s & 3)) * TW) * 64;
            bf16x8 bg[COBN];
#pragma unroll
            for (int c = 0; c < COBN; ++c) bg[c] = tr_pair(gs + c * GS_PLANE, lane_g + sg, lane_g + sg + 4 * 64);
#pragma unroll
            for (int t = 0; t < 7; ++t) {
                bf16x8 ax;
                if (wv == 3 && t == 6) ax = ones;
                else ax = tr_pair(xs, xoff[t] + sx, xoff[t] + sx + 4 * 64);
#pragma unroll
                for (int c = 0; c < COBN; ++c) acc[t][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax, bg[c], acc[t][c], 0, 0, 0);
            }
        }
    }

    float *out = p.ws + (int64_t)blockIdx.x * p.per_split;
#pragma unroll
    for (int t = 0; t < 7; ++t) {
        const int tap = wv * 7 + t;
#pragma unroll
        for (int c = 0; c < COBN; ++c) {
            const int co = (cob0 + c) * 32 + (lane & 31);
            if (tap <= 26) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    int ci = cib * 32 + (i >> 2) * 8 + hb * 4 + (i & 3);
                    out[((int64_t)tap * cin + ci) * p.cout + co] = acc[t][c][i];
                }
            } else if (cib == 0 && hb == 0) {
                out[(int64_t)27 * cin * p.cout + co] = acc[t][c][0];  // row 0 of ones^T * g
            }
        }
    }
}

static void wgrad_plan(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout, int *cobn,
                       int64_t *ntiles, int *nsplit)
{
    *cobn = (cout % 64 == 0) ? 2 : 1;
    *ntiles = N * ((D + wg::TD - 1) / wg::TD) * ((H + wg::TH - 1) / wg::TH) * ((W + wg::TW - 1) / wg::TW);
    // about two resident workgroups per CU in total, and at least four tiles per workgroup so the
    // partial-sum traffic stays small next to the tensor reads
    int64_t yz = (cin / 32) * (cout / (32 * *cobn));
    int64_t s = 512 / yz;
    if (s > *ntiles / 4) s = *ntiles / 4;
    if (s < 1) s = 1;
    *nsplit = (int)s;
}

size_t conv_wgrad_mfma_ws_bytes(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout)
{
    // either kernel may run (the pipelined one takes no ReLU mask): size for both
    const size_t a = conv_wgrad_mfma_ws_bytes_for(N, D, H, W, cin, cout, true);
    const size_t b = conv_wgrad_mfma_ws_bytes_for(N, D, H, W, cin, cout, false);
    return a > b ? a : b;
}

// What the kernel that conv_wgrad_mfma picks for a call with / without a ReLU mask writes.
size_t conv_wgrad_mfma_ws_bytes_for(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout, bool masked)
{
    if (!masked && conv_wgrad_pipe_ok(N, D, H, W, cin, cout)) return conv_wgrad_pipe_ws_bytes(N, D, H, W, cin, cout);
    int cobn, nsplit;
    int64_t ntiles;
    wgrad_plan(N, D, H, W, cin, cout, &cobn, &ntiles, &nsplit);
    return (size_t)nsplit * (size_t)(27 * cin * cout + cout) * sizeof(float);
}

template <int COBN>
static int launch_wgrad(const WgradParams &p, dim3 grid, hipStream_t st)
{
    constexpr int lds = wg::XS_BYTES + COBN * wg::GS_PLANE;
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_wgrad_mfma_kernel<COBN>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    conv_wgrad_mfma_kernel<COBN><<<grid, 256, lds, st>>>(p);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

int conv_wgrad_mfma(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st)
{
    WgradParams p{};
    int64_t cin = a.c1 + a.c2;
    if (!a.ymask && conv_wgrad_pipe_ok(a.N, a.D, a.H, a.W, cin, a.cout)) return conv_wgrad_pipe(a, dW, db, ws, st);
    int cobn;
    wgrad_plan(a.N, a.D, a.H, a.W, cin, a.cout, &cobn, &p.ntiles, &p.nsplit);
    p.x1 = (const bf16_t *)a.x;
    p.x2 = (const bf16_t *)a.x2;
    p.c1 = (int)a.c1;
    p.c2 = (int)a.c2;
    p.dy = (const bf16_t *)a.dy;
    p.mask = (const bf16_t *)a.ymask;
    p.cout = (int)a.cout;
    p.ws = ws;
    p.per_split = 27 * cin * a.cout + a.cout;
    p.N = (int)a.N; p.D = (int)a.D; p.H = (int)a.H; p.W = (int)a.W;
    p.ntd = (int)((a.D + wg::TD - 1) / wg::TD);
    p.nth = (int)((a.H + wg::TH - 1) / wg::TH);
    p.ntw = (int)((a.W + wg::TW - 1) / wg::TW);
    dim3 grid((unsigned)p.nsplit, (unsigned)(cin / 32), (unsigned)(a.cout / (32 * cobn)));
    int rc = cobn == 2 ? launch_wgrad<2>(p, grid, st) : launch_wgrad<1>(p, grid, st);
    if (rc != K3_OK) return rc;
    return launch_reduce_partials(ws, dW, db, 27 * cin * a.cout, p.per_split, p.nsplit, st);
}

}  // namespace k3
