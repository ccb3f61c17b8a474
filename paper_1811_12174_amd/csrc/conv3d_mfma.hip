// bf16 MFMA implicit-GEMM kernels for the 3x3x3 convolution forward and backward-data
// passes on gfx950 (CDNA4, wave64).
//
// GEMM view: D[co][voxel] = sum_{tap, ci} Wp[co][tap, ci] * X[tap, ci][voxel], so the
// weights are the MFMA "A" operand (rows = output channels) and the activations the "B"
// operand (columns = voxels).  With v_mfma_f32_32x32x16_bf16 a lane then owns, for one
// voxel, 16 output channels; the packed weight rows are permuted so that these 16 are
// consecutive and the epilogue writes 32 contiguous bytes per lane.
//
// A workgroup (4 waves) owns a TD x TH x TW block of output voxels and 32*MB output
// channels.  Per 16-channel input chunk it stages the halo tile of the input (zero
// filled outside the volume, and multiplied by the ReLU mask in the backward pass) and a
// group of weight taps in LDS; each wave multiplies its 32-voxel patches by all taps.
// Backward-data is the same kernel run on dy with the taps mirrored and the channel roles
// swapped (done once, when the weights are packed).
#include "common.h"
#include "conv_internal.h"

namespace k3 {

// acc index i of lane half hb maps to MFMA row (i/4)*8 + hb*4 + i%4; row r therefore
// carries channel (r/4%2)*16 + (r/8)*4 + r%4 of its 32-channel block.
__host__ __device__ static inline int row_to_channel(int r) { return ((r >> 2) & 1) * 16 + (r >> 3) * 4 + (r & 3); }

// ---------------------------------------------------------------------------- packing
// packed = [fwd form | bwd form], each 27*cin*cout bf16:
//   fwd[cob][tap][kc][lane][j] = W[tap][kc*16 + (lane/32)*8 + j][cob*32 + row_to_channel(lane%32)]
//   bwd[cib][tap][kc][lane][j] = W[26-tap][cib*32 + row_to_channel(lane%32)][kc*16 + (lane/32)*8 + j]
__global__ __launch_bounds__(256) void pack_weights_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ packed,
                                                          int cin, int cout)
{
    int64_t per = (int64_t)27 * cin * cout;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= 2 * per) return;
    bool bwd = i >= per;
    int64_t r = bwd ? i - per : i;
    int j = (int)(r & 7);
    int lane = (int)((r >> 3) & 63);
    int64_t q = r >> 9;
    int K = bwd ? cout : cin;  // contraction channels
    int nkc = K / 16;
    int kc = (int)(q % nkc);
    q /= nkc;
    int tap = (int)(q % 27);
    int mblk = (int)(q / 27);
    int kch = kc * 16 + (lane >> 5) * 8 + j;
    int mch = mblk * 32 + row_to_channel(lane & 31);
    bf16_t v;
    if (!bwd) v = w[((int64_t)tap * cin + kch) * cout + mch];
    else v = w[((int64_t)(26 - tap) * cin + mch) * cout + kch];
    packed[i] = v;
}

size_t conv_packed_bytes(int64_t cin, int64_t cout) { return (size_t)2 * 27 * cin * cout * sizeof(bf16_t); }

int conv_pack_weights(const void *w, int64_t cin, int64_t cout, void *packed, hipStream_t st)
{
    int64_t total = 2 * 27 * cin * cout;
    pack_weights_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, st>>>((const bf16_t *)w, (bf16_t *)packed,
                                                                               (int)cin, (int)cout);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

// ---------------------------------------------------------------------------- kernel
struct MfmaParams {
    const bf16_t *src1, *src2, *mask;  // mask applies to src1 (src2 is null whenever mask is set)
    int c1, c2;                        // contraction channels per source
    const bf16_t *packed;              // [mblk][27][nkc][64][8]
    const float *bias;
    int relu;
    bf16_t *dst1, *dst2;
    int cd1, cd2;                      // output channels per destination
    int N, D, H, W;
    int ntd, nth, ntw;                 // tiles per axis
    int ncg;                           // output-channel groups (of 32*MB)
    int64_t total, per_xcd;            // logical blocks, and blocks per XCD slice
};

template <int TD_, int TH_, int TW_, int MB_, int TAPS_>
struct TileCfg {
    static constexpr int TD = TD_, TH = TH_, TW = TW_, MB = MB_, TAPS = TAPS_;
    static constexpr int CK = 16;
    static constexpr int HD = TD + 2, HH = TH + 2, HW = TW + 2;
    static constexpr int NHALO = HD * HH * HW;
    // LDS tile: 32 bytes per voxel (16 channels), rows of HW voxels padded by one 16-byte slot.
    // A ds_read_b128 serves 16 lanes per cycle = two 8-voxel rows of a patch; voxels of one row
    // land on the even 16-byte slots and, thanks to the odd row pitch, the next row on the odd
    // ones, so the 16 lanes cover all 64 banks exactly once.
    static constexpr int XS_VOX = CK * 2;
    static constexpr int XS_ROW = HW * XS_VOX + 16;
    static constexpr int XS_PLANE = HH * XS_ROW;
    static constexpr int XS_BYTES = HD * XS_PLANE;
    static constexpr int WS_BYTES = TAPS * MB * 1024;
    static constexpr int LDS_BYTES = XS_BYTES + WS_BYTES;
    static constexpr int PW = TW / 8, PH = TH / 4;  // 4x8 (h x w) voxel patches per plane
    static constexpr int NBLK = TD * PH * PW;
    static constexpr int NBW = NBLK / 4;             // patches per wave
    static_assert(TW % 8 == 0 && TH % 4 == 0 && NBLK % 4 == 0, "tile must split into 4x8 patches over 4 waves");
    static_assert(27 % TAPS == 0, "tap groups must divide 27");
};

__device__ __forceinline__ uint32_t mask_pair(uint32_t v, uint32_t m)
{
    // keep each bf16 half of v where the matching half of m is > 0 (sign clear and nonzero)
    uint32_t lo = ((m & 0x8000u) == 0 && (m & 0x7fffu) != 0) ? 0x0000ffffu : 0u;
    uint32_t hi = ((m & 0x80000000u) == 0 && (m & 0x7fff0000u) != 0) ? 0xffff0000u : 0u;
    return v & (lo | hi);
}

template <class C>
__global__ __launch_bounds__(256, 2) void conv_mfma_kernel(MfmaParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *xs = smem;
    unsigned char *wsm = smem + C::XS_BYTES;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int hb = lane >> 5, vl = lane & 31;

    // XCD-aware block order: hardware deals consecutive block ids round-robin to the 8
    // XCDs, so slice the logical order into 8 contiguous runs, one per XCD, to keep
    // neighbouring tiles (shared halos) and the channel groups of one tile in one L2.
    const int64_t logical = (int64_t)(blockIdx.x & 7) * p.per_xcd + (blockIdx.x >> 3);
    if (logical >= p.total) return;
    const int cg = (int)(logical % p.ncg);
    int64_t tile = logical / p.ncg;
    const int twi = (int)(tile % p.ntw);
    tile /= p.ntw;
    const int thi = (int)(tile % p.nth);
    tile /= p.nth;
    const int tdi = (int)(tile % p.ntd);
    const int n = (int)(tile / p.ntd);
    const int d0 = tdi * C::TD, h0 = thi * C::TH, w0 = twi * C::TW;
    const int mb0 = cg * C::MB;
    const int nkc = (p.c1 + p.c2) / 16;

    f32x16 acc[C::NBW][C::MB];
#pragma unroll
    for (int a = 0; a < C::NBW; ++a)
#pragma unroll
        for (int b = 0; b < C::MB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // LDS byte offset (tap 0,0,0 corner, this lane's channel half) of the lane's voxel in each patch
    int vbase[C::NBW];
#pragma unroll
    for (int a = 0; a < C::NBW; ++a) {
        int nb = wv * C::NBW + a;
        int bw = nb % C::PW, bh = (nb / C::PW) % C::PH, bd = nb / (C::PW * C::PH);
        vbase[a] = bd * C::XS_PLANE + (bh * 4 + (vl >> 3)) * C::XS_ROW + (bw * 8 + (vl & 7)) * C::XS_VOX + hb * 16;
    }

    for (int c = 0; c < nkc; ++c) {
        const int ch0 = c * 16;
        const bool first = ch0 < p.c1;
        const bf16_t *src = first ? p.src1 : p.src2;
        const bf16_t *msk = first ? p.mask : nullptr;
        const int Csrc = first ? p.c1 : p.c2;
        const int chs = first ? ch0 : ch0 - p.c1;
        __syncthreads();  // everyone finished reading the previous chunk
        for (int i = tid; i < C::NHALO * 2; i += 256) {
            int vox = i >> 1, half = i & 1;
            int lw = vox % C::HW, lh = (vox / C::HW) % C::HH, ld = vox / (C::HW * C::HH);
            int gd = d0 + ld - 1, gh = h0 + lh - 1, gw = w0 + lw - 1;
            uint4 val = make_uint4(0, 0, 0, 0);
            if (gd >= 0 && gd < p.D && gh >= 0 && gh < p.H && gw >= 0 && gw < p.W) {
                int64_t g = ((((int64_t)n * p.D + gd) * p.H + gh) * p.W + gw) * Csrc + chs + half * 8;
                val = *reinterpret_cast<const uint4 *>(src + g);
                if (msk) {
                    uint4 m = *reinterpret_cast<const uint4 *>(msk + g);
                    val.x = mask_pair(val.x, m.x);
                    val.y = mask_pair(val.y, m.y);
                    val.z = mask_pair(val.z, m.z);
                    val.w = mask_pair(val.w, m.w);
                }
            }
            *reinterpret_cast<uint4 *>(xs + ld * C::XS_PLANE + lh * C::XS_ROW + lw * C::XS_VOX + half * 16) = val;
        }
        for (int g = 0; g < 27 / C::TAPS; ++g) {
            if (g > 0) __syncthreads();  // previous tap group consumed
            for (int i = tid; i < C::TAPS * C::MB * 64; i += 256) {
                int ln = i & 63, mb = (i >> 6) % C::MB, tl = i / (64 * C::MB);
                int tap = g * C::TAPS + tl;
                const uint4 *s = reinterpret_cast<const uint4 *>(p.packed) +
                                 ((((int64_t)(mb0 + mb) * 27 + tap) * nkc + c) * 64 + ln);
                *reinterpret_cast<uint4 *>(wsm + ((tl * C::MB + mb) * 64 + ln) * 16) = *s;
            }
            __syncthreads();
            const int goff = (C::TAPS == 27) ? 0 : g * (C::TAPS / 9) * C::XS_PLANE;
#pragma unroll
            for (int tl = 0; tl < C::TAPS; ++tl) {
                const int toff = (tl / 9) * C::XS_PLANE + ((tl / 3) % 3) * C::XS_ROW + (tl % 3) * C::XS_VOX;
                bf16x8 a[C::MB];
#pragma unroll
                for (int mb = 0; mb < C::MB; ++mb)
                    a[mb] = *reinterpret_cast<const bf16x8 *>(wsm + ((tl * C::MB + mb) * 64 + lane) * 16);
#pragma unroll
                for (int nb = 0; nb < C::NBW; ++nb) {
                    bf16x8 b = *reinterpret_cast<const bf16x8 *>(xs + vbase[nb] + goff + toff);
#pragma unroll
                    for (int mb = 0; mb < C::MB; ++mb)
                        acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mb], b, acc[nb][mb], 0, 0, 0);
                }
            }
        }
    }

    // epilogue: bias, ReLU, round to bf16, 32 contiguous bytes per lane and channel block
#pragma unroll
    for (int nb = 0; nb < C::NBW; ++nb) {
        int blk = wv * C::NBW + nb;
        int bw = blk % C::PW, bh = (blk / C::PW) % C::PH, bd = blk / (C::PW * C::PH);
        int gd = d0 + bd, gh = h0 + bh * 4 + (vl >> 3), gw = w0 + bw * 8 + (vl & 7);
        if (gd >= p.D || gh >= p.H || gw >= p.W) continue;
        int64_t vox = (((int64_t)n * p.D + gd) * p.H + gh) * p.W + gw;
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) {
            int co0 = (mb0 + mb) * 32 + hb * 16;
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float t = acc[nb][mb][i] + (p.bias ? p.bias[co0 + i] : 0.f);
                v[i] = (p.relu && !(t > 0.f)) ? 0.f : t;
            }
            bf16_t *dst = co0 < p.cd1 ? p.dst1 + vox * p.cd1 + co0 : p.dst2 + vox * p.cd2 + (co0 - p.cd1);
            uint4 o0 = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
            uint4 o1 = make_uint4(pack2bf(v[8], v[9]), pack2bf(v[10], v[11]), pack2bf(v[12], v[13]), pack2bf(v[14], v[15]));
            reinterpret_cast<uint4 *>(dst)[0] = o0;
            reinterpret_cast<uint4 *>(dst)[1] = o1;
        }
    }
}

template <class C>
static int launch_cfg(MfmaParams p, int64_t mblocks, hipStream_t st)
{
    p.ntd = (p.D + C::TD - 1) / C::TD;
    p.nth = (p.H + C::TH - 1) / C::TH;
    p.ntw = (p.W + C::TW - 1) / C::TW;
    p.ncg = (int)(mblocks / C::MB);
    p.total = (int64_t)p.N * p.ntd * p.nth * p.ntw * p.ncg;
    p.per_xcd = (p.total + 7) / 8;
    if (p.per_xcd * 8 > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    static bool attr_done = false;  // raising the dynamic LDS limit is idempotent
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_kernel<C>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        attr_done = true;
    }
    conv_mfma_kernel<C><<<dim3((unsigned)(p.per_xcd * 8)), 256, C::LDS_BYTES, st>>>(p);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

static int launch_mfma(MfmaParams p, int64_t mchannels, hipStream_t st)
{
    int64_t mblocks = mchannels / 32;
    if (mblocks % 2 == 0) return launch_cfg<TileCfg<8, 8, 8, 2, 9>>(p, mblocks, st);
    return launch_cfg<TileCfg<8, 8, 8, 1, 27>>(p, mblocks, st);
}

int conv_fwd_mfma(const ConvArgs &a, hipStream_t st)
{
    MfmaParams p{};
    p.src1 = (const bf16_t *)a.x;
    p.src2 = (const bf16_t *)a.x2;
    p.mask = nullptr;
    p.c1 = (int)a.c1;
    p.c2 = (int)a.c2;
    p.packed = (const bf16_t *)a.packed;
    p.bias = a.bias;
    p.relu = a.relu;
    p.dst1 = (bf16_t *)a.y;
    p.dst2 = nullptr;
    p.cd1 = (int)a.cout;
    p.cd2 = 0;
    p.N = (int)a.N; p.D = (int)a.D; p.H = (int)a.H; p.W = (int)a.W;
    return launch_mfma(p, a.cout, st);
}

int conv_dgrad_mfma(const ConvArgs &a, hipStream_t st)
{
    MfmaParams p{};
    int64_t cin = a.c1 + a.c2;
    p.src1 = (const bf16_t *)a.dy;
    p.src2 = nullptr;
    p.mask = (const bf16_t *)a.ymask;
    p.c1 = (int)a.cout;
    p.c2 = 0;
    p.packed = (const bf16_t *)a.packed + (int64_t)27 * cin * a.cout;  // bwd form follows the fwd form
    p.bias = nullptr;
    p.relu = 0;
    p.dst1 = (bf16_t *)a.dx;
    p.dst2 = (bf16_t *)a.dx2;
    p.cd1 = (int)a.c1;
    p.cd2 = (int)a.c2;
    p.N = (int)a.N; p.D = (int)a.D; p.H = (int)a.H; p.W = (int)a.W;
    return launch_mfma(p, cin, st);
}

}  // namespace k3
