// 2x2x2 stride-2 transposed convolution (decoder up-sampling), forward, backward-data and
// backward-weight, for gfx950.
//
// Every output voxel (2d+i, 2h+j, 2w+k) receives exactly one tap, so the forward pass is
// eight independent 1x1x1 GEMMs that share their input, and backward-data is one GEMM with
// contraction over (tap, C_out).  On the MFMA path (bf16, channels multiples of 32) the
// weights are the A operand (rows = produced channels, permuted so that a lane owns 16
// consecutive channels) and the activations the B operand, read straight from global
// memory: a lane needs 8 consecutive channels of one voxel, which is a 16-byte load.
// Backward-weight contracts over voxels and uses transposing LDS reads like the 3x3x3
// weight-gradient kernel.  Other dtypes / channel counts use direct kernels.
#include "common.h"
#include "conv_internal.h"

namespace k3 {

__host__ __device__ static inline int up_row_to_channel(int r) { return ((r >> 2) & 1) * 16 + (r >> 3) * 4 + (r & 3); }

static inline bool up_mfma_ok(int dtype, int64_t cin, int64_t cout)
{
    return dtype == K3_BF16 && cin % 32 == 0 && cout % 32 == 0;
}

// ------------------------------------------------------------------ packing
// fwd[tap][cob][kc][lane][j] = W[tap][kc*16 + (lane/32)*8 + j][cob*32 + r2c(lane%32)]
// bwd[cib][tap][kc][lane][j] = W[tap][cib*32 + r2c(lane%32)][kc*16 + (lane/32)*8 + j]
__global__ __launch_bounds__(256) void up_pack_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ packed,
                                                     int cin, int cout)
{
    int64_t per = (int64_t)8 * cin * cout;
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= 2 * per) return;
    bool bwd = i >= per;
    int64_t r = bwd ? i - per : i;
    int j = (int)(r & 7), lane = (int)((r >> 3) & 63);
    int64_t q = r >> 9;
    bf16_t v;
    if (!bwd) {
        int nkc = cin / 16, ncob = cout / 32;
        int kc = (int)(q % nkc);
        q /= nkc;
        int cob = (int)(q % ncob);
        int tap = (int)(q / ncob);
        v = w[((int64_t)tap * cin + kc * 16 + (lane >> 5) * 8 + j) * cout + cob * 32 + up_row_to_channel(lane & 31)];
    } else {
        int nkc = cout / 16;
        int kc = (int)(q % nkc);
        q /= nkc;
        int tap = (int)(q % 8);
        int cib = (int)(q / 8);
        v = w[((int64_t)tap * cin + cib * 32 + up_row_to_channel(lane & 31)) * cout + kc * 16 + (lane >> 5) * 8 + j];
    }
    packed[i] = v;
}

// ------------------------------------------------------------------ MFMA forward
// wave = 32 consecutive input voxels x one 32-channel output block x 8 taps
__global__ __launch_bounds__(256) void up_fwd_mfma_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ packed,
                                                         const float *__restrict__ bias, bf16_t *__restrict__ y,
                                                         int64_t V, int D, int H, int W, int cin, int cout)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int hb = lane >> 5, vl = lane & 31;
    const int64_t nb = (int64_t)blockIdx.x * 4 + wv;
    const int cob = blockIdx.y, ncob = cout / 32, nkc = cin / 16;
    const int64_t v = nb * 32 + vl;
    const bool live = v < V;
    f32x16 acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
    const uint4 *xp = reinterpret_cast<const uint4 *>(x + (live ? v : 0) * cin + hb * 8);
    const uint4 *ap = reinterpret_cast<const uint4 *>(packed) + lane;
    for (int kc = 0; kc < nkc; ++kc) {
        uint4 braw = live ? xp[kc * 2] : make_uint4(0, 0, 0, 0);
        bf16x8 b = __builtin_bit_cast(bf16x8, braw);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            uint4 araw = ap[(((int64_t)t * ncob + cob) * nkc + kc) * 64];
            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, araw), b, acc[t], 0, 0, 0);
        }
    }
    if (!live) return;
    int w = (int)(v % W);
    int h = (int)((v / W) % H);
    int d = (int)((v / ((int64_t)W * H)) % D);
    int64_t n = v / ((int64_t)W * H * D);
    const int co0 = cob * 32 + hb * 16;
    float bv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bv[i] = bias ? bias[co0 + i] : 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        int64_t o = ((n * 2 * D + 2 * d + (t >> 2)) * 2 * H + 2 * h + ((t >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (t & 1);
        float r[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) r[i] = acc[t][i] + bv[i];
        uint4 *dst = reinterpret_cast<uint4 *>(y + o * cout + co0);
        dst[0] = make_uint4(pack2bf(r[0], r[1]), pack2bf(r[2], r[3]), pack2bf(r[4], r[5]), pack2bf(r[6], r[7]));
        dst[1] = make_uint4(pack2bf(r[8], r[9]), pack2bf(r[10], r[11]), pack2bf(r[12], r[13]), pack2bf(r[14], r[15]));
    }
}

// ------------------------------------------------------------------ MFMA forward, weights in LDS
// The op is HBM-bound (it writes 8 output voxels per input voxel), so the kernel must not
// spend its memory pipe on weights: a persistent workgroup copies the packed weights of its
// COBG output blocks (8 taps x COBG x NKC fragments of 1 KB) into LDS once and then streams
// blocks of 128 input voxels.  A wave holds the NKC B fragments of its 32 voxels in registers
// (loaded with 16-byte accesses that together cover the voxels' contiguous rows) and, per
// (tap, output block), runs NKC MFMAs against LDS-resident A fragments, adds the bias and
// stores 32 bytes per lane.
template <int NKC, int COBG>
__global__ __launch_bounds__(256) void up_fwd_lds_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ packed,
                                                        const float *__restrict__ bias, bf16_t *__restrict__ y,
                                                        int64_t V, int D, int H, int W, int cout)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int cin = NKC * 16;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int hb = lane >> 5, vl = lane & 31;
    const int cob0 = blockIdx.y * COBG, ncob = cout / 32;
    {   // weights of this workgroup's output blocks: LDS [tap][cb][kc][lane] x 16 bytes
        const uint4 *src = reinterpret_cast<const uint4 *>(packed);
        uint4 *dst = reinterpret_cast<uint4 *>(smem);
        for (int i = threadIdx.x; i < 8 * COBG * NKC * 64; i += 256) {
            const int ln = i & 63, kc = (i >> 6) % NKC, cb = (i / (64 * NKC)) % COBG, t = i / (64 * NKC * COBG);
            dst[i] = src[(((int64_t)t * ncob + cob0 + cb) * NKC + kc) * 64 + ln];
        }
    }
    __syncthreads();
    float bv[COBG][16];
#pragma unroll
    for (int cb = 0; cb < COBG; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) bv[cb][i] = bias ? bias[(cob0 + cb) * 32 + hb * 16 + i] : 0.f;
    const int64_t nblk = (V + 127) / 128;
    for (int64_t blk = blockIdx.x; blk < nblk; blk += gridDim.x) {
        const int64_t v = blk * 128 + wv * 32 + vl;
        const bool live = v < V;
        const uint4 *xp = reinterpret_cast<const uint4 *>(x + (live ? v : 0) * cin + hb * 8);
        bf16x8 b[NKC];
#pragma unroll
        for (int kc = 0; kc < NKC; ++kc) {
            uint4 raw = xp[kc * 2];
            if (!live) raw = make_uint4(0, 0, 0, 0);
            b[kc] = __builtin_bit_cast(bf16x8, raw);
        }
        const int64_t vv = live ? v : 0;
        const int w = (int)(vv % W);
        const int h = (int)((vv / W) % H);
        const int d = (int)((vv / ((int64_t)W * H)) % D);
        const int64_t n = vv / ((int64_t)W * H * D);
        const int64_t o0 = ((n * 2 * D + 2 * d) * 2 * H + 2 * h) * (2 * (int64_t)W) + 2 * w;   // output voxel of tap 0
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const int64_t o = o0 + ((int64_t)(t >> 2) * 2 * H + ((t >> 1) & 1)) * (2 * (int64_t)W) + (t & 1);
#pragma unroll
            for (int cb = 0; cb < COBG; ++cb) {
                f32x16 acc;
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[i] = bv[cb][i];
                const bf16x8 *ap = reinterpret_cast<const bf16x8 *>(smem) + ((t * COBG + cb) * NKC) * 64 + lane;
#pragma unroll
                for (int kc = 0; kc < NKC; ++kc) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ap[kc * 64], b[kc], acc, 0, 0, 0);
                if (live) {
                    uint4 *dst = reinterpret_cast<uint4 *>(y + o * cout + (cob0 + cb) * 32 + hb * 16);
                    dst[0] = make_uint4(pack2bf(acc[0], acc[1]), pack2bf(acc[2], acc[3]), pack2bf(acc[4], acc[5]),
                                        pack2bf(acc[6], acc[7]));
                    dst[1] = make_uint4(pack2bf(acc[8], acc[9]), pack2bf(acc[10], acc[11]), pack2bf(acc[12], acc[13]),
                                        pack2bf(acc[14], acc[15]));
                }
            }
        }
    }
}

template <int NKC, int COBG>
static int launch_up_fwd_lds(const bf16_t *x, const bf16_t *packed, const float *bias, bf16_t *y, int64_t V, int D, int H,
                             int W, int cout, hipStream_t st)
{
    constexpr int lds = 8 * COBG * NKC * 1024;
    static_assert(lds <= 160 * 1024, "LDS budget");
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&up_fwd_lds_kernel<NKC, COBG>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    const int ncog = cout / 32 / COBG;
    int64_t nblk = (V + 127) / 128;
    int64_t gx = 512 / ncog;   // about two workgroups' worth of blocks per CU in total
    if (gx < 1) gx = 1;
    if (gx > nblk) gx = nblk;
    up_fwd_lds_kernel<NKC, COBG><<<dim3((unsigned)gx, (unsigned)ncog), 256, lds, st>>>(x, packed, bias, y, V, D, H, W, cout);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

// ------------------------------------------------------------------ MFMA forward, deep levels (C_in = 256, 512)
// With 256 or 512 input channels the op is as much a GEMM as a stream (16 or 32 MFMAs per tap, block
// and 32 voxels) and a wave is alone on its SIMD (the weights fill the LDS), so the kernel above loses
// its time to latencies: its loads are waited for right where they are issued, and the MFMAs of a
// (tap, block) form one dependent chain on a single accumulator.  Here
//   * a workgroup owns one 32-channel output block and NT taps (blockIdx.z picks the tap group:
//     NT x NKC KB of packed weights in LDS, 128 KB for both channel counts),
//   * the B fragments of the NEXT block of voxels are requested before the current block is multiplied
//     (two register sets used in turn; clamped addresses, so the loop has no conditional memory
//     operation and the waits are counted),
//   * two accumulator chains run interleaved: two groups of 32 voxels against the same weight fragment
//     (VG = 2, C_in = 256: one LDS read per two MFMAs) or two taps against the same voxels (VG = 1,
//     C_in = 512, where two voxel groups would not fit the registers twice),
//   * results leave through a descriptor at the block's first output voxel with 32-bit offsets; lanes
//     beyond the last voxel get an offset outside its range and their stores are dropped.
template <int NKC, int NT, int VG>
__global__ __launch_bounds__(256, 1) void up_fwd_deep_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ packed,
                                                            const float *__restrict__ bias, bf16_t *__restrict__ y,
                                                            int64_t V, int D, int H, int W, int cout)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int cin = NKC * 16;
    constexpr int BV = 128 * VG;                      // voxels per block
    const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int hb = lane >> 5, vl = lane & 31;
    const int cob = blockIdx.y, ncob = cout / 32, tap0 = blockIdx.z * NT;
    {   // weights of this workgroup's output block and taps: LDS [tap][kc][lane] x 16 bytes
        const uint4 *src = reinterpret_cast<const uint4 *>(packed);
        uint4 *dst = reinterpret_cast<uint4 *>(smem);
        for (int i = threadIdx.x; i < NT * NKC * 64; i += 256) {
            const int ln = i & 63, kc = (i >> 6) % NKC, t = i / (64 * NKC);
            dst[i] = src[(((int64_t)(tap0 + t) * ncob + cob) * NKC + kc) * 64 + ln];
        }
    }
    float bv[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) bv[i] = bias ? bias[cob * 32 + hb * 16 + i] : 0.f;
    __syncthreads();
    const int64_t nblk = (V + BV - 1) / BV;
    const unsigned HW = (unsigned)H * (unsigned)W;

    auto load_b = [&](int64_t blk, bf16x8 (&b)[VG][NKC]) __attribute__((always_inline)) {
#pragma unroll
        for (int g = 0; g < VG; ++g) {
            int64_t v = blk * BV + (g * 4 + wv) * 32 + vl;
            v = v < V ? v : V - 1;
            const uint4 *xp = reinterpret_cast<const uint4 *>(x + v * cin + hb * 8);
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) b[g][kc] = __builtin_bit_cast(bf16x8, xp[kc * 2]);
        }
    };
    // output voxel index of input voxel v (tap 0): 8 H W (n D + d) + 4 h W + 2 w
    auto out_index = [&](unsigned v) __attribute__((always_inline)) {
        const unsigned plane = v / HW, r = v - plane * HW, h = r / (unsigned)W, w = r - h * (unsigned)W;
        return (int64_t)plane * (8 * (int64_t)HW) + (int64_t)(4 * h * (unsigned)W + 2 * w);
    };
    auto store16 = [&](const f32x16 &acc, __amdgpu_buffer_rsrc_t rs, int off) __attribute__((always_inline)) {
        typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
        u32x4 lo = {pack2bf(acc[0], acc[1]), pack2bf(acc[2], acc[3]), pack2bf(acc[4], acc[5]), pack2bf(acc[6], acc[7])};
        u32x4 hi = {pack2bf(acc[8], acc[9]), pack2bf(acc[10], acc[11]), pack2bf(acc[12], acc[13]), pack2bf(acc[14], acc[15])};
        __builtin_amdgcn_raw_buffer_store_b128(lo, rs, off, 0, 0);
        __builtin_amdgcn_raw_buffer_store_b128(hi, rs, off, 16, 0);
        // a 16-byte buffer store may read its data registers a few cycles after it has issued: keep them untouched
        asm volatile("s_nop 7" : "+v"(lo), "+v"(hi));
    };
    auto compute = [&](int64_t blk, const bf16x8 (&b)[VG][NKC]) __attribute__((always_inline)) {
        const unsigned vfirst = (unsigned)(blk * BV);                  // (V fits 31 bits: checked at launch)
        const int64_t ofirst = out_index(vfirst);
        __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(y + ofirst * cout + cob * 32, 0, 0x7ffffff0, 0x00020000);
        int off0[VG];                                                  // byte offset of the lane's tap-0 output voxel, or "dropped"
#pragma unroll
        for (int g = 0; g < VG; ++g) {
            const int64_t v = blk * BV + (g * 4 + wv) * 32 + vl;
            const bool live = v < V;
            const int64_t o = out_index(live ? (unsigned)v : vfirst) - ofirst;
            off0[g] = live ? ((int)o * cout + hb * 16) * 2 : -1;
        }
        const bf16x8 *aw = reinterpret_cast<const bf16x8 *>(smem) + lane;
        if (VG == 2) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int tap = tap0 + t;
                const int toff = (((tap >> 2) * 2 * H + ((tap >> 1) & 1)) * (2 * W) + (tap & 1)) * cout * 2;
                f32x16 a0, a1;
#pragma unroll
                for (int i = 0; i < 16; ++i) a0[i] = a1[i] = bv[i];
#pragma unroll
                for (int kc = 0; kc < NKC; ++kc) {
                    const bf16x8 a = aw[(t * NKC + kc) * 64];
                    a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[0][kc], a0, 0, 0, 0);
                    a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b[VG - 1][kc], a1, 0, 0, 0);
                }
                store16(a0, rs, off0[0] < 0 ? -1 : off0[0] + toff);
                store16(a1, rs, off0[VG - 1] < 0 ? -1 : off0[VG - 1] + toff);
            }
        } else {
#pragma unroll
            for (int t = 0; t < NT; t += 2) {
                const int tapa = tap0 + t, tapb = tap0 + t + 1;
                const int toffa = (((tapa >> 2) * 2 * H + ((tapa >> 1) & 1)) * (2 * W) + (tapa & 1)) * cout * 2;
                const int toffb = (((tapb >> 2) * 2 * H + ((tapb >> 1) & 1)) * (2 * W) + (tapb & 1)) * cout * 2;
                f32x16 a0, a1;
#pragma unroll
                for (int i = 0; i < 16; ++i) a0[i] = a1[i] = bv[i];
#pragma unroll
                for (int kc = 0; kc < NKC; ++kc) {
                    a0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aw[(t * NKC + kc) * 64], b[0][kc], a0, 0, 0, 0);
                    a1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aw[((t + 1) * NKC + kc) * 64], b[0][kc], a1, 0, 0, 0);
                }
                store16(a0, rs, off0[0] < 0 ? -1 : off0[0] + toffa);
                store16(a1, rs, off0[0] < 0 ? -1 : off0[0] + toffb);
            }
        }
    };

    if ((int64_t)blockIdx.x >= nblk) return;
    bf16x8 b0[VG][NKC], b1[VG][NKC];
    load_b(blockIdx.x, b0);
    for (int64_t blk = blockIdx.x; blk < nblk; blk += 2 * (int64_t)gridDim.x) {
        const int64_t nx = blk + gridDim.x, nx2 = blk + 2 * (int64_t)gridDim.x;
        load_b(nx < nblk ? nx : nblk - 1, b1);          // (beyond the end: the last block again, unused)
        compute(blk, b0);
        if (nx >= nblk) break;
        load_b(nx2 < nblk ? nx2 : nblk - 1, b0);
        compute(nx, b1);
    }
}

template <int NKC, int NT, int VG>
static int launch_up_fwd_deep(const bf16_t *x, const bf16_t *packed, const float *bias, bf16_t *y, int64_t V, int D, int H,
                              int W, int cout, hipStream_t st)
{
    constexpr int lds = NT * NKC * 1024;
    static_assert(lds <= 160 * 1024 && 8 % NT == 0 && (VG == 2 || NT % 2 == 0), "LDS budget / tap groups");
    // 32-bit voxel arithmetic and byte offsets from a block's first output voxel (a block of BV consecutive
    // input voxels spans at most 8 BV + 12 H W output voxels, a tap adds at most 4 H W + 2 W + 1)
    const int64_t span = 8 * (int64_t)(128 * VG) + 16 * (int64_t)H * W + 2 * (int64_t)W + 2;
    if (V > 0x7fffffffLL || span * cout * 2 + 64 > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&up_fwd_deep_kernel<NKC, NT, VG>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    const int ncob = cout / 32, ntg = 8 / NT;
    const int64_t nblk = (V + 128 * VG - 1) / (128 * VG);
    int64_t gx = 256 / (ncob * ntg);   // one workgroup per CU in total (the weights fill its LDS)
    if (gx < 1) gx = 1;
    if (gx > nblk) gx = nblk;
    up_fwd_deep_kernel<NKC, NT, VG><<<dim3((unsigned)gx, (unsigned)ncob, (unsigned)ntg), 256, lds, st>>>(x, packed, bias, y, V, D, H,
                                                                                                      W, cout);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

// returns K3_E_UNSUPPORTED when the shape has no LDS-resident variant (the caller falls back)
static int up_fwd_lds_dispatch(const bf16_t *x, const bf16_t *packed, const float *bias, bf16_t *y, int64_t V, int D, int H,
                               int W, int cin, int cout, hipStream_t st)
{
    const bool two = (cout / 32) % 2 == 0;
    switch (cin) {
    case 32: return two ? launch_up_fwd_lds<2, 2>(x, packed, bias, y, V, D, H, W, cout, st)
                        : launch_up_fwd_lds<2, 1>(x, packed, bias, y, V, D, H, W, cout, st);
    case 64: return two ? launch_up_fwd_lds<4, 2>(x, packed, bias, y, V, D, H, W, cout, st)
                        : launch_up_fwd_lds<4, 1>(x, packed, bias, y, V, D, H, W, cout, st);
    case 128: return two ? launch_up_fwd_lds<8, 2>(x, packed, bias, y, V, D, H, W, cout, st)
                         : launch_up_fwd_lds<8, 1>(x, packed, bias, y, V, D, H, W, cout, st);
    case 256: {
        const int rc = launch_up_fwd_deep<16, 8, 2>(x, packed, bias, y, V, D, H, W, cout, st);
        return rc != K3_E_UNSUPPORTED ? rc : launch_up_fwd_lds<16, 1>(x, packed, bias, y, V, D, H, W, cout, st);
    }
    case 512: return launch_up_fwd_deep<32, 4, 1>(x, packed, bias, y, V, D, H, W, cout, st);
    default: return K3_E_UNSUPPORTED;
    }
}

__device__ __forceinline__ uint32_t up_mask_pair(uint32_t v, uint32_t m)
{
    // keep each bf16 half of v where the matching half of m is > 0 (sign clear and nonzero)
    uint32_t lo = ((m & 0x8000u) == 0 && (m & 0x7fffu) != 0) ? 0x0000ffffu : 0u;
    uint32_t hi = ((m & 0x80000000u) == 0 && (m & 0x7fff0000u) != 0) ? 0xffff0000u : 0u;
    return v & (lo | hi);
}

// ------------------------------------------------------------------ MFMA backward-data
// wave = 32 consecutive input voxels x MB 32-channel blocks of dx; contraction over (tap, C_out).
// This first form requests one fragment pair per 16-channel step and serves the channel counts
// the tap-preload form below has no instantiation for.
template <int MB>
__global__ __launch_bounds__(256) void up_dgrad_mfma_kernel(const bf16_t *__restrict__ dy,
                                                           const bf16_t *__restrict__ packed, bf16_t *__restrict__ dx,
                                                           const bf16_t *__restrict__ omask, int64_t V, int D, int H,
                                                           int W, int cin, int cout)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int hb = lane >> 5, vl = lane & 31;
    const int64_t nb = (int64_t)blockIdx.x * 4 + wv;
    const int cib0 = blockIdx.y * MB, nkc = cout / 16;
    const int64_t v = nb * 32 + vl;
    const bool live = v < V;
    const int64_t vv = live ? v : 0;
    int w = (int)(vv % W);
    int h = (int)((vv / W) % H);
    int d = (int)((vv / ((int64_t)W * H)) % D);
    int64_t n = vv / ((int64_t)W * H * D);
    f32x16 acc[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[m][i] = 0.f;
    const uint4 *ap = reinterpret_cast<const uint4 *>(packed) + lane;
    for (int t = 0; t < 8; ++t) {
        int64_t o = ((n * 2 * D + 2 * d + (t >> 2)) * 2 * H + 2 * h + ((t >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (t & 1);
        const uint4 *gp = reinterpret_cast<const uint4 *>(dy + o * cout + hb * 8);
        for (int kc = 0; kc < nkc; ++kc) {
            uint4 braw = live ? gp[kc * 2] : make_uint4(0, 0, 0, 0);
            bf16x8 b = __builtin_bit_cast(bf16x8, braw);
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                uint4 araw = ap[(((int64_t)(cib0 + m) * 8 + t) * nkc + kc) * 64];
                acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, araw), b, acc[m], 0, 0, 0);
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const int64_t eo = v * cin + (cib0 + m) * 32 + hb * 16;
        uint4 o0 = make_uint4(pack2bf(acc[m][0], acc[m][1]), pack2bf(acc[m][2], acc[m][3]), pack2bf(acc[m][4], acc[m][5]),
                              pack2bf(acc[m][6], acc[m][7]));
        uint4 o1 = make_uint4(pack2bf(acc[m][8], acc[m][9]), pack2bf(acc[m][10], acc[m][11]),
                              pack2bf(acc[m][12], acc[m][13]), pack2bf(acc[m][14], acc[m][15]));
        if (omask) {
            const uint4 *mp = reinterpret_cast<const uint4 *>(omask + eo);
            uint4 m0 = mp[0], m1 = mp[1];
            o0.x = up_mask_pair(o0.x, m0.x); o0.y = up_mask_pair(o0.y, m0.y); o0.z = up_mask_pair(o0.z, m0.z); o0.w = up_mask_pair(o0.w, m0.w);
            o1.x = up_mask_pair(o1.x, m1.x); o1.y = up_mask_pair(o1.y, m1.y); o1.z = up_mask_pair(o1.z, m1.z); o1.w = up_mask_pair(o1.w, m1.w);
        }
        uint4 *dst = reinterpret_cast<uint4 *>(dx + eo);
        dst[0] = o0;
        dst[1] = o1;
    }
}

// Variant with the loads of a whole tap in flight at once: the NKC dy fragments and the MB * NKC
// weight fragments of tap t are requested before the tap's matrix instructions, so a wave pays
// one memory round trip per tap instead of one per 16-channel step.  NKC = C_out / 16 is a
// template parameter so that the fragments live in registers.
template <int MB, int NKC, int KCH>
__global__ __launch_bounds__(256) void up_dgrad_tap_kernel(const bf16_t *__restrict__ dy, const bf16_t *__restrict__ packed,
                                                          bf16_t *__restrict__ dx, const bf16_t *__restrict__ omask,
                                                          int64_t V, int D, int H, int W, int cin)
{
    constexpr int cout = NKC * 16;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int hb = lane >> 5, vl = lane & 31;
    const int64_t nb = (int64_t)blockIdx.x * 4 + wv;
    const int cib0 = blockIdx.y * MB;
    const int64_t v = nb * 32 + vl;
    const bool live = v < V;
    const int64_t vv = live ? v : V - 1;   // dead lanes read a valid voxel and store nothing
    const int w = (int)(vv % W);
    const int h = (int)((vv / W) % H);
    const int d = (int)((vv / ((int64_t)W * H)) % D);
    const int64_t n = vv / ((int64_t)W * H * D);
    f32x16 acc[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[m][i] = 0.f;
    const uint4 *ap = reinterpret_cast<const uint4 *>(packed) + lane;
#pragma unroll 1
    for (int t = 0; t < 8; ++t) {
        const int64_t o = ((n * 2 * D + 2 * d + (t >> 2)) * 2 * H + 2 * h + ((t >> 1) & 1)) * (2 * (int64_t)W) + 2 * w + (t & 1);
        const uint4 *gp = reinterpret_cast<const uint4 *>(dy + o * cout + hb * 8);
#pragma unroll
        for (int k0 = 0; k0 < NKC; k0 += KCH) {
            uint4 braw[KCH], araw[MB][KCH];
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) braw[kc] = gp[(k0 + kc) * 2];
#pragma unroll
            for (int m = 0; m < MB; ++m)
#pragma unroll
                for (int kc = 0; kc < KCH; ++kc) araw[m][kc] = ap[(((int64_t)(cib0 + m) * 8 + t) * NKC + k0 + kc) * 64];
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc)
#pragma unroll
                for (int m = 0; m < MB; ++m)
                    acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, araw[m][kc]),
                                                                     __builtin_bit_cast(bf16x8, braw[kc]), acc[m], 0, 0, 0);
        }
    }
    if (!live) return;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const int64_t eo = v * cin + (cib0 + m) * 32 + hb * 16;
        uint4 o0 = make_uint4(pack2bf(acc[m][0], acc[m][1]), pack2bf(acc[m][2], acc[m][3]), pack2bf(acc[m][4], acc[m][5]),
                              pack2bf(acc[m][6], acc[m][7]));
        uint4 o1 = make_uint4(pack2bf(acc[m][8], acc[m][9]), pack2bf(acc[m][10], acc[m][11]),
                              pack2bf(acc[m][12], acc[m][13]), pack2bf(acc[m][14], acc[m][15]));
        if (omask) {
            const uint4 *mp = reinterpret_cast<const uint4 *>(omask + eo);
            uint4 m0 = mp[0], m1 = mp[1];
            o0.x = up_mask_pair(o0.x, m0.x); o0.y = up_mask_pair(o0.y, m0.y); o0.z = up_mask_pair(o0.z, m0.z); o0.w = up_mask_pair(o0.w, m0.w);
            o1.x = up_mask_pair(o1.x, m1.x); o1.y = up_mask_pair(o1.y, m1.y); o1.z = up_mask_pair(o1.z, m1.z); o1.w = up_mask_pair(o1.w, m1.w);
        }
        uint4 *dst = reinterpret_cast<uint4 *>(dx + eo);
        dst[0] = o0;
        dst[1] = o1;
    }
}

template <int MB, int NKC, int KCH>
static void launch_up_dgrad_tap(const bf16_t *dy, const bf16_t *pb, bf16_t *dx, const bf16_t *mask, int64_t V, int D, int H,
                                int W, int cin, hipStream_t st)
{
    const int64_t blocks = (V + 127) / 128;
    up_dgrad_tap_kernel<MB, NKC, KCH><<<dim3((unsigned)blocks, (unsigned)(cin / 32 / MB)), 256, 0, st>>>(dy, pb, dx, mask, V, D, H, W, cin);
}

// Picks the tap-preload instantiation for the shape; false when there is none (C_out not 32, 64,
// 128 or 256).  MB (32-channel blocks of dx per wave) is the largest of 4, 2, 1 that divides the
// block count and still gives the chip at least one workgroup per compute unit: small volumes
// want many short waves, large ones want dy fetched by as few channel groups as possible.  The
// fragments of KCH 16-channel steps are in registers at once: (MB + 1) * KCH vectors of four.
static bool up_dgrad_tap_dispatch(const bf16_t *dy, const bf16_t *pb, bf16_t *dx, const bf16_t *mask, int64_t V, int D, int H,
                                  int W, int cin, int cout, hipStream_t st)
{
    const int nb = cin / 32;
    const int64_t blocks = (V + 127) / 128;
    int mb = 1;
    if (nb % 4 == 0 && blocks * (nb / 4) >= 256) mb = 4;
    else if (nb % 2 == 0 && blocks * (nb / 2) >= 256) mb = 2;
#define K3_UPT(MBV, NKCV, KCHV)                                                         \
    if (mb == MBV && cout == NKCV * 16) {                                               \
        launch_up_dgrad_tap<MBV, NKCV, KCHV>(dy, pb, dx, mask, V, D, H, W, cin, st);    \
        return true;                                                                    \
    }
    K3_UPT(1, 2, 2) K3_UPT(2, 2, 2) K3_UPT(4, 2, 2)
    K3_UPT(1, 4, 4) K3_UPT(2, 4, 4) K3_UPT(4, 4, 4)
    K3_UPT(1, 8, 8) K3_UPT(2, 8, 8) K3_UPT(4, 8, 4)
    K3_UPT(1, 16, 8) K3_UPT(2, 16, 8) K3_UPT(4, 16, 4)
#undef K3_UPT
    return false;
}

// ------------------------------------------------------------------ MFMA backward-data, weights in LDS
// The kernels above read every weight fragment from global memory / L2 right before its matrix
// instruction: 1 KB per MFMA, which at the 64- to 256-channel levels of a large volume is several
// times the traffic of dy itself and sets the pace.  Here a persistent workgroup keeps the packed
// weights of its MBW 32-channel blocks of dx in LDS (MBW x 8 taps x NKC KB = 128 KB for the three
// shapes served) and walks blocks of 128 * VG input voxels.  Per tap the NKC dy fragments of a voxel
// group are in registers; the fragments of the NEXT tap (or of the next block's first tap) are
// requested before the current tap is multiplied, into the other of two register sets.  VG * MBW
// accumulators give independent MFMA chains, and with VG = 2 a weight fragment read from LDS serves
// two matrix instructions.  All loads go through descriptors at the block's first voxel with
// 32-bit offsets and are unconditional (lanes beyond the last voxel read the block's first voxel
// and their stores are dropped), so the waits are counted.  The ReLU mask of dx, when given, is
// requested at the start of a block and applied at its end.
template <int NKC, int MBW, int VG, bool MASK>
__global__ __launch_bounds__(256, 1) void up_dgrad_lds_kernel(const bf16_t *__restrict__ dy, const bf16_t *__restrict__ packed,
                                                             bf16_t *__restrict__ dx, const bf16_t *__restrict__ omask,
                                                             int64_t V, int D, int H, int W, int cin)
{
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int cout = NKC * 16;
    constexpr int BV = 128 * VG;
    const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int hb = lane >> 5, vl = lane & 31;
    const int cib0 = blockIdx.y * MBW;
    {   // weights of this workgroup's blocks of dx: LDS [m][tap][kc][lane] x 16 bytes (the packed order)
        const uint4 *src = reinterpret_cast<const uint4 *>(packed) + (int64_t)cib0 * 8 * NKC * 64;
        uint4 *dst = reinterpret_cast<uint4 *>(smem);
        for (int i = threadIdx.x; i < MBW * 8 * NKC * 64; i += 256) dst[i] = src[i];
    }
    __syncthreads();
    const int64_t nblk = (V + BV - 1) / BV;
    if ((int64_t)blockIdx.x >= nblk) return;
    const unsigned HW = (unsigned)H * (unsigned)W;
    // output voxel index of input voxel v (tap 0): 8 H W (n D + d) + 4 h W + 2 w
    auto out_index = [&](unsigned v) __attribute__((always_inline)) {
        const unsigned plane = v / HW, r = v - plane * HW, h = r / (unsigned)W, w = r - h * (unsigned)W;
        return (int64_t)plane * (8 * (int64_t)HW) + (int64_t)(4 * h * (unsigned)W + 2 * w);
    };
    struct Src {
        __amdgpu_buffer_rsrc_t rs;   // dy at the block's first output voxel
        int voff[VG];                // the lane's tap-0 byte offset from there
    };
    auto make_src = [&](int64_t blk) __attribute__((always_inline)) {
        Src s;
        const unsigned vfirst = (unsigned)(blk * BV);                  // (V fits 31 bits: checked at launch)
        const int64_t ofirst = out_index(vfirst);
        s.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dy) + ofirst * cout, 0, 0x7ffffff0, 0x00020000);
#pragma unroll
        for (int g = 0; g < VG; ++g) {
            const int64_t v = blk * BV + (g * 4 + wv) * 32 + vl;
            const int64_t o = out_index(v < V ? (unsigned)v : vfirst) - ofirst;
            s.voff[g] = (int)o * cout * 2 + hb * 16;
        }
        return s;
    };
    auto load_tap = [&](const Src &s, int t, u32x4 (&b)[VG][NKC]) __attribute__((always_inline)) {
        const int toff = (((t >> 2) * 2 * H + ((t >> 1) & 1)) * (2 * W) + (t & 1)) * cout * 2;
#pragma unroll
        for (int g = 0; g < VG; ++g)
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) b[g][kc] = __builtin_amdgcn_raw_buffer_load_b128(s.rs, s.voff[g] + kc * 32, toff, 0);
    };
    f32x16 acc[VG][MBW];
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int g = 0; g < VG; ++g)
#pragma unroll
            for (int m = 0; m < MBW; ++m)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[g][m][i] = 0.f;
    };
    const bf16x8 *aw = reinterpret_cast<const bf16x8 *>(smem) + lane;
    auto mfma_tap = [&](int t, const u32x4 (&b)[VG][NKC]) __attribute__((always_inline)) {
#pragma unroll
        for (int kc = 0; kc < NKC; ++kc)
#pragma unroll
            for (int m = 0; m < MBW; ++m) {
                const bf16x8 a = aw[((m * 8 + t) * NKC + kc) * 64];
#pragma unroll
                for (int g = 0; g < VG; ++g)
                    acc[g][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, b[g][kc]), acc[g][m], 0, 0, 0);
            }
    };

    int64_t blk = blockIdx.x;
    Src cur = make_src(blk);
    u32x4 b0[VG][NKC], b1[VG][NKC];
    load_tap(cur, 0, b0);
    zero_acc();
    for (;;) {
        // dx (and its mask) of this block: descriptors at the block's first voxel, first channel of the workgroup
        const int64_t vfirst = blk * BV;
        __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(dx + vfirst * cin + cib0 * 32, 0, 0x7ffffff0, 0x00020000);
        __amdgpu_buffer_rsrc_t mrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(MASK ? omask : dx) + vfirst * cin + cib0 * 32,
                                                                       0, 0x7ffffff0, 0x00020000);
        int xoff[VG];
        u32x4 mk[VG][MBW][2];
#pragma unroll
        for (int g = 0; g < VG; ++g) {
            const int64_t v = vfirst + (g * 4 + wv) * 32 + vl;
            const int lo = ((int)(v - vfirst) * cin + hb * 16) * 2;
            xoff[g] = v < V ? lo : -1;
            if (MASK) {
                const int mo = v < V ? lo : hb * 32;
#pragma unroll
                for (int m = 0; m < MBW; ++m) {
                    mk[g][m][0] = __builtin_amdgcn_raw_buffer_load_b128(mrs, mo, m * 64, 0);
                    mk[g][m][1] = __builtin_amdgcn_raw_buffer_load_b128(mrs, mo, m * 64 + 16, 0);
                }
            }
        }
        const int64_t nb = blk + gridDim.x;
        Src nxt = cur;
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            if (t < 7) {
                load_tap(cur, t + 1, (t & 1) ? b0 : b1);
            } else {
                nxt = make_src(nb < nblk ? nb : nblk - 1);      // (beyond the end: the last block again, unused)
                load_tap(nxt, 0, b0);
            }
            mfma_tap(t, (t & 1) ? b1 : b0);
        }
#pragma unroll
        for (int g = 0; g < VG; ++g)
#pragma unroll
            for (int m = 0; m < MBW; ++m) {
                const f32x16 &a = acc[g][m];
                u32x4 o0 = {pack2bf(a[0], a[1]), pack2bf(a[2], a[3]), pack2bf(a[4], a[5]), pack2bf(a[6], a[7])};
                u32x4 o1 = {pack2bf(a[8], a[9]), pack2bf(a[10], a[11]), pack2bf(a[12], a[13]), pack2bf(a[14], a[15])};
                if (MASK) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        o0[i] = up_mask_pair(o0[i], mk[g][m][0][i]);
                        o1[i] = up_mask_pair(o1[i], mk[g][m][1][i]);
                    }
                }
                __builtin_amdgcn_raw_buffer_store_b128(o0, xrs, xoff[g], m * 64, 0);
                __builtin_amdgcn_raw_buffer_store_b128(o1, xrs, xoff[g], m * 64 + 16, 0);
                // a 16-byte buffer store may read its data registers a few cycles after it has issued: keep them untouched
                asm volatile("s_nop 7" : "+v"(o0), "+v"(o1));
            }
        zero_acc();
        blk = nb;
        if (blk >= nblk) break;
        cur = nxt;
    }
}

template <int NKC, int MBW, int VG>
static int launch_up_dgrad_lds(const bf16_t *dy, const bf16_t *pb, bf16_t *dx, const bf16_t *mask, int64_t V, int D, int H, int W,
                               int cin, hipStream_t st)
{
    constexpr int lds = MBW * 8 * NKC * 1024;
    static_assert(lds <= 160 * 1024, "LDS budget");
    constexpr int cout = NKC * 16;
    // 32-bit voxel arithmetic and byte offsets from a block's first voxel (a block of BV consecutive input
    // voxels spans at most 8 BV + 12 H W output voxels, a tap adds at most 4 H W + 2 W + 1)
    const int64_t span = 8 * (int64_t)(128 * VG) + 16 * (int64_t)H * W + 2 * (int64_t)W + 2;
    if (V > 0x7fffffffLL || span * cout * 2 + 64 > 0x7fffffffLL || (int64_t)128 * VG * cin * 2 > 0x7fffffffLL ||
        (cin / 32) % MBW != 0)
        return K3_E_UNSUPPORTED;
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&up_dgrad_lds_kernel<NKC, MBW, VG, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&up_dgrad_lds_kernel<NKC, MBW, VG, true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    const int ngrp = cin / 32 / MBW;
    const int64_t nblk = (V + 128 * VG - 1) / (128 * VG);
    int64_t gx = 256 / ngrp;   // one workgroup per CU in total (the weights fill its LDS)
    if (gx < 1) gx = 1;
    if (gx > nblk) gx = nblk;
    if (mask)
        up_dgrad_lds_kernel<NKC, MBW, VG, true><<<dim3((unsigned)gx, (unsigned)ngrp), 256, lds, st>>>(dy, pb, dx, mask, V, D, H, W, cin);
    else
        up_dgrad_lds_kernel<NKC, MBW, VG, false><<<dim3((unsigned)gx, (unsigned)ngrp), 256, lds, st>>>(dy, pb, dx, mask, V, D, H, W, cin);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

// The LDS-resident form serves the levels of a large volume: enough voxel blocks to give every compute unit
// several, and a channel pair it has an instantiation for.  K3_E_UNSUPPORTED: the caller uses the forms above.
static int up_dgrad_lds_dispatch(const bf16_t *dy, const bf16_t *pb, bf16_t *dx, const bf16_t *mask, int64_t V, int D, int H,
                                 int W, int cin, int cout, hipStream_t st)
{
    if (V < 4 * 256 * 128) return K3_E_UNSUPPORTED;
    if (cout == 64 && cin % 128 == 0) return launch_up_dgrad_lds<4, 4, 1>(dy, pb, dx, mask, V, D, H, W, cin, st);
    if (cout == 128 && cin % 64 == 0) return launch_up_dgrad_lds<8, 2, 2>(dy, pb, dx, mask, V, D, H, W, cin, st);
    if (cout == 256) return launch_up_dgrad_lds<16, 1, 2>(dy, pb, dx, mask, V, D, H, W, cin, st);
    return K3_E_UNSUPPORTED;
}

// ------------------------------------------------------------------ MFMA backward-weight
// dW[t][ci][co] = sum_v x[v][ci] * dy[2v + t][co]: the contraction runs over input voxels and
// dy is the large tensor (8 voxels per input voxel), so the pass is HBM-bound and every byte
// of dy should be fetched once.  A persistent workgroup owns CIBG 32-channel blocks of x and
// COBG blocks of dy -- the whole weight gradient when C_in <= 128 and C_out <= 64 -- and a
// contiguous range of 2x2x8 input-voxel tiles (4x4x16 output voxels).  Tiles move from global
// memory into a ring of three LDS stages with asynchronous copies, two tiles ahead of the one
// being multiplied.  Wave wv owns the taps (i, j) = (wv / 2, wv % 2), k = 0, 1, for all
// channel blocks: 2 * CIBG * COBG accumulator blocks.  The operands (8 consecutive voxels of
// one channel per lane) come from transposing LDS reads.  The bias gradient is summed on the
// vector ALU from the dy fragments the wave reads anyway.  Partials per split are added in a
// fixed order by reduce_partials_kernel.
namespace uw {
constexpr int TD = 2, TH = 2, TW = 8;
constexpr int NVOX = TD * TH * TW;            // 32 input voxels = 2 K-steps
constexpr int XB = NVOX * 64;                 // one 32-channel block of the x tile
constexpr int GB = NVOX * 8 * 64;             // one 32-channel block of the dy tile
constexpr int NST = 3;                        // ring of stages: one in use, two incoming
constexpr int xk(int cibg) { return (cibg * 2 + 3) / 4; }   // copies per wave: x groups (1 KB each)
constexpr int gk(int cobg) { return cobg * 4; }             // dy groups
constexpr int stage_bytes(int cibg, int cobg) { return cibg * XB + cobg * GB; }
constexpr int lds_bytes(int cibg, int cobg) { return NST * stage_bytes(cibg, cobg) + 1024 + 4 * 64 * 4; }
}  // namespace uw

struct UpWgradParams {
    const bf16_t *x, *dy;
    float *ws;
    int64_t per_split;
    int N, D, H, W, cin, cout;
    int ntd, nth, ntw;
    int ntiles, nsplit, tbase, trem;   // split s owns tiles [s*tbase + min(s, trem), ...)
};

static __device__ uint4 g_uzero[4];   // zero-initialised: source of every out-of-volume item

__device__ __forceinline__ bf16x8 up_tr_pair(const unsigned char *base, int off0, int off1)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(base + off0));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(base + off1));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

template <int CIBG, int COBG>
__global__ __launch_bounds__(256, 1) void up_wgrad_pipe_kernel(UpWgradParams p)
{
    using namespace uw;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int STB = stage_bytes(CIBG, COBG);
    constexpr int XK = xk(CIBG), GK = gk(COBG), OPS = XK + GK;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hb = lane >> 5, g16 = (lane >> 4) & 1, j = lane & 15;
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned dump = lds0 + NST * STB;
    float *dbs = reinterpret_cast<float *>(smem + NST * STB + 1024);   // [4 waves][COBG * 32]
    const unsigned char *zero = reinterpret_cast<const unsigned char *>(g_uzero);
    const int split = blockIdx.x, cig = blockIdx.y, cog = blockIdx.z;
    const int ti = wv >> 1, tj = wv & 1;
    const int D2 = 2 * p.D, H2 = 2 * p.H, W2 = 2 * p.W;

    // ---- per-lane copy items.  x stage layout [cib][vox 32][32 ch], dy [cob][vox 256][32 ch]
    int xoff[XK], xco[XK];
    unsigned xsl = 0;
#pragma unroll
    for (int k = 0; k < XK; ++k) {
        const int slot = (wv + 4 * k) * 64 + lane;
        const int cib = slot >> 7, vox = (slot >> 2) & 31, part = slot & 3;
        const int ld = vox >> 4, lh = (vox >> 3) & 1, lw = vox & 7;
        xoff[k] = ((ld * p.H + lh) * p.W + lw) * p.cin * 2 + ((cig * CIBG + cib) * 32) * 2 + part * 16;
        xco[k] = ld | (lh << 8) | (lw << 16);
        xsl |= ((wv + 4 * k < CIBG * 2) ? 1u : 0u) << k;
    }
    int goff[GK], gco[GK];
#pragma unroll
    for (int k = 0; k < GK; ++k) {
        const int slot = (wv + 4 * k) * 64 + lane;
        const int cob = slot >> 10, vox = (slot >> 2) & 255, part = slot & 3;
        const int ld = vox >> 6, lh = (vox >> 4) & 3, lw = vox & 15;
        goff[k] = ((ld * H2 + lh) * W2 + lw) * p.cout * 2 + ((cog * COBG + cob) * 32) * 2 + part * 16;
        gco[k] = ld | (lh << 8) | (lw << 16);
    }
    // ---- lane-constant parts of the transposing-read addresses (K-step 0, first block)
    const int lane_x = (hb * TW + (j >> 2)) * 64 + g16 * 32 + (j & 3) * 8;
    const int lane_g = CIBG * XB + ((ti * 4 + 2 * hb + tj) * 16 + 2 * (j >> 2)) * 64 + g16 * 32 + (j & 3) * 8;

    f32x16 acc[2][CIBG][COBG];
#pragma unroll
    for (int k = 0; k < 2; ++k)
#pragma unroll
        for (int a = 0; a < CIBG; ++a)
#pragma unroll
            for (int b = 0; b < COBG; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[k][a][b][i] = 0.f;
    float dbacc[COBG];
#pragma unroll
    for (int b = 0; b < COBG; ++b) dbacc[b] = 0.f;

    const int t0 = split * p.tbase + (split < p.trem ? split : p.trem);
    const int nt = p.tbase + (split < p.trem ? 1 : 0);

    auto issue = [&](int tile, int buf, bool on) __attribute__((always_inline)) {
        unsigned q = (unsigned)(on ? tile : 0);
        const int twi = (int)(q % (unsigned)p.ntw);
        q /= (unsigned)p.ntw;
        const int thi = (int)(q % (unsigned)p.nth);
        q /= (unsigned)p.nth;
        const int tdi = (int)(q % (unsigned)p.ntd);
        const int n = (int)(q / (unsigned)p.ntd);
        const int d0 = tdi * TD, h0 = thi * TH, w0 = twi * TW;
        const unsigned char *xb = reinterpret_cast<const unsigned char *>(
            p.x + ((((int64_t)n * p.D + d0) * p.H + h0) * p.W + w0) * p.cin);
        const unsigned char *gb = reinterpret_cast<const unsigned char *>(
            p.dy + ((((int64_t)n * D2 + 2 * d0) * H2 + 2 * h0) * W2 + 2 * w0) * p.cout);
        const unsigned sb = lds0 + buf * STB;
#pragma unroll
        for (int k = 0; k < XK; ++k) {
            const int ld = xco[k] & 255, lh = (xco[k] >> 8) & 255, lw = xco[k] >> 16;
            const bool grp = on && ((xsl >> k) & 1);
            const bool in = grp && d0 + ld < p.D && h0 + lh < p.H && w0 + lw < p.W;
            dma16(grp ? sb + (wv + 4 * k) * 1024 : dump, in ? xb + xoff[k] : zero);
        }
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            const int ld = gco[k] & 255, lh = (gco[k] >> 8) & 255, lw = gco[k] >> 16;
            const bool in = on && 2 * d0 + ld < D2 && 2 * h0 + lh < H2 && 2 * w0 + lw < W2;
            dma16(on ? sb + CIBG * XB + (wv + 4 * k) * 1024 : dump, in ? gb + goff[k] : zero);
        }
    };

    // prologue: the first two tiles; afterwards stage i fetches tile i + 2
    issue(t0, 0, nt > 0);
    issue(t0 + 1, 1, nt > 1);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(OPS) : "memory");
    __syncthreads();
    int buf = 0;
    for (int i = 0; i < nt; ++i) {
        {
            int nb = buf + 2;
            if (nb >= NST) nb -= NST;
            issue(t0 + i + 2, nb, i + 2 < nt);
        }
        const unsigned char *st = smem + buf * STB;
#pragma unroll
        for (int s = 0; s < 2; ++s) {   // K-step s: input voxels (d = s, h = hb, w = 0..7)
            bf16x8 ax[CIBG], bg[2][COBG];
#pragma unroll
            for (int a = 0; a < CIBG; ++a) {
                const int o = a * XB + lane_x + s * (TH * TW * 64);
                ax[a] = up_tr_pair(st, o, o + 4 * 64);
            }
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int b = 0; b < COBG; ++b) {
                    const int o = b * GB + lane_g + s * (2 * 64 * 64) + k * 64;
                    bg[k][b] = up_tr_pair(st, o, o + 8 * 64);
                }
#pragma unroll
            for (int k = 0; k < 2; ++k)
#pragma unroll
                for (int b = 0; b < COBG; ++b) {
#pragma unroll
                    for (int a = 0; a < CIBG; ++a)
                        acc[k][a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax[a], bg[k][b], acc[k][a][b], 0, 0, 0);
                    float sum = 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) sum += (float)bg[k][b][e];
                    dbacc[b] += sum;
                }
        }
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(OPS) : "memory");
        __syncthreads();
        if (++buf == NST) buf = 0;
    }

    float *out = p.ws + (int64_t)split * p.per_split;
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int tap = (ti * 2 + tj) * 2 + k;
#pragma unroll
        for (int a = 0; a < CIBG; ++a)
#pragma unroll
            for (int b = 0; b < COBG; ++b) {
                const int co = (cog * COBG + b) * 32 + (lane & 31);
                float *o = out + ((int64_t)tap * p.cin + (cig * CIBG + a) * 32 + hb * 4) * p.cout + co;
#pragma unroll
                for (int i = 0; i < 16; ++i) o[((i >> 2) * 8 + (i & 3)) * p.cout] = acc[k][a][b][i];
            }
    }
    if (cig == 0) {   // bias gradient: lane halves, then the four waves, in a fixed order
#pragma unroll
        for (int b = 0; b < COBG; ++b) {
            const float other = __shfl_xor(dbacc[b], 32);
            if (hb == 0) dbs[wv * (COBG * 32) + b * 32 + lane] = dbacc[b] + other;
        }
        __syncthreads();
        if (tid < COBG * 32) {
            const int n32 = COBG * 32;
            out[(int64_t)8 * p.cin * p.cout + cog * n32 + tid] = ((dbs[tid] + dbs[n32 + tid]) + dbs[2 * n32 + tid]) + dbs[3 * n32 + tid];
        }
    }
}

// ------------------------------------------------------------------ direct kernels
template <typename T>
__global__ __launch_bounds__(256) void up_fwd_direct_kernel(const T *__restrict__ x, const T *__restrict__ w,
                                                           const float *__restrict__ bias, T *__restrict__ y,
                                                           int64_t total, int D, int H, int W, int cin, int cout)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;  // over output elements; D,H,W are input sizes
    if (gid >= total) return;
    int co = (int)(gid % cout);
    int64_t o = gid / cout;
    int ow = (int)(o % (2 * W));
    int oh = (int)((o / (2 * W)) % (2 * H));
    int od = (int)((o / ((int64_t)4 * W * H)) % (2 * D));
    int64_t n = o / ((int64_t)8 * W * H * D);
    int tap = ((od & 1) * 2 + (oh & 1)) * 2 + (ow & 1);
    int64_t v = ((n * D + (od >> 1)) * H + (oh >> 1)) * (int64_t)W + (ow >> 1);
    float acc = bias ? bias[co] : 0.f;
    const T *xp = x + v * cin;
    const T *wp = w + (int64_t)tap * cin * cout + co;
    for (int ci = 0; ci < cin; ++ci) acc += elem<T>::ld(xp + ci) * elem<T>::ld(wp + (int64_t)ci * cout);
    elem<T>::st(y + gid, acc);
}

template <typename T>
__global__ __launch_bounds__(256) void up_dgrad_direct_kernel(const T *__restrict__ dy, const T *__restrict__ w,
                                                             T *__restrict__ dx, const T *__restrict__ omask,
                                                             int64_t total, int D, int H, int W, int cin, int cout)
{
    int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (gid >= total) return;
    int ci = (int)(gid % cin);
    int64_t v = gid / cin;
    int ww = (int)(v % W);
    int hh = (int)((v / W) % H);
    int dd = (int)((v / ((int64_t)W * H)) % D);
    int64_t n = v / ((int64_t)W * H * D);
    float acc = 0.f;
    for (int t = 0; t < 8; ++t) {
        int64_t o = ((n * 2 * D + 2 * dd + (t >> 2)) * 2 * H + 2 * hh + ((t >> 1) & 1)) * (2 * (int64_t)W) + 2 * ww + (t & 1);
        const T *gp = dy + o * cout;
        const T *wp = w + ((int64_t)t * cin + ci) * cout;
        for (int co = 0; co < cout; ++co) acc += elem<T>::ld(gp + co) * elem<T>::ld(wp + co);
    }
    if (omask && !(elem<T>::ld(omask + gid) > 0.f)) acc = 0.f;
    elem<T>::st(dx + gid, acc);
}

constexpr int UW_CIB = 8;
// block (split, ci-block, co-block): thread owns channel co and every (256/CB)-th input voxel
template <typename T>
__global__ __launch_bounds__(256) void up_wgrad_direct_kernel(const T *__restrict__ x, const T *__restrict__ dy,
                                                             float *__restrict__ ws, int64_t V, int D, int H, int W,
                                                             int cin, int cout, int CB, int64_t slab, int64_t per_split)
{
    __shared__ float red[256];
    int tid = threadIdx.x;
    int nvs = 256 / CB;
    int cl = tid % CB, vs = tid / CB;
    int co = blockIdx.z * CB + cl;
    bool active = (vs < nvs) && (co < cout);
    int ci0 = blockIdx.y * UW_CIB;
    int64_t v0 = (int64_t)blockIdx.x * slab;
    int64_t v1 = v0 + slab < V ? v0 + slab : V;
    float acc[8][UW_CIB];
    float accb = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int c = 0; c < UW_CIB; ++c) acc[t][c] = 0.f;
    if (active) {
        for (int64_t v = v0 + vs; v < v1; v += nvs) {
            int ww = (int)(v % W);
            int hh = (int)((v / W) % H);
            int dd = (int)((v / ((int64_t)W * H)) % D);
            int64_t n = v / ((int64_t)W * H * D);
            float xv[UW_CIB];
#pragma unroll
            for (int c = 0; c < UW_CIB; ++c) xv[c] = (ci0 + c < cin) ? elem<T>::ld(x + v * cin + ci0 + c) : 0.f;
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                int64_t o = ((n * 2 * D + 2 * dd + (t >> 2)) * 2 * H + 2 * hh + ((t >> 1) & 1)) * (2 * (int64_t)W) + 2 * ww + (t & 1);
                float g = elem<T>::ld(dy + o * cout + co);
                accb += g;
#pragma unroll
                for (int c = 0; c < UW_CIB; ++c) acc[t][c] += xv[c] * g;
            }
        }
    }
    float *out = ws + (int64_t)blockIdx.x * per_split;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int c = 0; c < UW_CIB; ++c) {
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
            out[(int64_t)8 * cin * cout + co] = s;
        }
    }
}

static int64_t up_direct_nsplit(int64_t V)
{
    int64_t s = V / 256;
    return s < 1 ? 1 : (s > 1024 ? 1024 : s);
}

static void up_wgrad_plan(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout, int64_t *ntiles,
                          int *nsplit, int *cibg, int *cobg)
{
    *ntiles = N * ((D + uw::TD - 1) / uw::TD) * ((H + uw::TH - 1) / uw::TH) * ((W + uw::TW - 1) / uw::TW);
    const int64_t nci = cin / 32, nco = cout / 32;
    *cibg = nci % 4 == 0 ? 4 : (nci % 2 == 0 ? 2 : 1);
    *cobg = nco % 2 == 0 ? 2 : 1;
    int64_t yz = (nci / *cibg) * (nco / *cobg);
    int64_t s = 256 / yz;   // one persistent workgroup per CU in total
    if (s < 1) s = 1;
    if (s > *ntiles) s = *ntiles;
    *nsplit = (int)s;
}

template <int CIBG, int COBG>
static int launch_up_wgrad(const UpWgradParams &p, dim3 grid, hipStream_t st)
{
    constexpr int lds = uw::lds_bytes(CIBG, COBG);
    static_assert(lds <= 160 * 1024, "LDS budget");
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&up_wgrad_pipe_kernel<CIBG, COBG>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    up_wgrad_pipe_kernel<CIBG, COBG><<<grid, 256, lds, st>>>(p);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

}  // namespace k3

using namespace k3;

extern "C" {

int k3_upconv3d_packed_bytes(int64_t cin, int64_t cout, int dtype, size_t *bytes)
{
    if (!bytes || cin <= 0 || cout <= 0 || (dtype != K3_BF16 && dtype != K3_F32)) return K3_E_BADARG;
    *bytes = up_mfma_ok(dtype, cin, cout) ? (size_t)2 * 8 * cin * cout * sizeof(bf16_t) : 0;
    return K3_OK;
}

int k3_upconv3d_pack_weights(const void *w, int64_t cin, int64_t cout, int dtype, void *packed, size_t packed_bytes,
                             void *stream)
{
    size_t need = 0;
    int rc = k3_upconv3d_packed_bytes(cin, cout, dtype, &need);
    if (rc != K3_OK) return rc;
    if (need == 0) return K3_OK;
    if (!w || !packed) return K3_E_BADARG;
    if (packed_bytes < need) return K3_E_WORKSPACE;
    int64_t total = 2 * 8 * cin * cout;
    up_pack_kernel<<<dim3((unsigned)((total + 255) / 256)), 256, 0, (hipStream_t)stream>>>((const bf16_t *)w, (bf16_t *)packed,
                                                                                         (int)cin, (int)cout);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

static int up_check(const k3_tensor *xd, const k3_tensor *yd)
{
    if (!desc_ok(xd) || !desc_ok(yd)) return K3_E_BADARG;
    if (yd->n != xd->n || yd->d != 2 * xd->d || yd->h != 2 * xd->h || yd->w != 2 * xd->w || yd->dtype != xd->dtype)
        return K3_E_SHAPE;
    if (yd->d > 0x3fffffff || yd->h > 0x3fffffff || yd->w > 0x3fffffff || xd->c > 0x3fffffff || yd->c > 0x3fffffff)
        return K3_E_UNSUPPORTED;
    return K3_OK;
}

int k3_upconv3d_fwd(const k3_tensor *xd, const void *x, const void *w, const void *packed, const float *bias,
                    const k3_tensor *yd, void *y, void *stream)
{
    int rc = up_check(xd, yd);
    if (rc != K3_OK) return rc;
    if (!x || !w || !y) return K3_E_BADARG;
    hipStream_t st = (hipStream_t)stream;
    int64_t V = voxels(xd);
    int cin = (int)xd->c, cout = (int)yd->c;
    if (up_mfma_ok(xd->dtype, cin, cout)) {
        if (!packed) return K3_E_BADARG;
        int64_t blocks = (V + 127) / 128;
        if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
        rc = up_fwd_lds_dispatch((const bf16_t *)x, (const bf16_t *)packed, bias, (bf16_t *)y, V, (int)xd->d, (int)xd->h,
                                 (int)xd->w, cin, cout, st);
        if (rc != K3_E_UNSUPPORTED) return rc;
        up_fwd_mfma_kernel<<<dim3((unsigned)blocks, (unsigned)(cout / 32)), 256, 0, st>>>(
            (const bf16_t *)x, (const bf16_t *)packed, bias, (bf16_t *)y, V, (int)xd->d, (int)xd->h, (int)xd->w, cin, cout);
        K3_LAUNCH_CHECK();
        return K3_OK;
    }
    int64_t total = V * 8 * cout;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    if (xd->dtype == K3_F32)
        up_fwd_direct_kernel<float><<<dim3((unsigned)blocks), 256, 0, st>>>((const float *)x, (const float *)w, bias, (float *)y,
                                                                            total, (int)xd->d, (int)xd->h, (int)xd->w, cin, cout);
    else
        up_fwd_direct_kernel<bf16_t><<<dim3((unsigned)blocks), 256, 0, st>>>((const bf16_t *)x, (const bf16_t *)w, bias,
                                                                             (bf16_t *)y, total, (int)xd->d, (int)xd->h,
                                                                             (int)xd->w, cin, cout);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

int k3_upconv3d_bwd_data(const k3_tensor *dyd, const void *dy, const void *w, const void *packed, const k3_tensor *dxd,
                         void *dx, const void *dx_mask, void *stream)
{
    int rc = up_check(dxd, dyd);
    if (rc != K3_OK) return rc;
    if (!dy || !w || !dx) return K3_E_BADARG;
    hipStream_t st = (hipStream_t)stream;
    int64_t V = voxels(dxd);
    int cin = (int)dxd->c, cout = (int)dyd->c;
    int D = (int)dxd->d, H = (int)dxd->h, W = (int)dxd->w;
    if (up_mfma_ok(dxd->dtype, cin, cout)) {
        if (!packed) return K3_E_BADARG;
        const bf16_t *pb = (const bf16_t *)packed + (int64_t)8 * cin * cout;
        int64_t blocks = (V + 127) / 128;
        if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
        int nb = cin / 32;
        rc = up_dgrad_lds_dispatch((const bf16_t *)dy, pb, (bf16_t *)dx, (const bf16_t *)dx_mask, V, D, H, W, cin, cout, st);
        if (rc != K3_E_UNSUPPORTED) return rc;
        if (up_dgrad_tap_dispatch((const bf16_t *)dy, pb, (bf16_t *)dx, (const bf16_t *)dx_mask, V, D, H, W, cin, cout, st)) {
            K3_LAUNCH_CHECK();
            return K3_OK;
        }
        if (nb % 4 == 0)
            up_dgrad_mfma_kernel<4><<<dim3((unsigned)blocks, (unsigned)(nb / 4)), 256, 0, st>>>((const bf16_t *)dy, pb, (bf16_t *)dx, (const bf16_t *)dx_mask, V, D, H, W, cin, cout);
        else if (nb % 2 == 0)
            up_dgrad_mfma_kernel<2><<<dim3((unsigned)blocks, (unsigned)(nb / 2)), 256, 0, st>>>((const bf16_t *)dy, pb, (bf16_t *)dx, (const bf16_t *)dx_mask, V, D, H, W, cin, cout);
        else
            up_dgrad_mfma_kernel<1><<<dim3((unsigned)blocks, (unsigned)nb), 256, 0, st>>>((const bf16_t *)dy, pb, (bf16_t *)dx, (const bf16_t *)dx_mask, V, D, H, W, cin, cout);
        K3_LAUNCH_CHECK();
        return K3_OK;
    }
    int64_t total = V * cin;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    if (dxd->dtype == K3_F32)
        up_dgrad_direct_kernel<float><<<dim3((unsigned)blocks), 256, 0, st>>>((const float *)dy, (const float *)w, (float *)dx, (const float *)dx_mask, total, D, H, W, cin, cout);
    else
        up_dgrad_direct_kernel<bf16_t><<<dim3((unsigned)blocks), 256, 0, st>>>((const bf16_t *)dy, (const bf16_t *)w, (bf16_t *)dx, (const bf16_t *)dx_mask, total, D, H, W, cin, cout);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

int k3_upconv3d_bwd_weight_workspace_bytes(const k3_tensor *xd, const k3_tensor *dyd, size_t *bytes)
{
    int rc = up_check(xd, dyd);
    if (rc != K3_OK) return rc;
    if (!bytes) return K3_E_BADARG;
    int64_t cin = xd->c, cout = dyd->c;
    int64_t per = 8 * cin * cout + cout;
    if (up_mfma_ok(xd->dtype, cin, cout)) {
        int64_t ntiles;
        int nsplit, cibg, cobg;
        up_wgrad_plan(xd->n, xd->d, xd->h, xd->w, cin, cout, &ntiles, &nsplit, &cibg, &cobg);
        *bytes = (size_t)nsplit * per * sizeof(float);
    } else {
        *bytes = (size_t)up_direct_nsplit(voxels(xd)) * per * sizeof(float);
    }
    return K3_OK;
}

int k3_upconv3d_bwd_weight(const k3_tensor *xd, const void *x, const k3_tensor *dyd, const void *dy, float *dW, float *db,
                           void *ws, size_t ws_bytes, void *stream)
{
    size_t need = 0;
    int rc = k3_upconv3d_bwd_weight_workspace_bytes(xd, dyd, &need);
    if (rc != K3_OK) return rc;
    if (!x || !dy || !dW || !ws) return K3_E_BADARG;
    if (ws_bytes < need) return K3_E_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    int64_t V = voxels(xd);
    int cin = (int)xd->c, cout = (int)dyd->c;
    int D = (int)xd->d, H = (int)xd->h, W = (int)xd->w;
    int64_t per = (int64_t)8 * cin * cout + cout;
    if (up_mfma_ok(xd->dtype, cin, cout)) {
        int64_t ntiles;
        int nsplit, cibg, cobg;
        up_wgrad_plan(xd->n, D, H, W, cin, cout, &ntiles, &nsplit, &cibg, &cobg);
        // 32-bit byte offsets inside a tile and 32-bit tile counts
        if (ntiles > 0x3fffffffLL || (int64_t)4 * (2 * H) * (2 * W) * cout * 2 > 0x7fffffffLL ||
            (int64_t)2 * H * W * cin * 2 > 0x7fffffffLL)
            return K3_E_UNSUPPORTED;
        UpWgradParams p{};
        p.x = (const bf16_t *)x; p.dy = (const bf16_t *)dy; p.ws = (float *)ws; p.per_split = per;
        p.N = (int)xd->n; p.D = D; p.H = H; p.W = W; p.cin = cin; p.cout = cout;
        p.ntd = (D + uw::TD - 1) / uw::TD; p.nth = (H + uw::TH - 1) / uw::TH; p.ntw = (W + uw::TW - 1) / uw::TW;
        p.ntiles = (int)ntiles; p.nsplit = nsplit; p.tbase = p.ntiles / nsplit; p.trem = p.ntiles % nsplit;
        dim3 grid((unsigned)nsplit, (unsigned)(cin / 32 / cibg), (unsigned)(cout / 32 / cobg));
        if (cibg == 4 && cobg == 2) rc = launch_up_wgrad<4, 2>(p, grid, st);
        else if (cibg == 4) rc = launch_up_wgrad<4, 1>(p, grid, st);
        else if (cibg == 2 && cobg == 2) rc = launch_up_wgrad<2, 2>(p, grid, st);
        else if (cibg == 2) rc = launch_up_wgrad<2, 1>(p, grid, st);
        else if (cobg == 2) rc = launch_up_wgrad<1, 2>(p, grid, st);
        else rc = launch_up_wgrad<1, 1>(p, grid, st);
        if (rc != K3_OK) return rc;
        return launch_reduce_partials((const float *)ws, dW, db, (int64_t)8 * cin * cout, per, nsplit, st);
    }
    int64_t nsplit = up_direct_nsplit(V);
    int64_t slab = (V + nsplit - 1) / nsplit;
    int CB = cout < 256 ? cout : 256;
    dim3 grid((unsigned)nsplit, (unsigned)((cin + UW_CIB - 1) / UW_CIB), (unsigned)((cout + CB - 1) / CB));
    if (grid.y > 65535 || grid.z > 65535) return K3_E_UNSUPPORTED;
    if (xd->dtype == K3_F32)
        up_wgrad_direct_kernel<float><<<grid, 256, 0, st>>>((const float *)x, (const float *)dy, (float *)ws, V, D, H, W, cin, cout, CB, slab, per);
    else
        up_wgrad_direct_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t *)x, (const bf16_t *)dy, (float *)ws, V, D, H, W, cin, cout, CB, slab, per);
    K3_LAUNCH_CHECK();
    return launch_reduce_partials((const float *)ws, dW, db, (int64_t)8 * cin * cout, per, (int)nsplit, st);
}

}  // extern "C"
