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

static __device__ uint4 g_fzero[4];   // zero-initialised: source of out-of-volume copy items

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
// (the tile count fits 31 bits, checked at launch: 32-bit divisions, a fraction of the 64-bit ones' cost)
__device__ __forceinline__ FirstTile first_tile(int64_t tile64, int ntd, int nth, int ntw)
{
    FirstTile t;
    unsigned tile = (unsigned)tile64;
    t.w0 = (int)(tile % (unsigned)ntw) * first::TW;
    tile /= (unsigned)ntw;
    t.h0 = (int)(tile % (unsigned)nth) * first::TH;
    tile /= (unsigned)nth;
    t.d0 = (int)(tile % (unsigned)ntd) * first::TD;
    t.n = (int)(tile / (unsigned)ntd);
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

// ---------------------------------------------------------------------------- MFMA variants
// For C_out a multiple of 32 both passes run on the matrix cores with the 27 taps as the
// contraction (forward) or as the 32 output rows (backward-weight); the single-channel halo
// tile sits in LDS as bf16 and the im2col operand of a lane is gathered from it with eight
// 16-bit LDS reads.  The thread-per-channel kernels above need 27 LDS reads and 108 FMAs per
// 4 outputs and are LDS-bound at ~1.5-1.9 TB/s; these stream at the HBM rate.
namespace firstm {
constexpr int TD = 4, TH = 8, TW = 16;
constexpr int HD = TD + 2, HH = TH + 2, HW = TW + 2;
constexpr int NHALO = HD * HH * HW;               // 1080 bf16 values
constexpr int NVOX = TD * TH * TW;                // 512 = 16 patches of 2 rows x 16 columns
__host__ __device__ constexpr int tapoff(int t) { return (((t / 9) * HH + (t / 3) % 3) * HW + t % 3) * 2; }   // bytes
}  // namespace firstm

__host__ __device__ static inline int first_row_to_channel(int r) { return ((r >> 2) & 1) * 16 + (r >> 3) * 4 + (r & 3); }

__device__ __forceinline__ void stage_x_bf16(const bf16_t *__restrict__ x, bf16_t *xs, const FirstTile &t, int D, int H, int W)
{
    using namespace firstm;
    for (int i = threadIdx.x; i < NHALO; i += 256) {
        int lw = i % HW, lh = (i / HW) % HH, ld = i / (HW * HH);
        int gd = t.d0 + ld - 1, gh = t.h0 + lh - 1, gw = t.w0 + lw - 1;
        bf16_t v = 0;
        if (gd >= 0 && gd < D && gh >= 0 && gh < H && gw >= 0 && gw < W) v = x[(((int64_t)t.n * D + gd) * H + gh) * W + gw];
        xs[i] = v;
    }
}

// The same in two halves, so that the loads of the next tile are in flight while the current tile is
// computed: a thread holds its (at most) five halo values in registers in between.  Loads and stores
// of a wave complete in issue order on one counter, so everything between the two halves must be
// straight-line code (no conditional memory operation): the compiler can then wait for exactly these
// loads and leave the tile's later stores in flight; behind a branch it would wait for everything.
constexpr int FIRST_XPT = (firstm::NHALO + 255) / 256;
constexpr int FIRST_XS = FIRST_XPT * 256;   // entries of a halo buffer: every thread stores all its values (zeros beyond the tile)
struct FirstHaloRegs {
    bf16_t v[FIRST_XPT];
    unsigned inside;   // bit k: value k lies inside the volume (else a zero is stored)
};
__device__ __forceinline__ void load_x_regs(const bf16_t *__restrict__ x, FirstHaloRegs &r, const FirstTile &t, int D, int H, int W)
{
    using namespace firstm;
    r.inside = 0;
#pragma unroll
    for (int k = 0; k < FIRST_XPT; ++k) {
        const int i = threadIdx.x + k * 256;
        const int lw = i % HW, lh = (i / HW) % HH, ld = i / (HW * HH);
        const int gd = t.d0 + ld - 1, gh = t.h0 + lh - 1, gw = t.w0 + lw - 1;
        // every lane loads from a clamped (valid) position, and what lies outside is replaced by zero only
        // when the values are stored: no branch and no use of a loaded value here, so the loads leave back
        // to back and the only wait is in store_x_regs
        const int cd = gd < 0 ? 0 : (gd < D ? gd : D - 1), ch = gh < 0 ? 0 : (gh < H ? gh : H - 1), cw = gw < 0 ? 0 : (gw < W ? gw : W - 1);
        r.v[k] = x[(((int64_t)t.n * D + cd) * H + ch) * W + cw];
        r.inside |= (i < NHALO && cd == gd && ch == gh && cw == gw ? 1u : 0u) << k;
    }
}
__device__ __forceinline__ void store_x_regs(bf16_t *xs, const FirstHaloRegs &r)
{
#pragma unroll
    for (int k = 0; k < FIRST_XPT; ++k)   // unconditional stores (the buffer is padded): a load whose use is conditional sinks to it
        xs[threadIdx.x + k * 256] = (r.inside >> k) & 1u ? r.v[k] : (bf16_t)0;
}

// eight halo values at byte offsets o0..o7 from p, packed as an MFMA operand
template <int O0, int O1, int O2, int O3, int O4, int O5, int O6, int O7>
__device__ __forceinline__ bf16x8 gather8(const unsigned char *p)
{
    typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;
    u16x8 v;
    v[0] = *reinterpret_cast<const unsigned short *>(p + O0);
    v[1] = *reinterpret_cast<const unsigned short *>(p + O1);
    v[2] = *reinterpret_cast<const unsigned short *>(p + O2);
    v[3] = *reinterpret_cast<const unsigned short *>(p + O3);
    v[4] = *reinterpret_cast<const unsigned short *>(p + O4);
    v[5] = *reinterpret_cast<const unsigned short *>(p + O5);
    v[6] = *reinterpret_cast<const unsigned short *>(p + O6);
    v[7] = *reinterpret_cast<const unsigned short *>(p + O7);
    return __builtin_bit_cast(bf16x8, v);
}
// The same with volatile reads, for scattered offsets: left to itself the compiler merges taps that are
// neighbours in w into 4-byte reads at 2-byte-aligned addresses, which the LDS serves far slower than
// separate 2-byte reads (forward pass, 32 channels: 75 -> 55 us at 128^3).  A run of eight consecutive values
// (backward-weight) is better served by the merged wide read.
template <int O0, int O1, int O2, int O3, int O4, int O5, int O6, int O7>
__device__ __forceinline__ bf16x8 gather8_scattered(const unsigned char *p)
{
    typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;
    u16x8 v;
    v[0] = *reinterpret_cast<const volatile unsigned short *>(p + O0);
    v[1] = *reinterpret_cast<const volatile unsigned short *>(p + O1);
    v[2] = *reinterpret_cast<const volatile unsigned short *>(p + O2);
    v[3] = *reinterpret_cast<const volatile unsigned short *>(p + O3);
    v[4] = *reinterpret_cast<const volatile unsigned short *>(p + O4);
    v[5] = *reinterpret_cast<const volatile unsigned short *>(p + O5);
    v[6] = *reinterpret_cast<const volatile unsigned short *>(p + O6);
    v[7] = *reinterpret_cast<const volatile unsigned short *>(p + O7);
    return __builtin_bit_cast(bf16x8, v);
}

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// Forward: D[co][voxel] = sum_tap W[tap][co] * x[voxel + tap]; K = 32 (27 taps + 5 zero rows) = 2 MFMAs
// per 32 voxels and 32-channel block.  Persistent blocks walk the 4x8x16 tiles.
template <int MB, bool BITS>
__global__ __launch_bounds__(256, MB <= 2 ? 4 : 3) void conv_first_fwd_mfma_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ w,
                                                                 const float *__restrict__ bias, int relu,
                                                                 bf16_t *__restrict__ y, unsigned short *__restrict__ ybits,
                                                                 int D, int H, int W, int ntd, int nth, int ntw,
                                                                 int64_t ntiles)
{
    using namespace firstm;
    constexpr int cout = 32 * MB;
    __shared__ __attribute__((aligned(16))) bf16_t xs[2][FIRST_XS];
    // A wave's results pass through LDS on their way out: the accumulator layout gives a lane 32 bytes of
    // one voxel, so a store instruction would write 64 separate 16-byte pieces; read back row-major, a
    // store instruction writes whole runs of voxels (1 KB per half row of a patch).  Rows are padded by 16
    // bytes against bank conflicts.  Private to the wave: no barrier, LDS operations of a wave are in order.
    constexpr int ROWB = 64 * MB, ROWP = ROWB + 16;
    constexpr int LPVX = ROWB / 16, VPI = 64 / LPVX;       // lanes per voxel / voxels per store instruction when reading back
    __shared__ __attribute__((aligned(16))) unsigned char ost[4][32 * ROWP];
    __shared__ __attribute__((aligned(16))) unsigned short obits[4][32 * 2 * MB];   // the bit words of a patch, voxel-major
    __shared__ __attribute__((aligned(16))) float bl[cout];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int hb = lane >> 5, vl = lane & 31;
    for (int i = threadIdx.x; i < cout; i += 256) bl[i] = bias ? bias[i] : 0.f;
    // A operand: weights, rows permuted so that a lane ends up with 16 consecutive channels
    bf16x8 aw[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;
            u16x8 v;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int tap = m * 16 + hb * 8 + e;
                v[e] = tap < 27 ? w[(int64_t)tap * cout + mb * 32 + first_row_to_channel(vl)] : (unsigned short)0;
            }
            aw[mb][m] = __builtin_bit_cast(bf16x8, v);
        }
    const float floor_ = relu ? 0.f : -__builtin_inff();
    unsigned char *ow = ost[wv];
    int buf = 0;
    if ((int64_t)blockIdx.x < ntiles) stage_x_bf16(x, xs[0], first_tile(blockIdx.x, ntd, nth, ntw), D, H, W);
    __syncthreads();
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x, buf ^= 1) {
        const FirstTile t = first_tile(tile, ntd, nth, ntw);
        // The next tile's halo is requested now and stored to the other buffer behind this tile's work
        // (that buffer was last read before the barrier that ended the previous iteration).  The last
        // tile requests itself again: the loop body has no conditional memory operation (see load_x_regs).
        const bool more = tile + gridDim.x < ntiles;
        FirstHaloRegs xnext;
        load_x_regs(x, xnext, first_tile(more ? tile + gridDim.x : tile, ntd, nth, ntw), D, H, W);
        // results leave through descriptors at the tile's first voxel: a lane whose voxel lies outside the
        // volume gets an offset beyond the range, and such stores are dropped
        const int64_t origin = (((int64_t)t.n * D + t.d0) * H + t.h0) * W + t.w0;
        __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc(y + origin * cout, 0, 0x7ffffff0, 0x00020000);
        __amdgpu_buffer_rsrc_t brs = __builtin_amdgcn_make_buffer_rsrc(BITS ? ybits + origin * (cout / 16) : (unsigned short *)y, 0,
                                                                       0x7ffffff0, 0x00020000);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int patch = wv * 4 + q;                 // 16 patches: depth plane patch / 4, rows 2 * (patch % 4) ..+1
            const int ld = patch >> 2, lh = (patch & 3) * 2 + (vl >> 4), lw = vl & 15;
            const unsigned char *p = reinterpret_cast<const unsigned char *>(xs[buf]) + ((ld * HH + lh) * HW + lw) * 2;
            // taps 0-7 / 8-15 (first K chunk) and 16-23 / 24-26 (second), by lane half
            const bf16x8 lo0 = gather8_scattered<tapoff(0), tapoff(1), tapoff(2), tapoff(3), tapoff(4), tapoff(5), tapoff(6), tapoff(7)>(p);
            const bf16x8 hi0 = gather8_scattered<tapoff(8), tapoff(9), tapoff(10), tapoff(11), tapoff(12), tapoff(13), tapoff(14), tapoff(15)>(p);
            const bf16x8 lo1 = gather8_scattered<tapoff(16), tapoff(17), tapoff(18), tapoff(19), tapoff(20), tapoff(21), tapoff(22), tapoff(23)>(p);
            bf16x8 hi1;                                         // taps 24-26; rows 27-31 of the contraction do not exist
            {
                typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;
                u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
                v[0] = *reinterpret_cast<const volatile unsigned short *>(p + tapoff(24));
                v[1] = *reinterpret_cast<const volatile unsigned short *>(p + tapoff(25));
                v[2] = *reinterpret_cast<const volatile unsigned short *>(p + tapoff(26));
                hi1 = __builtin_bit_cast(bf16x8, v);
            }
            const bf16x8 b0 = hb ? hi0 : lo0, b1 = hb ? hi1 : lo1;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                f32x16 acc;
                {
                    const f32x4 *bq = reinterpret_cast<const f32x4 *>(bl + mb * 32 + hb * 16);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const f32x4 qv = bq[i];
                        acc[4 * i] = qv[0]; acc[4 * i + 1] = qv[1]; acc[4 * i + 2] = qv[2]; acc[4 * i + 3] = qv[3];
                    }
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aw[mb][0], b0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aw[mb][1], b1, acc, 0, 0, 0);
                float v[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) v[i] = fmaxf(acc[i], floor_);
                const uint32_t dd[8] = {pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]), pack2bf(v[6], v[7]),
                                        pack2bf(v[8], v[9]), pack2bf(v[10], v[11]), pack2bf(v[12], v[13]), pack2bf(v[14], v[15])};
                uint4 *od = reinterpret_cast<uint4 *>(ow + vl * ROWP + mb * 64 + hb * 32);
                od[0] = make_uint4(dd[0], dd[1], dd[2], dd[3]);
                od[1] = make_uint4(dd[4], dd[5], dd[6], dd[7]);
                if (BITS)   // one bit per stored element: set where it is > 0
                    obits[wv][vl * (2 * MB) + mb * 2 + hb] = (unsigned short)relu_bits16(dd);
            }
            // read the patch back row-major: instruction k carries voxels k * VPI ... of the patch (voxel j:
            // row j / 16, column j % 16 of the patch's two rows), LPVX lanes of 16 bytes per voxel
#pragma unroll
            for (int k = 0; k < 32 / VPI; ++k) {
                const int j = k * VPI + lane / LPVX, piece = lane % LPVX;
                const int jh = (patch & 3) * 2 + (j >> 4), jw = j & 15;
                const bool jin = t.d0 + ld < D && t.h0 + jh < H && t.w0 + jw < W;
                const int voff = jin ? (((ld * H + jh) * W + jw) * cout) * 2 + piece * 16 : -1;
                uint4 d = *reinterpret_cast<const uint4 *>(ow + j * ROWP + piece * 16);
                __builtin_amdgcn_raw_buffer_store_b128(u32x4{d.x, d.y, d.z, d.w}, yrs, voff, 0, 0);
                // With several waves on a SIMD a 16-byte buffer store still reads its data registers a few
                // cycles after it has issued; the two wait states the compiler leaves before the next write
                // of such a register were not enough (single lanes stored a later value at 4 x 320^3).
                // Keep the registers untouched for eight more cycles.
                asm volatile("s_nop 7" : "+v"(d.x), "+v"(d.y), "+v"(d.z), "+v"(d.w));
            }
            if (BITS) {   // lane j < 32 stores the 2 * MB bit words of voxel j in one piece
                const int j = lane & 31, jh = (patch & 3) * 2 + (j >> 4), jw = j & 15;
                const bool jin = lane < 32 && t.d0 + ld < D && t.h0 + jh < H && t.w0 + jw < W;
                const int boff = jin ? ((ld * H + jh) * W + jw) * (cout / 8) : -1;
                const unsigned short *ob = &obits[wv][j * (2 * MB)];
                if (MB == 1) {
                    __builtin_amdgcn_raw_buffer_store_b32(*reinterpret_cast<const unsigned *>(ob), brs, boff, 0, 0);
                } else if (MB == 2) {
                    typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
                    const uint2 w2 = *reinterpret_cast<const uint2 *>(ob);
                    __builtin_amdgcn_raw_buffer_store_b64(u32x2{w2.x, w2.y}, brs, boff, 0, 0);
                } else {
                    uint4 w4 = *reinterpret_cast<const uint4 *>(ob);
                    __builtin_amdgcn_raw_buffer_store_b128(u32x4{w4.x, w4.y, w4.z, w4.w}, brs, boff, 0, 0);
                    asm volatile("s_nop 7" : "+v"(w4.x), "+v"(w4.y), "+v"(w4.z), "+v"(w4.w));
                }
            }
        }
        store_x_regs(xs[buf ^ 1], xnext);
        __syncthreads();
    }
}

// Backward-weight: rows = taps (row 27 multiplies ones: the bias gradient), columns = channels,
// contraction over voxels, 16 per MFMA (one row of the 16-wide tile).  dy tiles are copied
// global -> LDS asynchronously, double buffered, as [block][voxel][32 channels]; the dy operand
// comes from transposing LDS reads, the x operand from eight 16-bit reads of the halo tile.
// The four waves split the 32 rows of a tile and add their accumulators through LDS in a
// fixed order at the end; one partial per workgroup.
template <int MB>
__global__ __launch_bounds__(256) void conv_first_wgrad_mfma_kernel(const bf16_t *__restrict__ x, const bf16_t *__restrict__ dy,
                                                                   float *__restrict__ ws, int64_t per_split, int D, int H,
                                                                   int W, int ntd, int nth, int ntw, int64_t ntiles,
                                                                   int ctot, int coff)
{
    // This launch handles the 32 * MB channels [coff, coff + 32 * MB) of a layer with ctot channels.
    using namespace firstm;
    constexpr int GB = NVOX * 64;          // one 32-channel block of the dy tile
    constexpr int GSTAGE = MB * GB;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [2][GSTAGE] dy, then 2 x halo tiles, then 4 KB
    bf16_t *xs0 = reinterpret_cast<bf16_t *>(smem + 2 * GSTAGE);
    float *red = reinterpret_cast<float *>(smem + 2 * GSTAGE + 2 * FIRST_XS * 2);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hb = lane >> 5, r = lane & 31, g16 = (lane >> 4) & 1, j = lane & 15;
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned char *zero = reinterpret_cast<const unsigned char *>(g_fzero);
    // copy items of a dy tile: MB * 32 groups of 64 slots; wave wv copies groups wv, wv + 4, ...
    constexpr int GK = MB * 8;
    int goff[GK], gco[GK];
#pragma unroll
    for (int k = 0; k < GK; ++k) {
        const int slot = (wv + 4 * k) * 64 + lane;
        const int cb = slot >> 11, vox = (slot >> 2) & 511, part = slot & 3;
        const int ld = vox >> 7, lh = (vox >> 4) & 7, lw = vox & 15;
        goff[k] = ((ld * H + lh) * W + lw) * ctot * 2 + (coff + cb * 32) * 2 + part * 16;
        gco[k] = ld | (lh << 8) | (lw << 16);
    }
    auto issue_g = [&](int64_t tile, int buf) __attribute__((always_inline)) {
        const FirstTile t = first_tile(tile, ntd, nth, ntw);
        const unsigned char *gb = reinterpret_cast<const unsigned char *>(dy + ((((int64_t)t.n * D + t.d0) * H + t.h0) * W + t.w0) * ctot);
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            const int ld = gco[k] & 255, lh = (gco[k] >> 8) & 255, lw = gco[k] >> 16;
            const bool in = t.d0 + ld < D && t.h0 + lh < H && t.w0 + lw < W;
            dma16(lds0 + buf * GSTAGE + (wv + 4 * k) * 1024, in ? gb + goff[k] : zero);
        }
    };
    // this lane's row of the x operand: tap r (rows 27-31: address of tap 26, value replaced below)
    const int tap = r < 27 ? r : 26;
    const int xrow = tapoff(tap) + hb * 16;   // + 8 voxels for the upper lane half
    const int lane_g = (hb * 8 + (j >> 2)) * 64 + g16 * 32 + (j & 3) * 8;
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
    bf16x8 zeros8;
#pragma unroll
    for (int e = 0; e < 8; ++e) zeros8[e] = (__bf16)0.f;

    f32x16 acc[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[mb][i] = 0.f;

    int buf = 0;
    if ((int64_t)blockIdx.x < ntiles) {
        issue_g(blockIdx.x, 0);
        stage_x_bf16(x, xs0, first_tile(blockIdx.x, ntd, nth, ntw), D, H, W);
    }
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x, buf ^= 1) {
        bf16_t *xs = xs0 + buf * FIRST_XS;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();   // dy tile and halo tile of this stage are in LDS; the other buffers are free
        // the next tile: its dy copies and its halo loads are in flight while this tile is multiplied; the
        // halo values wait in registers and go to the other halo buffer behind the work
        const bool more = tile + gridDim.x < ntiles;
        FirstHaloRegs xnext;
        if (more) issue_g(tile + gridDim.x, buf ^ 1);
        load_x_regs(x, xnext, first_tile(more ? tile + gridDim.x : tile, ntd, nth, ntw), D, H, W);   // (the last tile: itself again, unused)
        const unsigned char *gs = smem + buf * GSTAGE;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int row = wv * 8 + q;            // K-step: depth plane row / 8, tile row row % 8, 16 voxels along w
            const int ld = row >> 3, lh = row & 7;
            const unsigned char *p = reinterpret_cast<const unsigned char *>(xs) + ((ld * HH + lh) * HW) * 2 + xrow;
            bf16x8 ax = gather8<0, 2, 4, 6, 8, 10, 12, 14>(p);
            if (r == 27) ax = ones;
            if (r > 27) ax = zeros8;
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) {
                const int o = mb * GB + (row * 16) * 64 + lane_g;
                typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
                s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(gs + o));
                s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(gs + o + 4 * 64));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax, __builtin_bit_cast(bf16x8, v), acc[mb], 0, 0, 0);
            }
        }
        store_x_regs(xs0 + (buf ^ 1) * FIRST_XS, xnext);
    }
    // add the four waves in wave order; acc[mb][i] is row (i/4)*8 + hb*4 + i%4, column mb*32 + lane%32
    float *out = ws + (int64_t)blockIdx.x * per_split;
    __syncthreads();
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int row = (i >> 2) * 8 + hb * 4 + (i & 3);
            __syncthreads();
            if (row < 28) red[wv * 64 + lane] = acc[mb][i];
            __syncthreads();
            if (wv == 0 && row < 28)
                out[(int64_t)row * ctot + coff + mb * 32 + (lane & 31)] = ((red[lane] + red[64 + lane]) + red[128 + lane]) + red[192 + lane];
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

static bool first_mfma_ok(const ConvArgs &a)
{
    // 32-bit byte offsets inside a tile
    return (a.cout == 32 || a.cout == 64 || a.cout == 128) && (int64_t)(first::TD + 1) * a.H * a.W * a.cout * 2 < 0x7fffffffLL;
}

template <int MB, bool BITS>
static void launch_first_fwd_mfma(const ConvArgs &a, int ntd, int nth, int ntw, int64_t ntiles, hipStream_t st)
{
    const unsigned grid = (unsigned)(ntiles < 2048 ? ntiles : 2048);
    conv_first_fwd_mfma_kernel<MB, BITS><<<dim3(grid), 256, 0, st>>>((const bf16_t *)a.x, (const bf16_t *)a.w, a.bias, a.relu,
                                                                    (bf16_t *)a.y, (unsigned short *)a.ybits, (int)a.D, (int)a.H,
                                                                    (int)a.W, ntd, nth, ntw, ntiles);
}

int conv_first_fwd(const ConvArgs &a, hipStream_t st)
{
    int ntd, nth, ntw;
    int64_t ntiles = first_tiles(a, &ntd, &nth, &ntw);
    if (ntiles > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    if (first_mfma_ok(a)) {
        const bool bits = a.ybits != nullptr;
        if (a.cout == 128) bits ? launch_first_fwd_mfma<4, true>(a, ntd, nth, ntw, ntiles, st) : launch_first_fwd_mfma<4, false>(a, ntd, nth, ntw, ntiles, st);
        else if (a.cout == 64) bits ? launch_first_fwd_mfma<2, true>(a, ntd, nth, ntw, ntiles, st) : launch_first_fwd_mfma<2, false>(a, ntd, nth, ntw, ntiles, st);
        else bits ? launch_first_fwd_mfma<1, true>(a, ntd, nth, ntw, ntiles, st) : launch_first_fwd_mfma<1, false>(a, ntd, nth, ntw, ntiles, st);
        K3_LAUNCH_CHECK();
        return K3_OK;
    }
    conv_first_fwd_kernel<<<dim3((unsigned)ntiles), 256, 0, st>>>((const bf16_t *)a.x, (const bf16_t *)a.w, a.bias, a.relu,
                                                                  (bf16_t *)a.y, (int)a.D, (int)a.H, (int)a.W, (int)a.cout,
                                                                  ntd, nth, ntw);
    K3_LAUNCH_CHECK();
    if (a.ybits) return launch_relu_bits(a.dtype, a.y, a.ybits, a.V() * a.cout / 16, st);
    return K3_OK;
}

static int64_t first_nsplit(int64_t ntiles) { return ntiles < 2048 ? ntiles : 2048; }
static int64_t first_nsplit_mfma(int64_t ntiles) { return ntiles < 256 ? ntiles : 256; }   // one workgroup per CU

template <int MB>
static int launch_first_wgrad_mfma(const ConvArgs &a, float *ws, int64_t per, int ntd, int nth, int ntw, int64_t ntiles,
                                   hipStream_t st, int coff = 0)
{
    constexpr int lds = 2 * MB * firstm::NVOX * 64 + 2 * FIRST_XS * 2 + 256 * 4;
    static_assert(lds <= 160 * 1024, "LDS budget");
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_first_wgrad_mfma_kernel<MB>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    conv_first_wgrad_mfma_kernel<MB><<<dim3((unsigned)first_nsplit_mfma(ntiles)), 256, lds, st>>>(
        (const bf16_t *)a.x, (const bf16_t *)a.dy, ws, per, (int)a.D, (int)a.H, (int)a.W, ntd, nth, ntw, ntiles, (int)a.cout, coff);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

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
    if (ntiles > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    int64_t nsplit = first_nsplit(ntiles);
    int64_t per = 28 * a.cout;   // 27 tap rows + the bias row: canonical [27][1][cout] followed by db
    if (first_mfma_ok(a) && !a.ymask) {
        // 128 channels: two passes of 64 (the double-buffered dy tile of 128 channels exceeds LDS);
        // they write disjoint columns of the same partial sums
        int rc = a.cout == 32 ? launch_first_wgrad_mfma<1>(a, ws, per, ntd, nth, ntw, ntiles, st)
                              : launch_first_wgrad_mfma<2>(a, ws, per, ntd, nth, ntw, ntiles, st);
        if (rc == K3_OK && a.cout == 128) rc = launch_first_wgrad_mfma<2>(a, ws, per, ntd, nth, ntw, ntiles, st, 64);
        if (rc != K3_OK) return rc;
        return launch_reduce_partials(ws, dW, db, 27 * a.cout, per, (int)first_nsplit_mfma(ntiles), st);
    }
    conv_first_wgrad_kernel<<<dim3((unsigned)nsplit), 256, 0, st>>>((const bf16_t *)a.x, (const bf16_t *)a.dy,
                                                                    (const bf16_t *)a.ymask, ws, per, (int)a.D, (int)a.H,
                                                                    (int)a.W, (int)a.cout, ntd, nth, ntw, ntiles);
    K3_LAUNCH_CHECK();
    return launch_reduce_partials(ws, dW, db, 27 * a.cout, per, (int)nsplit, st);
}

}  // namespace k3
