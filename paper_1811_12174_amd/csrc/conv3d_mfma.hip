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
#include <type_traits>

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
    const bf16_t *omask;               // optional: dst1 is zeroed where omask (same shape) is <= 0
    const unsigned short *omask_bits;  // the same mask as one bit per element (word j of a voxel: channels 16j..16j+15)
    unsigned short *bits_out;          // optional: receives that bit mask of dst1 (set where the stored value is > 0)
    bf16_t *pool_out;                  // optional (plane-streaming kernel, ReLU on): receives the 2x2x2 max-pool of dst1
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
            uint4 o0 = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
            uint4 o1 = make_uint4(pack2bf(v[8], v[9]), pack2bf(v[10], v[11]), pack2bf(v[12], v[13]), pack2bf(v[14], v[15]));
            const bool d1 = co0 < p.cd1;
            const int64_t eo = d1 ? vox * p.cd1 + co0 : vox * p.cd2 + (co0 - p.cd1);
            if (d1 && p.omask) {
                const uint4 *mp = reinterpret_cast<const uint4 *>(p.omask + eo);
                uint4 m0 = mp[0], m1 = mp[1];
                o0.x = mask_pair(o0.x, m0.x); o0.y = mask_pair(o0.y, m0.y); o0.z = mask_pair(o0.z, m0.z); o0.w = mask_pair(o0.w, m0.w);
                o1.x = mask_pair(o1.x, m1.x); o1.y = mask_pair(o1.y, m1.y); o1.z = mask_pair(o1.z, m1.z); o1.w = mask_pair(o1.w, m1.w);
            }
            uint4 *dst = reinterpret_cast<uint4 *>((d1 ? p.dst1 : p.dst2) + eo);
            dst[0] = o0;
            dst[1] = o1;
        }
    }
}

// ---------------------------------------------------------------------------- pipelined kernel
// Same GEMM mapping as conv_mfma_kernel, organised for one workgroup per CU: a larger tile, so
// each wave keeps NBW x MB accumulator blocks (fewer LDS bytes per MFMA), and asynchronous
// staging.  A stage is (16-channel chunk c, tap plane kd): 9 taps.  While the waves multiply
// stage s out of LDS, the data of stage s+1 -- the next tap plane of packed weights and one
// third of the next chunk's halo tile -- is in flight from global memory straight into the
// other LDS buffers (16-byte-per-lane copies to LDS through a buffer descriptor: lane l of a
// wave writes 16 bytes to LDS slot base + l, from descriptor base + its own offset; no registers
// are staged).  One vmcnt wait and one barrier per stage.  Voxels outside the volume and the
// row-padding slots carry an offset beyond the descriptor's range and arrive as zeros.  This
// kernel takes no input-side ReLU mask (the asynchronous copy cannot apply one); backward passes
// feed it gradients that were masked by their producer.
static __device__ uint4 g_zero_block[4];   // zero-initialised; source of the mask requests of out-of-volume lanes

template <int TD_, int TH_, int TW_, int MB_>
struct PipeCfg {
    static constexpr int TD = TD_, TH = TH_, TW = TW_, MB = MB_;
    static constexpr int HD = TD + 2, HH = TH + 2, HW = TW + 2;
    static constexpr int ROWSLOTS = HW * 2 + 1;               // 16-byte slots per halo row (32 B per voxel + 1 pad)
    static constexpr int XS_ROW = ROWSLOTS * 16;              // odd number of slots: see TileCfg
    static constexpr int XS_PLANE = HH * XS_ROW;
    static constexpr int NSLOT = HD * HH * ROWSLOTS;
    static constexpr int XGROUPS = (NSLOT + 63) / 64;         // 64-slot (1 KB) copy groups per chunk
    static constexpr int XS_BYTES = XGROUPS * 1024;
    static constexpr int XG_STAGE = (XGROUPS + 2) / 3;        // groups copied per stage
    static constexpr int XG_WAVE = (XG_STAGE + 3) / 4;        // per wave and stage
    static constexpr int WFRAGS = 9 * MB;                     // 1 KB weight fragments per stage
    static constexpr int WF_WAVE = (WFRAGS + 3) / 4;
    static constexpr int WS_BYTES = WFRAGS * 1024;
    static constexpr int BIAS_OFF = 2 * XS_BYTES + 2 * WS_BYTES;   // fp32 bias of every output channel
    static constexpr int BIAS_MAX = 1024;
    static constexpr int DUMP_OFF = BIAS_OFF + BIAS_MAX * 4;       // 1 KB target of the padding copies
    static constexpr int LDS_BYTES = DUMP_OFF + 1024;
    static constexpr int PW = TW / 8, PH = TH / 4;
    static constexpr int NBLK = TD * PH * PW;
    static constexpr int NBW = NBLK / 4;
    static_assert(TW % 8 == 0 && TH % 4 == 0 && NBLK % 4 == 0, "tile must split into 4x8 patches over 4 waves");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static_assert(3 * XG_WAVE <= 32, "validity bits are kept in one 32-bit mask");
};

// One tile of work: output block origin, output-channel group and the halo validity bits.
struct PipeTile {
    int n, d0, h0, w0, mb0;
    int64_t origin;     // linear voxel index of (n, d0, h0, w0)
    unsigned vmask;     // bit idx: the lane's halo slot idx lies inside the volume
    bool valid;
};

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// 16-byte global load whose completion the caller tracks itself (wait_vm below): the compiler
// inserts no wait for it, so a value may only be used after a wait that covers it.  Used where a
// compiler-generated wait would also wait for the asynchronous copies issued in between.
__device__ __forceinline__ u32x4 gload16_nowait(const void *ptr)
{
    u32x4 v;
    asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(v) : "v"(ptr) : "memory");
    return v;
}

__device__ __forceinline__ unsigned gload_u16_nowait(const void *ptr)
{
    unsigned v;
    asm volatile("global_load_ushort %0, %1, off" : "=v"(v) : "v"(ptr) : "memory");
    return v;
}

// s_waitcnt vmcnt(n) for a count that is a compile-time constant after unrolling (the instruction
// takes an immediate; every case folds away but one)
#define K3_WVM(n) case n: asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory"); break;
__device__ __forceinline__ void wait_vm(int n)
{
    switch (n) {
        K3_WVM(0) K3_WVM(1) K3_WVM(2) K3_WVM(3) K3_WVM(4) K3_WVM(5) K3_WVM(6) K3_WVM(7) K3_WVM(8) K3_WVM(9) K3_WVM(10)
        K3_WVM(11) K3_WVM(12) K3_WVM(13) K3_WVM(14) K3_WVM(15) K3_WVM(16) K3_WVM(17) K3_WVM(18) K3_WVM(19) K3_WVM(20)
        K3_WVM(21) K3_WVM(22) K3_WVM(23) K3_WVM(24) K3_WVM(25) K3_WVM(26) K3_WVM(27) K3_WVM(28) K3_WVM(29) K3_WVM(30)
        K3_WVM(31) K3_WVM(32) K3_WVM(33) K3_WVM(34) K3_WVM(35) K3_WVM(36) K3_WVM(37) K3_WVM(38) K3_WVM(39) K3_WVM(40)
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;   // never less safe: waits for everything
    }
}
#undef K3_WVM

// Masked output (the backward-data pass that applies the ReLU mask of its result): the 32 mask
// bytes of every accumulator block are requested into registers long before the block is
// finished.  The first R patches are requested one stage before the last stage of the tile; that
// stage ends with a wait that leaves fewer operations outstanding than it issued itself, so
// those requests have completed when the last stage starts.  With more than R patches per wave
// (R is what the register file allows) patch q >= R is requested into the slot of patch q - R
// right after that patch's last block was stored, and waited for by count:
// loads, asynchronous copies and stores of a wave complete in the order they were issued and
// share one counter, so "at most n operations outstanding" covers exactly the operations issued
// before the last n.  Inside item i of the last stage the order is: matrix instructions; the
// item's copy (items j * SP, j < NOPS); the two stores of a finished block (block (e, 0) in item
// (e + 1) * 9 + 2, block (e, MB - 1) in item (e + 1) * 9 + 5 when MB > 1; the last patch after
// the loop); mask requests (2 * MB per patch).  after(q) = operations issued behind the requests
// of patch q and before the stores of its first block.
template <int NBW, int MB, int NOPS, int SP>
struct MaskOrder {
    static constexpr int R = MB == 1 ? NBW : (NBW < 4 ? NBW : 4);
    static constexpr int NI = 9 * NBW;
    static constexpr int last_store_item(int e) { return (e + 1) * 9 + (MB > 1 ? 5 : 2); }
    static constexpr int issue_item(int q) { return last_store_item(q - R); }                // q >= R
    static constexpr int use_item(int q) { return q + 1 < NBW ? (q + 1) * 9 + 2 : NI; }      // NI: after the loop
    static constexpr int after(int q)
    {
        const int I = issue_item(q), U = use_item(q);
        int n = 0;
        for (int j = 0; j < NOPS; ++j)          // copies behind the requests (same item: before them), up to item U
            if (j * SP > I && j * SP <= U) ++n;
        for (int r = q + 1; r < NBW; ++r)       // mask requests of later patches
            if (issue_item(r) < U) n += 2 * MB;
        for (int e = 0; e + 1 < NBW; ++e) {     // stores of blocks finished in between
            const int i0 = (e + 1) * 9 + 2, i1 = (e + 1) * 9 + 5;
            if (i0 > I && i0 < U) n += 2;
            if (MB > 1 && i1 > I && i1 < U) n += 2;
        }
        return n;
    }
};

// OMASK 0: no output mask, 1: mask given as the bf16 tensor, 2: as one bit per element.  BITS: the
// bit mask of the first destination is written (a template parameter, not a test of p.bits_out:
// a wave-uniform branch per epilogue step costs more than the step)
template <class C, int OMASK, bool BITS>
__global__ __launch_bounds__(256, 1) void conv_mfma_pipe_kernel(MfmaParams p)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hb = lane >> 5, vl = lane & 31;
    const int nkc = (p.c1 + p.c2) / 16;
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    const unsigned char *zero = reinterpret_cast<const unsigned char *>(g_zero_block);

    // ---- tile-independent description of the halo slots this lane copies in each stage part
    int coords[3 * C::XG_WAVE];        // halo coordinates of the slot, packed ld | lh << 8 | lw << 16
    unsigned hvox[3 * C::XG_WAVE];     // voxel offset of the slot from the halo tile's first voxel
    unsigned smask = 0, hmask = 0;     // slot is a real (voxel, half) item / holds the upper 8 channels
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
        for (int k = 0; k < C::XG_WAVE; ++k) {
            const int idx = g * C::XG_WAVE + k;
            const int G = g * C::XG_STAGE + k * 4 + wv;
            const int slot = G * 64 + lane;
            const int r = slot / C::ROWSLOTS, pos = slot - r * C::ROWSLOTS;
            const int ld = r / C::HH, lh = r - ld * C::HH, lw = pos >> 1;
            const bool ok = G < C::XGROUPS && slot < C::NSLOT && pos < C::ROWSLOTS - 1;
            coords[idx] = ld | (lh << 8) | (lw << 16);
            hvox[idx] = (unsigned)((ld * p.H + lh) * p.W + lw);
            smask |= (ok ? 1u : 0u) << idx;
            hmask |= (unsigned)(pos & 1) << idx;
        }

    // Persistent workgroups: virtual block vb = blockIdx.x + j * gridDim.x (gridDim.x is a multiple
    // of 8, so a workgroup stays on its XCD).  The logical tile order is cut into 8 contiguous
    // runs, one per XCD, so halo-sharing neighbours and the channel groups of a tile share an L2.
    auto decode = [&](int64_t vb) {
        PipeTile t;
        const int64_t logical = (vb & 7) * p.per_xcd + (vb >> 3);
        t.valid = (vb >> 3) < p.per_xcd && logical < p.total;
        unsigned tile = t.valid ? (unsigned)logical : 0u;   // the tile count fits 31 bits (checked at launch)
        const int cg = (int)(tile % (unsigned)p.ncg);
        tile /= (unsigned)p.ncg;
        const int twi = (int)(tile % (unsigned)p.ntw);
        tile /= (unsigned)p.ntw;
        const int thi = (int)(tile % (unsigned)p.nth);
        tile /= (unsigned)p.nth;
        const int tdi = (int)(tile % (unsigned)p.ntd);
        t.n = (int)(tile / (unsigned)p.ntd);
        t.d0 = tdi * C::TD; t.h0 = thi * C::TH; t.w0 = twi * C::TW;
        t.mb0 = cg * C::MB;
        t.origin = (((int64_t)t.n * p.D + t.d0) * p.H + t.h0) * p.W + t.w0;
        // A halo coordinate l is inside the volume iff 0 <= t0 + l - 1 < size, i.e. lo <= l < hi.
        // Separable: one scalar word per axis with bit l set where l lies outside, then three
        // shifts per slot.
        auto axis_out = [](int t0, int n, int ext) __attribute__((always_inline)) {
            int lo = 1 - t0, hi = n + 1 - t0;
            if (lo < 0) lo = 0;
            if (hi > ext) hi = ext;
            return ~(((1u << hi) - 1u) & ~((1u << lo) - 1u));
        };
        const unsigned od = axis_out(t.d0, p.D, C::HD), oh = axis_out(t.h0, p.H, C::HH), ow = axis_out(t.w0, p.W, C::HW);
        unsigned nv = 0;
#pragma unroll
        for (int idx = 0; idx < 3 * C::XG_WAVE; ++idx) {
            const int cw = coords[idx];
            const unsigned ld = cw & 255, lh = (cw >> 8) & 255, lw = cw >> 16;
            nv |= (((od >> ld) | (oh >> lh) | (ow >> lw)) & 1u) << idx;
        }
        t.vmask = ~nv & smask;
        return t;
    };

    // Source of one stage's asynchronous copies (all wave-uniform): the weight fragments of the
    // next stage and one third of the next chunk's halo tile.  The copies go through buffer
    // descriptors: a lane with nothing to copy (halo item outside the volume, row padding, no next
    // stage) carries an offset beyond the descriptor's range and writes zeros.
    struct StageSrc {
        __amdgpu_buffer_rsrc_t wrs;   // packed weights of (first output block, first tap, chunk) of the stage
        __amdgpu_buffer_rsrc_t xrs;   // first channel of the chunk at the halo tile's first voxel
        unsigned strideB;             // bytes per voxel of the x source
        unsigned ninv;                // bit idx clear: the lane's halo slot idx lies inside the volume
        unsigned wvoff;               // lane offset inside a weight fragment, or "nothing"
        unsigned wlds, xlds;          // LDS byte addresses of the destination buffers
    };
    auto no_src = [&](StageSrc &s) {
        s.wrs = s.xrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(p.packed), 0, 0, 0x00020000);
        s.strideB = 0;
        s.ninv = 0xffffffffu;
        s.wvoff = 0xffffffffu;
        s.wlds = s.xlds = lds0 + C::DUMP_OFF;
    };
    auto w_src = [&](StageSrc &s, const PipeTile &t, int c, int g, int buf) {
        const unsigned char *wp = reinterpret_cast<const unsigned char *>(p.packed) + ((((int64_t)t.mb0 * 27 + g * 9) * nkc + c) * 1024);
        s.wrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(wp), 0, 0x7ffffff0, 0x00020000);
        s.wvoff = (unsigned)lane * 16u;
        s.wlds = lds0 + 2 * C::XS_BYTES + buf * C::WS_BYTES;
    };
    auto x_src = [&](StageSrc &s, const PipeTile &t, int c, int buf) {
        const int ch0 = c * 16;
        const bool first = ch0 < p.c1;
        const bf16_t *src = first ? p.src1 : p.src2;
        const int Csrc = first ? p.c1 : p.c2;
        const int chs = first ? ch0 : ch0 - p.c1;
        const int64_t halo0 = t.origin - ((int64_t)p.H * p.W + p.W + 1);
        const unsigned char *xp = reinterpret_cast<const unsigned char *>(src) + (halo0 * Csrc + chs) * 2;
        s.xrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(xp), 0, 0x7ffffff0, 0x00020000);
        s.strideB = Csrc * 2;
        s.ninv = ~t.vmask;
        s.xlds = lds0 + buf * C::XS_BYTES;
    };
    // copy operation j of a stage: first the weight fragments, then the halo groups of part g
    constexpr int NOPS = C::WF_WAVE + C::XG_WAVE;
    // Every wave issues exactly NOPS copies per stage, so that the number of copies still in
    // flight at a stage end is known at compile time (s_waitcnt takes an immediate): a slot that
    // has nothing to copy writes zeros into a dump area of LDS.
    // packed-weight offset of this wave's weight copy j: fragment f = 4 j + wv is (tap f / MB, block f % MB)
    unsigned wso[C::WF_WAVE];
#pragma unroll
    for (int j = 0; j < C::WF_WAVE; ++j) {
        const int f = j * 4 + wv, tl = f / C::MB, mb = f - tl * C::MB;
        wso[j] = (unsigned)((mb * 27 + tl) * nkc) * 1024u;
    }
    auto issue_op = [&](const StageSrc &s, int j, auto gtag) __attribute__((always_inline)) {
        constexpr int g = decltype(gtag)::value;
        const unsigned dump = lds0 + C::DUMP_OFF;
        if (j < C::WF_WAVE) {
            const int f = j * 4 + wv;   // fragment (tap tl, block mb) of the stage
            const bool ok = f < C::WFRAGS;
            dma16_buf(ok ? s.wlds + f * 1024 : dump, s.wrs, ok ? s.wvoff : 0xffffffffu, ok ? wso[j] : 0u);
        } else {
            const int k = j - C::WF_WAVE;
            const int idx = g * C::XG_WAVE + k;
            const int G = g * C::XG_STAGE + k * 4 + wv;
            const bool ok = k * 4 + wv < C::XG_STAGE && G < C::XGROUPS;
            // every factor is below 2^24 and the byte offset below 2^31 (checked at launch); all
            // ones where the slot is outside the volume (sign-extended bit idx)
            const unsigned off = __umul24(hvox[idx], s.strideB) + ((hmask >> idx) & 1) * 16;
            const unsigned inv = (unsigned)__builtin_amdgcn_sbfe(s.ninv, idx, 1);
            dma16_buf(ok ? s.xlds + G * 1024 : dump, s.xrs, ok ? (off | inv) : 0xffffffffu, 0u);
        }
    };

    // LDS byte offset of the lane's voxel (tap 0,0,0 corner, the lane's channel half) in patch 0 of
    // the wave; patch a of the wave lies PatchOff::lds(a) bytes further (a compile-time constant,
    // because the wave's NBW patches are whole depth planes of PW * PH patches)
    static_assert(C::NBW % (C::PW * C::PH) == 0, "a wave owns whole planes of patches");
    constexpr int PPL = C::PW * C::PH, WPL = C::NBW / PPL;   // patches per plane, planes per wave
    const int lrow = vl >> 3, lcol = vl & 7;
    const int vb0 = wv * WPL * C::XS_PLANE + lrow * C::XS_ROW + lcol * 32 + hb * 16;
    auto patch_lds = [](int a) __attribute__((always_inline)) {
        return (a / PPL) * C::XS_PLANE + (((a % PPL) / C::PW) * 4) * C::XS_ROW + ((a % PPL) % C::PW) * 8 * 32;
    };
    // voxel offset of the lane's voxel inside a patch from the patch's first voxel
    const int lvox = lrow * p.W + lcol;
    PipeTile cur = decode(blockIdx.x);
    if (!cur.valid) return;
    int64_t vb_next = (int64_t)blockIdx.x + gridDim.x;

    // ---- prologue: chunk 0 of the first tile and the weights of its stage (0, 0)
    {
        StageSrc s0;
        no_src(s0);
        w_src(s0, cur, 0, 0, 0);
        x_src(s0, cur, 0, 0);
#pragma unroll
        for (int j = 0; j < NOPS; ++j) {
            issue_op(s0, j, std::integral_constant<int, 0>());
            if (j >= C::WF_WAVE) {
                issue_op(s0, j, std::integral_constant<int, 1>());
                issue_op(s0, j, std::integral_constant<int, 2>());
            }
        }
    }
    // Requests the 32 mask bytes of every block of patch nb of tile t (the stored ReLU output at
    // the block's own output position); lanes outside the volume and blocks of the unmasked second
    // destination read the zero block, so that every wave issues the same number of requests.
    typedef MaskOrder<C::NBW, C::MB, NOPS, (C::MB == 1 ? 3 : 2)> MO;
    u32x4 mk[MO::R][C::MB][2];
    auto mask_request = [&](const PipeTile &t, int nb, u32x4 (&dst)[C::MB][2]) __attribute__((always_inline)) {
        const int bw = (nb % PPL) % C::PW, bh = (nb % PPL) / C::PW, bd = wv * WPL + nb / PPL;
        const bool inb = bd < p.D - t.d0 && bh * 4 + lrow < p.H - t.h0 && bw * 8 + lcol < p.W - t.w0;
        const int pvox = (bd * p.H + bh * 4) * p.W + bw * 8 + lvox;
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) {
            const int co0 = (t.mb0 + mb) * 32;
            const bool d1 = co0 < p.cd1;
            const bf16_t *mp = p.omask + t.origin * p.cd1 + co0 + (pvox * p.cd1 + hb * 16);
            const unsigned char *ptr = (d1 && inb) ? reinterpret_cast<const unsigned char *>(mp) : zero;
            dst[mb][0] = gload16_nowait(ptr);
            dst[mb][1] = gload16_nowait(ptr + 16);
        }
    };
    auto mask_pin = [&](u32x4 (&dst)[C::MB][2]) __attribute__((always_inline)) {
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) asm volatile("" : "+v"(dst[mb][0]), "+v"(dst[mb][1]));
    };
    // one-bit-per-element form: 2 bytes per block and lane, so all blocks of the wave are
    // requested at once (one register each)
    unsigned mkb[C::NBW][C::MB];
    auto maskbits_request = [&](const PipeTile &t) __attribute__((always_inline)) {
#pragma unroll
        for (int nb = 0; nb < C::NBW; ++nb) {
            const int bw = (nb % PPL) % C::PW, bh = (nb % PPL) / C::PW, bd = wv * WPL + nb / PPL;
            const bool inb = bd < p.D - t.d0 && bh * 4 + lrow < p.H - t.h0 && bw * 8 + lcol < p.W - t.w0;
            const int pvox = (bd * p.H + bh * 4) * p.W + bw * 8 + lvox;
#pragma unroll
            for (int mb = 0; mb < C::MB; ++mb) {
                const int co0 = (t.mb0 + mb) * 32;
                const bool d1 = co0 < p.cd1;
                const unsigned short *mp = p.omask_bits + (t.origin * p.cd1 + co0) / 16 + (pvox * (p.cd1 / 16) + hb);
                mkb[nb][mb] = gload_u16_nowait((d1 && inb) ? reinterpret_cast<const unsigned char *>(mp) : zero);
            }
        }
    };
    if constexpr (OMASK != 2) {
#pragma unroll
        for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
            for (int mb = 0; mb < C::MB; ++mb) mkb[nb][mb] = 0u;
    }
    if constexpr (OMASK != 1) {
#pragma unroll
        for (int r = 0; r < MO::R; ++r)
#pragma unroll
            for (int mb = 0; mb < C::MB; ++mb) mk[r][mb][0] = mk[r][mb][1] = u32x4{0u, 0u, 0u, 0u};
    }
    // while the first copies are in flight: the bias vector goes to LDS for the whole kernel
    // (zeros when there is none), and the next tile is decoded
    {
        float *bl = reinterpret_cast<float *>(smem + C::BIAS_OFF);
        const int nco = p.cd1 + p.cd2;
        for (int i = tid; i < nco; i += 256) bl[i] = p.bias ? p.bias[i] : 0.f;
    }
    PipeTile nxt = decode(vb_next);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    int xpar = 0, wpar = 0;   // LDS buffers holding the current chunk / the current stage's weights
    const float relu_floor = p.relu ? 0.f : -__builtin_inff();
    while (true) {
        // per-tile accumulators (not carried from tile to tile), started at the bias
        f32x16 acc[C::NBW][C::MB];
        {
            const f32x4 *bl = reinterpret_cast<const f32x4 *>(smem + C::BIAS_OFF) + (cur.mb0 * 32 + hb * 16) / 4;
#pragma unroll
            for (int b = 0; b < C::MB; ++b) {
                f32x4 q[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) q[i] = bl[b * 8 + i];
#pragma unroll
                for (int a = 0; a < C::NBW; ++a) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[a][b][i] = q[i >> 2][i & 3];
                    asm volatile("" : "+a"(acc[a][b]));   // straight into accumulator registers
                }
            }
        }
        const int dlim = p.D - cur.d0, hlim = p.H - cur.h0, wlim = p.W - cur.w0;

        // Finishes one accumulator block: bias, ReLU, optional output mask, round to bf16, store
        // 32 contiguous bytes per lane.
        auto emit = [&](int nb, int mb, u32x4 m0, u32x4 m1) __attribute__((always_inline)) {
            const unsigned mbits = mkb[nb][mb];
            const int bw = (nb % PPL) % C::PW, bh = (nb % PPL) / C::PW, bd = wv * WPL + nb / PPL;
            const bool inb = bd < dlim && bh * 4 + lrow < hlim && bw * 8 + lcol < wlim;
            const int pvox = (bd * p.H + bh * 4) * p.W + bw * 8 + lvox;
            const int co0 = (cur.mb0 + mb) * 32;   // wave-uniform; the lane's 16 channels start at co0 + hb * 16
            // keep the block in accumulator registers until here: without the pin the compiler
            // copies blocks to VGPRs right after their last MFMA and spills
            asm volatile("" : "+a"(acc[nb][mb]));
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) v[i] = fmaxf(acc[nb][mb][i], relu_floor);
            uint4 o0 = make_uint4(pack2bf(v[0], v[1]), pack2bf(v[2], v[3]), pack2bf(v[4], v[5]), pack2bf(v[6], v[7]));
            uint4 o1 = make_uint4(pack2bf(v[8], v[9]), pack2bf(v[10], v[11]), pack2bf(v[12], v[13]), pack2bf(v[14], v[15]));
            const bool d1 = co0 < p.cd1;
            const int cd = d1 ? p.cd1 : p.cd2;
            // wave-uniform 64-bit part + per-lane 32-bit element offset (fits: checked at launch)
            const int64_t ubase = cur.origin * cd + (d1 ? co0 : co0 - p.cd1);
            const int loff = pvox * cd + hb * 16;
            if constexpr (OMASK == 1) {
                if (d1) {
                    o0.x = mask_pair(o0.x, m0[0]); o0.y = mask_pair(o0.y, m0[1]); o0.z = mask_pair(o0.z, m0[2]); o0.w = mask_pair(o0.w, m0[3]);
                    o1.x = mask_pair(o1.x, m1[0]); o1.y = mask_pair(o1.y, m1[1]); o1.z = mask_pair(o1.z, m1[2]); o1.w = mask_pair(o1.w, m1[3]);
                }
            }
            if constexpr (OMASK == 2) {
                if (d1) {
                    uint32_t dd[8] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y, o1.z, o1.w};
                    apply_bits16(dd, mbits);
                    o0 = make_uint4(dd[0], dd[1], dd[2], dd[3]);
                    o1 = make_uint4(dd[4], dd[5], dd[6], dd[7]);
                }
            }
            if constexpr (BITS) {
                if (d1) {   // wave-uniform: the bit mask of what is stored below
                    const uint32_t dd[8] = {o0.x, o0.y, o0.z, o0.w, o1.x, o1.y, o1.z, o1.w};
                    const unsigned m = relu_bits16(dd);
                    unsigned short *bbase = p.bits_out + ubase / 16;
                    __amdgpu_buffer_rsrc_t brsrc = __builtin_amdgcn_make_buffer_rsrc(bbase, 0, 0x7ffffff0, 0x00020000);
                    __builtin_amdgcn_raw_buffer_store_b16((short)m, brsrc, inb ? (loff / 16) * 2 : -1, 0, 0);
                }
            }
            // buffer stores relative to the tile's first voxel: lanes outside the volume get an
            // offset beyond the range of the descriptor, which the hardware drops (no branch)
            bf16_t *dbase = (d1 ? p.dst1 : p.dst2) + ubase;
            __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(dbase, 0, 0x7ffffff0, 0x00020000);
            const int boff = inb ? loff * 2 : -1;
            __builtin_amdgcn_raw_buffer_store_b128(u32x4{o0.x, o0.y, o0.z, o0.w}, rsrc, boff, 0, 0);
            __builtin_amdgcn_raw_buffer_store_b128(u32x4{o1.x, o1.y, o1.z, o1.w}, rsrc, boff, 16, 0);
        };

        // The same in 8 steps per block (the variants without counted waits inside the last stage):
        // step i rounds values 2i, 2i+1 to bf16 and applies ReLU on the packed pair (as 16-bit
        // integers the negative bf16 values are the negative numbers), step 3 stores the lower 16
        // bytes of the lane's 32, step 7 the upper 16 and the mask word.  What does not depend on
        // the patch is prepared once per tile: descriptors, the lane's byte offset inside a patch.
        __amdgpu_buffer_rsrc_t ersrc[C::MB], ebrsrc[C::MB];
        int elane[C::MB], ecd2[C::MB];
        unsigned eforce[C::MB];   // OMASK == 2: 3 for a block of the unmasked second destination (keeps both halves)
#pragma unroll
        for (int mb = 0; mb < C::MB; ++mb) {
            const int co0 = (cur.mb0 + mb) * 32;
            const bool d1 = co0 < p.cd1;
            const int cd = d1 ? p.cd1 : p.cd2;
            const int64_t ubase = cur.origin * cd + (d1 ? co0 : co0 - p.cd1);
            ersrc[mb] = __builtin_amdgcn_make_buffer_rsrc((d1 ? p.dst1 : p.dst2) + ubase, 0, 0x7ffffff0, 0x00020000);
            // (bit masks are written by forward passes, which have one destination)
            ebrsrc[mb] = __builtin_amdgcn_make_buffer_rsrc((BITS ? p.bits_out : (unsigned short *)p.dst1) + (BITS ? ubase / 16 : 0),
                                                           0, 0x7ffffff0, 0x00020000);
            eforce[mb] = d1 ? 0u : 3u;
            elane[mb] = (lvox * cd + hb * 16) * 2;
            ecd2[mb] = cd * 2;
        }
        const unsigned relu_min = p.relu ? 0u : 0x80008000u;   // per 16-bit half: 0, or the most negative integer (no clamp)
        uint32_t eob[C::MB][8];
        unsigned ezb[C::MB];
        int evoff[C::MB];
        auto emit_step = [&](int nb, int mb, int i) __attribute__((always_inline)) {
            if (i == 0) asm volatile("" : "+a"(acc[nb][mb]));
            uint32_t o = pack2bf(acc[nb][mb][2 * i], acc[nb][mb][2 * i + 1]);
            o = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2_t, o), __builtin_bit_cast(s16x2_t, relu_min)));
            if constexpr (OMASK == 2) {
                const unsigned kk = ((mkb[nb][mb] >> (2 * i)) & 3u) | eforce[mb];
                const u16x2_t keep = __builtin_bit_cast(u16x2_t, (kk | (kk << 15)) & 0x00010001u);
                o = __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2_t, o) * keep);
            }
            if constexpr (BITS) ezb[mb] = i == 0 ? pair_positive_pk(o) : (ezb[mb] | (pair_positive_pk(o) << i));
            eob[mb][i] = o;
            if (i == 3) {
                const int bw = (nb % PPL) % C::PW, bh = (nb % PPL) / C::PW, bd = wv * WPL + nb / PPL;
                const bool inb = bd < dlim && bh * 4 + lrow < hlim && bw * 8 + lcol < wlim;
                evoff[mb] = inb ? elane[mb] : -1;
                const int soff = ((bd * p.H + bh * 4) * p.W + bw * 8) * ecd2[mb];   // wave-uniform: the patch's first voxel
                __builtin_amdgcn_raw_buffer_store_b128(u32x4{eob[mb][0], eob[mb][1], eob[mb][2], eob[mb][3]}, ersrc[mb], evoff[mb], soff, 0);
            }
            if (i == 7) {
                const int bw = (nb % PPL) % C::PW, bh = (nb % PPL) / C::PW, bd = wv * WPL + nb / PPL;
                const int soff = ((bd * p.H + bh * 4) * p.W + bw * 8) * ecd2[mb];
                __builtin_amdgcn_raw_buffer_store_b128(u32x4{eob[mb][4], eob[mb][5], eob[mb][6], eob[mb][7]}, ersrc[mb], evoff[mb], soff + 16, 0);
                if constexpr (BITS) {
                    unsigned z = ezb[mb];   // even elements in bits 0..7, odd ones in bits 16..23 (see relu_bits16)
                    z = (z | (z << 4)) & 0x0F0F0F0Fu;
                    z = (z | (z << 2)) & 0x33333333u;
                    z = (z | (z << 1)) & 0x55555555u;
                    z = (z | (z >> 15)) & 0xffffu;
                    // word of the lane's 16 channels: element offset / 16 words of 2 bytes = byte offset / 16
                    __builtin_amdgcn_raw_buffer_store_b16((short)z, ebrsrc[mb], evoff[mb] < 0 ? -1 : evoff[mb] / 16, soff / 16, 0);
                }
            }
        };

        // One stage = 9 taps of one depth plane of one 16-channel chunk.  FINAL marks the last
        // stage of the tile.
        auto stage = [&](int c, auto gtag, auto finaltag) __attribute__((always_inline)) {
            constexpr int g = decltype(gtag)::value;
            constexpr bool FINAL = decltype(finaltag)::value;
            // the data of the next stage (possibly the first stage of the next tile) starts moving
            // now; its copies are issued one at a time between the matrix instructions below
            const bool more = c + 1 < nkc;
            StageSrc ss;
            no_src(ss);
            if (g < 2) w_src(ss, cur, c, g + 1, wpar ^ 1);
            else if (more) w_src(ss, cur, c + 1, 0, wpar ^ 1);
            else if (nxt.valid) w_src(ss, nxt, 0, 0, wpar ^ 1);
            if (more) x_src(ss, cur, c + 1, xpar ^ 1);
            else if (nxt.valid) x_src(ss, nxt, 0, xpar ^ 1);
            const unsigned char *xs = smem + xpar * C::XS_BYTES + g * C::XS_PLANE;
            const unsigned char *wsm = smem + 2 * C::XS_BYTES + wpar * C::WS_BYTES + lane * 16;
            // Software pipeline over the 9 x NBW (tap, patch) items of the stage: the fragments of
            // item i+PD are requested from LDS before the MFMAs of item i issue, so LDS latency hides
            // behind matrix work even with a single wave per SIMD.  sched_barrier keeps the compiler
            // from undoing the order.
            constexpr int NI = 9 * C::NBW, PD = 3;
            constexpr int SP = C::MB == 1 ? 3 : 2;   // items between two copy operations
            static_assert(NOPS * SP <= NI, "copy operations must fit into the stage");
            auto ldb = [&](int tl, int nb) __attribute__((always_inline)) {
                return *reinterpret_cast<const bf16x8 *>(xs + vb0 + patch_lds(nb) + (tl / 3) * C::XS_ROW + (tl % 3) * 32);
            };
            auto lda = [&](int tl, int mb) __attribute__((always_inline)) { return *reinterpret_cast<const bf16x8 *>(wsm + (tl * C::MB + mb) * 1024); };
            if constexpr (!FINAL) {
                // tap-major order: the weight fragments of a tap serve all NBW patches
                bf16x8 bq[4], aq[2][C::MB];
#pragma unroll
                for (int mb = 0; mb < C::MB; ++mb) aq[0][mb] = lda(0, mb);
#pragma unroll
                for (int i = 0; i < PD; ++i) bq[i] = ldb(i / C::NBW, i % C::NBW);
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const int tl = i / C::NBW, nb = i % C::NBW;
                    if (i + PD < NI) bq[(i + PD) & 3] = ldb((i + PD) / C::NBW, (i + PD) % C::NBW);
                    if (nb == 0 && tl + 1 < 9) {
#pragma unroll
                        for (int mb = 0; mb < C::MB; ++mb) aq[(tl + 1) & 1][mb] = lda(tl + 1, mb);
                    }
#pragma unroll
                    for (int mb = 0; mb < C::MB; ++mb)
                        acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[tl & 1][mb], bq[i & 3], acc[nb][mb], 0, 0, 0);
                    if (i % SP == 0 && i / SP < NOPS) issue_op(ss, i / SP, gtag);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else if constexpr (OMASK != 1) {
                // The first T0 taps run tap-major like every other stage.  The remaining taps run
                // patch-major with their weight fragments held in registers: a patch is complete
                // after them, and the blocks of the previous patch are converted and stored, one
                // step behind each matrix instruction, while the next patch is multiplied.  (A
                // wave issues in order: with all nine taps patch-major the weight fragments were
                // re-read for every patch and the stage took 2.4 times as long as the others.)
                constexpr int T0 = 4, T1 = 9 - T0;
                static_assert(T1 <= T0 * C::NBW, "the register-resident fragments are read during the tap-major part");
                bf16x8 bq[4], aq[2][C::MB], af[T1][C::MB];
                auto ldb2 = [&](int j) __attribute__((always_inline)) {   // j: item of the combined order
                    if (j < T0 * C::NBW) return ldb(j / C::NBW, j % C::NBW);
                    const int r = j - T0 * C::NBW;
                    return ldb(T0 + r % T1, r / T1);
                };
                constexpr int NJ = 9 * C::NBW;
#pragma unroll
                for (int mb = 0; mb < C::MB; ++mb) aq[0][mb] = lda(0, mb);
#pragma unroll
                for (int j = 0; j < PD; ++j) bq[j] = ldb2(j);
#pragma unroll
                for (int j = 0; j < NJ; ++j) {
                    if (j + PD < NJ) bq[(j + PD) & 3] = ldb2(j + PD);
                    if (j < T0 * C::NBW) {
                        const int tl = j / C::NBW, nb = j % C::NBW;
                        if (nb == 0 && tl + 1 < T0) {
#pragma unroll
                            for (int mb = 0; mb < C::MB; ++mb) aq[(tl + 1) & 1][mb] = lda(tl + 1, mb);
                        }
                        // the fragments of the patch-major taps, one tap per item at the end of this part
                        if (j >= T0 * C::NBW - T1) {
#pragma unroll
                            for (int mb = 0; mb < C::MB; ++mb) af[j - (T0 * C::NBW - T1)][mb] = lda(T0 + j - (T0 * C::NBW - T1), mb);
                        }
#pragma unroll
                        for (int mb = 0; mb < C::MB; ++mb)
                            acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[tl & 1][mb], bq[j & 3], acc[nb][mb], 0, 0, 0);
                        if (j % SP == 0 && j / SP < NOPS) issue_op(ss, j / SP, gtag);
                        __builtin_amdgcn_sched_barrier(0);
                    } else {
                        const int r = j - T0 * C::NBW, nb = r / T1, t = r % T1;
#pragma unroll
                        for (int mb = 0; mb < C::MB; ++mb) {
                            acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[t][mb], bq[j & 3], acc[nb][mb], 0, 0, 0);
                            // steps of the previous patch's blocks: block mb2 takes steps behind the
                            // matrix instructions e = t * MB + mb with e / 8 == mb2 (MB = 2: e = 0..9,
                            // block 0 behind 0..7; block 1 behind 8, 9 and the rest doubled up)
                            if (nb > 0) {
                                constexpr int NE = T1 * C::MB;           // matrix instructions per patch
                                constexpr int NS = 8 * C::MB;            // emit steps per patch
                                const int e = t * C::MB + mb;
#pragma unroll
                                for (int q = e * NS / NE; q < (e + 1) * NS / NE; ++q) emit_step(nb - 1, q / 8, q % 8);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        if (j % SP == 0 && j / SP < NOPS) issue_op(ss, j / SP, gtag);
                    }
                }
#pragma unroll
                for (int mb = 0; mb < C::MB; ++mb) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) emit_step(C::NBW - 1, mb, e);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // (mask given as the bf16 tensor, waited for by count) patch-major order: a patch is
                // complete after its 9 taps, and its blocks are converted and stored between the
                // matrix instructions of the next patch (the weight fragments are re-read per patch)
                constexpr int PF = 2, RF = PF + 1;   // read-ahead and ring size of this stage
                bf16x8 bq[RF], aq[RF][C::MB];
#pragma unroll
                for (int i = 0; i < PF; ++i) {
                    bq[i] = ldb(i % 9, i / 9);
#pragma unroll
                    for (int mb = 0; mb < C::MB; ++mb) aq[i][mb] = lda(i % 9, mb);
                }
#pragma unroll
                for (int i = 0; i < NI; ++i) {
                    const int nb = i / 9, tl = i % 9;
                    if (i + PF < NI) {
                        bq[(i + PF) % RF] = ldb((i + PF) % 9, (i + PF) / 9);
#pragma unroll
                        for (int mb = 0; mb < C::MB; ++mb) aq[(i + PF) % RF][mb] = lda((i + PF) % 9, mb);
                    }
#pragma unroll
                    for (int mb = 0; mb < C::MB; ++mb)
                        acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[i % RF][mb], bq[i % RF], acc[nb][mb], 0, 0, 0);
                    if (i % SP == 0 && i / SP < NOPS) issue_op(ss, i / SP, gtag);
                    // blocks of the previous patch: one after taps 2 and 5 of this patch
                    if (nb > 0 && tl == 2) {
                        if constexpr (OMASK == 1) {
                            if (nb - 1 >= MO::R) {
                                wait_vm(MO::after(nb - 1));
                                mask_pin(mk[(nb - 1) % MO::R]);   // the values are defined from here on
                            }
                        }
                        emit(nb - 1, 0, mk[(nb - 1) % MO::R][0][0], mk[(nb - 1) % MO::R][0][1]);
                    }
                    if (nb > 0 && tl == 5 && C::MB > 1)
                        emit(nb - 1, C::MB - 1, mk[(nb - 1) % MO::R][C::MB - 1][0], mk[(nb - 1) % MO::R][C::MB - 1][1]);
                    if constexpr (OMASK == 1) {
                        // the slot of patch nb - 1 is free once its last block is stored
                        if (nb > 0 && tl == (C::MB > 1 ? 5 : 2) && nb - 1 + MO::R < C::NBW)
                            mask_request(cur, nb - 1 + MO::R, mk[(nb - 1) % MO::R]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (OMASK == 1) {
                    if (C::NBW - 1 >= MO::R) {
                        wait_vm(MO::after(C::NBW - 1));
                        mask_pin(mk[(C::NBW - 1) % MO::R]);
                    }
                }
#pragma unroll
                for (int mb = 0; mb < C::MB; ++mb) {
                    emit(C::NBW - 1, mb, mk[(C::NBW - 1) % MO::R][mb][0], mk[(C::NBW - 1) % MO::R][mb][1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // The next stage needs its weights, issued first in this stage; the halo thirds issued
            // after them are not read before the next chunk starts, so after the first two stages
            // of a chunk they may stay in flight (copies complete in issue order).
            // The last stage of a tile need not wait for its own stores: behind its last copy the
            // wave issued at least two stores per block of the patches stored after that copy (all
            // patches when the copies end inside the tap-major part, else the last patch).
            if constexpr (g < 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::XG_WAVE) : "memory");
            else if constexpr (FINAL && OMASK != 1) wait_vm((NOPS - 1) * SP < 4 * C::NBW ? 2 * C::MB * C::NBW : 2 * C::MB);
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
            wpar ^= 1;
        };

        for (int c = 0; c + 1 < nkc; ++c) {
            stage(c, std::integral_constant<int, 0>(), std::false_type());
            stage(c, std::integral_constant<int, 1>(), std::false_type());
            stage(c, std::integral_constant<int, 2>(), std::false_type());
            xpar ^= 1;
        }
        stage(nkc - 1, std::integral_constant<int, 0>(), std::false_type());
        if constexpr (OMASK == 2) {
            static_assert(C::XG_WAVE < NOPS, "a stage-end wait must cover operations issued before the stage");
            maskbits_request(cur);   // one stage ahead, complete after the next stage's closing wait
        }
        if constexpr (OMASK == 1) {
            // One stage ahead of their use: the wait that ends the next stage leaves fewer
            // operations outstanding than that stage issues, so these requests are complete after
            // it.  (Requested at the start of the tile, or with the prologue's copies, they compete
            // with those copies for the L2: measured no faster and 23 % more HBM traffic.)
            static_assert(C::XG_WAVE < NOPS, "a stage-end wait must cover operations issued before the stage");
#pragma unroll
            for (int nb = 0; nb < MO::R; ++nb) mask_request(cur, nb, mk[nb]);
        }
        stage(nkc - 1, std::integral_constant<int, 1>(), std::false_type());
        if constexpr (OMASK == 1) {
#pragma unroll
            for (int nb = 0; nb < MO::R; ++nb) mask_pin(mk[nb]);
        }
        if constexpr (OMASK == 2) {
#pragma unroll
            for (int nb = 0; nb < C::NBW; ++nb)
#pragma unroll
                for (int mb = 0; mb < C::MB; ++mb) asm volatile("" : "+v"(mkb[nb][mb]));
        }
        stage(nkc - 1, std::integral_constant<int, 2>(), std::true_type());
        xpar ^= 1;
        if (!nxt.valid) break;
        cur = nxt;
        vb_next += gridDim.x;
        nxt = decode(vb_next);
    }
}

// ---------------------------------------------------------------------------- plane-streaming kernel
// The 32-output-channel case (one MFMA row block per workgroup).  In the pipelined kernel above
// every activation fragment read from LDS feeds a single matrix instruction there, and the LDS
// read rate, not the matrix cores, sets the pace.  Here a wave owns one 4x8 patch position in all
// 8 depth planes of an 8x8x16 tile and walks the 10 halo planes of a 16-channel chunk in depth
// order: the fragment of halo plane z, tap (kh, kw) is read once and multiplied into the
// accumulators of output planes z, z-1, z-2 with the weights of taps kd = 0, 1, 2, which stay in
// registers for the whole chunk (27 fragments = 108 registers).  LDS traffic per matrix
// instruction drops 2.7x.  Walking the planes in order has two more effects:
//   * the first chunk of a workgroup is consumed while it arrives: plane z is waited for by
//     count (copies complete in issue order), so the matrix cores start after two copy
//     operations per wave instead of after the whole halo tile;
//   * an output plane is complete after halo plane d + 2 of the last chunk, and is converted and
//     stored, one register pair per step, between the matrix instructions of the next plane.
// Weight registers are recycled plane by plane: taps kd = 0 are last used in plane 7, so the next
// chunk's kd = 0 fragments are read from LDS during plane 8, kd = 1 during plane 9 and kd = 2
// during the next chunk's plane 0.  Two barriers per chunk: after plane 0 (every wave has taken
// its weights: the next chunk's weights may be copied into the one weight buffer, and the halo
// buffer of the chunk before is free) and before plane 8 (the next chunk's weights and halo tile
// have landed).
struct ZsCfg {
    static constexpr int TD = 8, TH = 8, TW = 16;
    static constexpr int HD = 10, HH = 10, HW = 18;
    static constexpr int ROWSLOTS = HW * 2 + 1;               // 16-byte slots per halo row (as PipeCfg)
    static constexpr int XS_ROW = ROWSLOTS * 16;
    static constexpr int XS_PLANE = HH * XS_ROW;
    static constexpr int PLANE_SLOTS = HH * ROWSLOTS;
    static constexpr int NSLOT = HD * PLANE_SLOTS;
    static constexpr int XGROUPS = (NSLOT + 63) / 64;         // 1 KB copy groups per chunk, in plane order
    static constexpr int XS_BYTES = XGROUPS * 1024;
    static constexpr int XOPS = (XGROUPS + 3) / 4;            // halo copies per wave and chunk
    static constexpr int WOPS = 7;                            // weight copies per wave and chunk (27 fragments)
    static constexpr int W_OFF = 2 * XS_BYTES;
    static constexpr int BIAS_OFF = W_OFF + 27 * 1024;
    static constexpr int BIAS_MAX = 1024;
    static constexpr int DUMP_OFF = BIAS_OFF + BIAS_MAX * 4;
    static constexpr int LDS_BYTES = DUMP_OFF + 1024;
    // halo copies of a wave (in issue order) that must be complete before plane z is read
    static constexpr int need(int z) { return (((z + 1) * PLANE_SLOTS - 1) / 64) / 4 + 1; }
    // copies a wave issues inside a chunk before plane z: the 7 weight copies in plane 1, three
    // halo copies in each of planes 2..6
    static constexpr int issued_before(int z) { return (z >= 2 ? WOPS : 0) + 3 * (z < 2 ? 0 : (z > 7 ? 5 : z - 2)); }
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};
static_assert(ZsCfg::XOPS == 15 && ZsCfg::need(9) == ZsCfg::XOPS, "the copy schedule assumes 15 halo copies per wave");

// Halo slot of (copy k, thread): halo coordinates ld | lh << 8 | lw << 16, bit 24 = the slot
// holds the upper 8 channels of its voxel, bit 25 = the slot is a real (voxel, half) item (not
// row padding, not beyond the tile).  Shape-independent, so it is a table and not arithmetic.
struct ZsSlotTable {
    int v[ZsCfg::XOPS * 256];
    constexpr ZsSlotTable() : v()
    {
        for (int k = 0; k < ZsCfg::XOPS; ++k)
            for (int t = 0; t < 256; ++t) {
                const int G = k * 4 + t / 64, slot = G * 64 + t % 64;
                const int r = slot / ZsCfg::ROWSLOTS, pos = slot - r * ZsCfg::ROWSLOTS;
                const int ld = r / ZsCfg::HH, lh = r - ld * ZsCfg::HH, lw = pos >> 1;
                const bool ok = G < ZsCfg::XGROUPS && slot < ZsCfg::NSLOT && pos < ZsCfg::ROWSLOTS - 1;
                v[k * 256 + t] = ok ? (ld | (lh << 8) | (lw << 16) | ((pos & 1) << 24) | (1 << 25)) : 0;
            }
    }
};
static __device__ const ZsSlotTable g_zs_slots = ZsSlotTable();

// OMASK 0: no output mask, 2: one bit per element; BITS: the output's bit mask is written; POOL: the
// 2x2x2 max-pool of the output is written as well (ReLU on: the maxima are taken on the packed bf16
// pairs as 16-bit integers, which order like the values only where these are not negative)
template <int OMASK, bool BITS, bool POOL>
__global__ __launch_bounds__(256, 1) void conv_mfma_zs_kernel(MfmaParams p)
{
    typedef ZsCfg C;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hb = lane >> 5, vl = lane & 31;
    const int nkc = (p.c1 + p.c2) / 16;
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;

    int coords[C::XOPS];
    // byte offset of each slot from the halo tile's first voxel (the sources have equal strides;
    // every factor is below 2^24 and the product below 2^31: checked at launch)
    const unsigned strideB = p.c1 * 2;
    unsigned xb[C::XOPS];
    auto slot_offset = [&](int cw) __attribute__((always_inline)) {
        const unsigned ld = cw & 255, lh = (cw >> 8) & 255, lw = (cw >> 16) & 255;
        const unsigned vox = __umul24(__umul24(ld, p.H) + lh, p.W) + lw;
        return __umul24(vox, strideB) + ((cw >> 24) & 1) * 16;
    };
    // Validity is separable: bit l of axis_out(t0, n, ext) is set iff halo coordinate l of an axis
    // lies outside the volume (inside iff 0 <= t0 + l - 1 < n); three scalar words per tile, then
    // a slot is outside iff any of its three bits is set or it is padding (1 = outside).
    auto axis_out = [](int t0, int n, int ext) __attribute__((always_inline)) {
        int lo = 1 - t0, hi = n + 1 - t0;
        if (lo < 0) lo = 0;
        if (hi > ext) hi = ext;
        return ~(((1u << hi) - 1u) & ~((1u << lo) - 1u));
    };
    auto slot_out = [](int cw, unsigned od, unsigned oh, unsigned ow) __attribute__((always_inline)) {
        const unsigned ld = cw & 255, lh = (cw >> 8) & 255, lw = (cw >> 16) & 255;
        return ((od >> ld) | (oh >> lh) | (ow >> lw) | (~(unsigned)cw >> 25)) & 1u;
    };

    // persistent workgroups and XCD-aware tile order as in conv_mfma_pipe_kernel
    auto decode = [&](int64_t vb, bool with_mask) {
        PipeTile t;
        const int64_t logical = (vb & 7) * p.per_xcd + (vb >> 3);
        t.valid = (vb >> 3) < p.per_xcd && logical < p.total;
        t.n = t.d0 = t.h0 = t.w0 = t.mb0 = 0;
        t.origin = 0;
        t.vmask = 0;
        if (t.valid) {
            unsigned tile = (unsigned)logical;
            const int cg = (int)(tile % (unsigned)p.ncg);
            tile /= (unsigned)p.ncg;
            const int twi = (int)(tile % (unsigned)p.ntw);
            tile /= (unsigned)p.ntw;
            const int thi = (int)(tile % (unsigned)p.nth);
            tile /= (unsigned)p.nth;
            const int tdi = (int)(tile % (unsigned)p.ntd);
            t.n = (int)(tile / (unsigned)p.ntd);
            t.d0 = tdi * C::TD; t.h0 = thi * C::TH; t.w0 = twi * C::TW;
            t.mb0 = cg;
            t.origin = (((int64_t)t.n * p.D + t.d0) * p.H + t.h0) * p.W + t.w0;
            if (with_mask) {
                const unsigned od = axis_out(t.d0, p.D, C::HD), oh = axis_out(t.h0, p.H, C::HH), ow = axis_out(t.w0, p.W, C::HW);
                unsigned nv = 0;
#pragma unroll
                for (int k = 0; k < C::XOPS; ++k) nv |= slot_out(coords[k], od, oh, ow) << k;
                t.vmask = ~nv;
            }
        }
        return t;
    };

    // Source of the copies of one chunk (all wave-uniform but ninv).  Every wave issues exactly
    // WOPS + XOPS copies per chunk so that the waits below can count them; a copy with nothing
    // to move writes zeros to a dump area of LDS.
    struct Src {
        __amdgpu_buffer_rsrc_t wrs, xrs;   // packed weights of (output block, tap 0, chunk) / the halo tile's first voxel, first channel of the chunk
        unsigned ninv;                     // bit k clear: halo slot k of this lane is inside the volume
        unsigned wvoff;                    // lane offset inside a weight fragment, or "nothing"
        unsigned xl, xl_last, wl, wl_last; // LDS destinations of this wave's copies 0 / of its last copy
    };
    const unsigned dump = lds0 + C::DUMP_OFF;
    const unsigned wso0 = (unsigned)(wv * nkc) * 1024u, wstep = (unsigned)(4 * nkc) * 1024u;
    auto set_src = [&](Src &s, const PipeTile &t, int c, int buf, bool ok) {
        const int ch0 = c * 16;
        const bool first = ch0 < p.c1;
        const bf16_t *src = first ? p.src1 : p.src2;
        const int chs = first ? ch0 : ch0 - p.c1;
        const int64_t halo0 = t.origin - ((int64_t)p.H * p.W + p.W + 1);
        const unsigned char *wp = reinterpret_cast<const unsigned char *>(p.packed) + (((int64_t)t.mb0 * 27) * nkc + c) * 1024;
        const unsigned char *xp = reinterpret_cast<const unsigned char *>(src) + (halo0 * p.c1 + chs) * 2;
        s.wrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(wp), 0, 0x7ffffff0, 0x00020000);
        s.xrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(xp), 0, 0x7ffffff0, 0x00020000);
        s.ninv = ok ? ~t.vmask : 0xffffffffu;
        s.wvoff = ok ? (unsigned)lane * 16u : 0xffffffffu;
        s.xl = lds0 + buf * C::XS_BYTES + wv * 1024;
        s.xl_last = (C::XOPS - 1) * 4 + wv < C::XGROUPS ? s.xl + (C::XOPS - 1) * 4096 : dump;
        s.wl = lds0 + C::W_OFF + wv * 1024;
        s.wl_last = (C::WOPS - 1) * 4 + wv < 27 ? s.wl + (C::WOPS - 1) * 4096 : dump;
    };
    auto issue_w = [&](const Src &s, int j) __attribute__((always_inline)) {
        // fragment (tap) f = 4 j + wv; the one beyond the 27 taps reads nothing into the dump area
        const bool lastj = j == C::WOPS - 1;
        const unsigned voff = (lastj && wv == 3) ? 0xffffffffu : s.wvoff;
        dma16_buf(lastj ? s.wl_last : s.wl + j * 4096, s.wrs, voff, wso0 + j * wstep);
    };
    auto issue_x = [&](const Src &s, int k) __attribute__((always_inline)) {
        // all ones where the slot is outside the volume (sign-extended bit k)
        const unsigned inv = (unsigned)__builtin_amdgcn_sbfe(s.ninv, k, 1);
        dma16_buf(k == C::XOPS - 1 ? s.xl_last : s.xl + k * 4096, s.xrs, xb[k] | inv, 0u);
    };

    // the wave's patch position inside a plane, and the lane's voxel inside the patch
    const int bh = wv >> 1, bw = wv & 1;
    const int lrow = vl >> 3, lcol = vl & 7;
    const int vbase = (bh * 4 + lrow) * C::XS_ROW + (bw * 8 + lcol) * 32 + hb * 16;   // LDS offset, tap (0,0,0), plane 0
    const int lvox = (bh * 4 + lrow) * p.W + bw * 8 + lcol;                          // voxel offset inside an output plane

    PipeTile cur = decode(blockIdx.x, false);
    if (!cur.valid) return;
    int64_t vb_next = (int64_t)blockIdx.x + gridDim.x;

    // ---- prologue: weights and halo tile of chunk 0 of the first tile, halo in plane order; each
    // slot's copy leaves as soon as its offset and validity are known
    {
        Src s0;
        set_src(s0, cur, 0, 0, true);
#pragma unroll
        for (int j = 0; j < C::WOPS; ++j) issue_w(s0, j);
        // Loads the compiler waits for (everything issued before them completes with them): the slot
        // table and the bias vector (to LDS for the whole kernel; zeros when there is none).  Behind
        // the weight copies, whose latency they share, and before the halo copies.
#pragma unroll
        for (int k = 0; k < C::XOPS; ++k) coords[k] = g_zs_slots.v[k * 256 + tid];
        {
            float *bl = reinterpret_cast<float *>(smem + C::BIAS_OFF);
            const int nco = p.cd1 + p.cd2;
            for (int i = tid; i < nco; i += 256) bl[i] = p.bias ? p.bias[i] : 0.f;
        }
        const unsigned od = axis_out(cur.d0, p.D, C::HD), oh = axis_out(cur.h0, p.H, C::HH), ow = axis_out(cur.w0, p.W, C::HW);
        unsigned nv = 0;
#pragma unroll
        for (int k = 0; k < C::XOPS; ++k) {
            xb[k] = slot_offset(coords[k]);
            const unsigned o = slot_out(coords[k], od, oh, ow);
            nv |= o << k;
            dma16_buf(k == C::XOPS - 1 ? s0.xl_last : s0.xl + k * 4096, s0.xrs, xb[k] | (0u - o), 0u);
        }
        cur.vmask = ~nv;
    }
    PipeTile nxt = decode(vb_next, true);
    // With more than one chunk the first chunk is consumed while its planes arrive (it is not
    // the one that stores, which keeps the counted waits free of conditional stores).
    const bool stream0 = nkc > 1;
    if (stream0) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::XOPS) : "memory");   // the weights: issued first
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    bf16x8 A[27];
    auto lda = [&](int tap) __attribute__((always_inline)) {
        return *reinterpret_cast<const bf16x8 *>(smem + C::W_OFF + tap * 1024 + lane * 16);
    };
#pragma unroll
    for (int t = 0; t < 27; ++t) A[t] = lda(t);

    unsigned mkb[8];   // OMASK == 2: the mask word of the lane's block in each output plane
#pragma unroll
    for (int d = 0; d < 8; ++d) mkb[d] = 0u;

    int xpar = 0;
    const float relu_floor = p.relu ? 0.f : -__builtin_inff();
    bool first = stream0;
    while (true) {
        f32x16 acc[8];
        {
            const f32x4 *bl = reinterpret_cast<const f32x4 *>(smem + C::BIAS_OFF) + (cur.mb0 * 32 + hb * 16) / 4;
            f32x4 q[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) q[i] = bl[i];
#pragma unroll
            for (int d = 0; d < 8; ++d) {
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[d][i] = q[i >> 2][i & 3];
                asm volatile("" : "+a"(acc[d]));
            }
        }
        // where the tile's results go: descriptor at the tile's first voxel and output channel,
        // the lane's byte offset inside an output plane (beyond the range where the lane's voxel
        // is outside the volume: such stores are dropped), the byte pitch of a plane
        const int dlim = p.D - cur.d0;
        const bool inhw = bh * 4 + lrow < p.H - cur.h0 && bw * 8 + lcol < p.W - cur.w0;
        const int co0 = cur.mb0 * 32;   // the lane's 16 channels start at co0 + hb * 16
        const bool d1 = co0 < p.cd1;
        const int cd = d1 ? p.cd1 : p.cd2;
        const int64_t ubase = cur.origin * cd + (d1 ? co0 : co0 - p.cd1);
        __amdgpu_buffer_rsrc_t orsrc = __builtin_amdgcn_make_buffer_rsrc((d1 ? p.dst1 : p.dst2) + ubase, 0, 0x7ffffff0, 0x00020000);
        const int obase = inhw ? (lvox * cd + hb * 16) * 2 : -1;
        const int oplane = p.H * p.W * cd * 2;
        // bit words (16 channels each): written (forward: one destination) or read (masked backward-data)
        __amdgpu_buffer_rsrc_t brsrc = __builtin_amdgcn_make_buffer_rsrc(
            (BITS ? p.bits_out : OMASK == 2 ? (unsigned short *)p.omask_bits : (unsigned short *)p.dst1) + ((BITS || OMASK == 2) && d1 ? ubase / 16 : 0),
            0, 0x7ffffff0, 0x00020000);
        const unsigned force = d1 ? 0u : 3u;   // OMASK == 2: a block of the unmasked second destination keeps both halves
        // POOL: output planes 2k, 2k+1 give pooled plane k; the maximum over the 2x2 (h, w) window is
        // taken across lanes (the lane's neighbours in w and h are lanes ^ 1 and ^ 8) and the lane
        // with even h and w stores it
        const int64_t porigin = ((((int64_t)cur.n * (p.D / 2) + cur.d0 / 2) * (p.H / 2) + cur.h0 / 2) * (p.W / 2) + cur.w0 / 2);
        __amdgpu_buffer_rsrc_t prsrc = __builtin_amdgcn_make_buffer_rsrc((POOL ? p.pool_out : p.dst1) + (POOL ? porigin * cd + co0 : 0),
                                                                         0, 0x7ffffff0, 0x00020000);
        const bool pactive = inhw && !(lrow & 1) && !(lcol & 1);
        const int pbase = pactive ? ((((bh * 4 + lrow) >> 1) * (p.W / 2) + ((bw * 8 + lcol) >> 1)) * cd + hb * 16) * 2 : -1;
        const int pplane = (p.H / 2) * (p.W / 2) * cd * 2;
        uint32_t obe[8], pb[8];
        const int bbase = inhw ? (lvox * (cd / 16) + hb) * 2 : -1;
        const int bplane = p.H * p.W * (cd / 16) * 2;

        // Output plane d leaves in 8 steps: step i converts values 2i, 2i+1 (ReLU, round to bf16),
        // step 3 stores the lower 16 bytes of the lane's 32, step 7 the upper 16 and the mask word.
        uint32_t ob[8];
        unsigned zb = 0;
        auto emit_cvt = [&](int d, int i) __attribute__((always_inline)) {
            if (i == 0) asm volatile("" : "+a"(acc[d]));   // the block stays in accumulator registers until here
            const float v0 = fmaxf(acc[d][2 * i], relu_floor), v1 = fmaxf(acc[d][2 * i + 1], relu_floor);
            uint32_t o = pack2bf(v0, v1);
            if constexpr (OMASK == 2) {
                const unsigned kk = ((mkb[d] >> (2 * i)) & 3u) | force;
                const u16x2_t keep = __builtin_bit_cast(u16x2_t, (kk | (kk << 15)) & 0x00010001u);
                o = __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2_t, o) * keep);
            }
            ob[i] = o;
            if constexpr (POOL) {
                if (d % 2 == 0) {
                    obe[i] = o;
                } else {
                    auto pkmax = [](uint32_t a, uint32_t b) __attribute__((always_inline)) {
                        return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2_t, a), __builtin_bit_cast(s16x2_t, b)));
                    };
                    uint32_t m = pkmax(obe[i], o);
                    m = pkmax(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]: lane ^ 1
                    m = pkmax(m, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)m, 0x128, 0xf, 0xf, false));   // row_ror 8: lane ^ 8
                    pb[i] = m;
                }
            }
        };
        auto emit_aux = [&](int d, int i) __attribute__((always_inline)) {
            if constexpr (BITS) zb = i == 0 ? pair_positive_pk(ob[i]) : (zb | (pair_positive_pk(ob[i]) << i));
            if (i == 3 || i == 7) {
                const int voff = d < dlim ? obase : -1;
                if (i == 3) __builtin_amdgcn_raw_buffer_store_b128(u32x4{ob[0], ob[1], ob[2], ob[3]}, orsrc, voff, d * oplane, 0);
                else __builtin_amdgcn_raw_buffer_store_b128(u32x4{ob[4], ob[5], ob[6], ob[7]}, orsrc, voff, d * oplane + 16, 0);
                if constexpr (POOL) {
                    if (d % 2 == 1) {
                        const int pvoff = d < dlim ? pbase : -1;
                        if (i == 3) __builtin_amdgcn_raw_buffer_store_b128(u32x4{pb[0], pb[1], pb[2], pb[3]}, prsrc, pvoff, (d / 2) * pplane, 0);
                        else __builtin_amdgcn_raw_buffer_store_b128(u32x4{pb[4], pb[5], pb[6], pb[7]}, prsrc, pvoff, (d / 2) * pplane + 16, 0);
                    }
                }
                if constexpr (BITS) {
                    if (i == 7) {
                        unsigned z = zb;   // even elements in bits 0..7, odd ones in bits 16..23 (see relu_bits16)
                        z = (z | (z << 4)) & 0x0F0F0F0Fu;
                        z = (z | (z << 2)) & 0x33333333u;
                        z = (z | (z << 1)) & 0x55555555u;
                        z = (z | (z >> 15)) & 0xffffu;
                        __builtin_amdgcn_raw_buffer_store_b16((short)z, brsrc, d < dlim ? bbase : -1, d * bplane, 0);
                    }
                }
            }
        };

        // One 16-channel chunk: 10 halo planes x 9 taps (kh, kw) x up to 3 output planes.  A wave
        // issues in order and alone on its SIMD, so whatever is not a matrix instruction is spread
        // thinly between the matrix instructions (one short group behind each).
        auto chunk = [&](int c, auto streamtag, auto lasttag) __attribute__((always_inline)) {
            constexpr bool STREAM = decltype(streamtag)::value;   // the chunk whose copies the prologue issued
            constexpr bool LAST = decltype(lasttag)::value;       // the chunk that completes the tile
            static_assert(!(STREAM && LAST), "the streamed chunk does not store");
            Src ns;
            if (c + 1 < nkc) set_src(ns, cur, c + 1, xpar ^ 1, true);
            else set_src(ns, nxt, 0, xpar ^ 1, nxt.valid);
            const unsigned char *xs = smem + xpar * C::XS_BYTES + vbase;
            auto ldb = [&](int q) __attribute__((always_inline)) {   // q = plane * 9 + tap
                return *reinterpret_cast<const bf16x8 *>(xs + (q / 9) * C::XS_PLANE + ((q % 9) / 3) * C::XS_ROW + (q % 3) * 32);
            };
            if constexpr (LAST && OMASK == 2) {
                // requested now, used from plane 3 on (the wait there counts the copies in between)
                if (d1) {
#pragma unroll
                    for (int d = 0; d < 8; ++d) {
                        unsigned v;
                        asm volatile("buffer_load_ushort %0, %1, %2, %3 offen" : "=v"(v) : "v"(d < dlim ? bbase : -1), "s"(brsrc), "s"(d * bplane) : "memory");
                        mkb[d] = v;
                    }
                } else {
#pragma unroll
                    for (int d = 0; d < 8; ++d) {
                        unsigned v;
                        asm volatile("buffer_load_ushort %0, %1, %2, %3 offen" : "=v"(v) : "v"(-1), "s"(brsrc), "s"(0) : "memory");
                        mkb[d] = v;
                    }
                }
            }
            constexpr int PD = 3;
            bf16x8 bq[4];
            if constexpr (!STREAM) {
#pragma unroll
                for (int q = 0; q < PD; ++q) bq[q] = ldb(q);
            }
#pragma unroll
            for (int z = 0; z < 10; ++z) {
                if constexpr (STREAM) {
                    if (z < 8) {
                        // plane z of the prologue's copies has landed once at most this many later
                        // operations of the wave are outstanding
                        wait_vm(C::XOPS - C::need(z) + C::issued_before(z));
                        __syncthreads();
                    }
                }
                if (z == 8) {
                    // the next chunk's weights and halo tile; behind the last copy (plane 6, tap 7) the
                    // wave issued the store of that step and the two of plane 7
                    wait_vm(LAST ? 3 : 0);
                    __syncthreads();
                }
                if constexpr (STREAM) {
#pragma unroll
                    for (int t = 0; t < PD; ++t) bq[(z * 9 + t) & 3] = ldb(z * 9 + t);
                }
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    const int q = z * 9 + t;
                    const int dA = z < 8 ? z : z - 1 < 8 ? z - 1 : z - 2;   // output planes of this step, oldest last
                    int nm = 0;
#pragma unroll
                    for (int kd = 0; kd < 3; ++kd) {
                        const int d = z - kd;
                        if (d < 0 || d >= 8) continue;
                        acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[kd * 9 + t], bq[q & 3], acc[d], 0, 0, 0);
                        // behind the first matrix instruction of the step: the fragment three steps ahead
                        // and the step's copy; behind the second: conversion; behind the third: the rest
                        if (nm == 0) {
                            if constexpr (STREAM) {
                                if (t + PD < 9) bq[(q + PD) & 3] = ldb(q + PD);
                            } else {
                                if (q + PD < 90) bq[(q + PD) & 3] = ldb(q + PD);
                            }
                            if (z == 1 && t < C::WOPS) issue_w(ns, t);
                            if (z >= 2 && z <= 6 && t % 3 == 1) issue_x(ns, (z - 2) * 3 + t / 3);
                        }
                        if (nm == 1 || (z == 9 && nm == 0)) {
                            if constexpr (LAST) {
                                if (z >= 3 && t < 8) {
                                    if constexpr (OMASK == 2) {
                                        if (z == 3 && t == 0) {
                                            // behind the mask requests: 7 weight copies, 3 halo copies of plane 2
                                            wait_vm(C::WOPS + 3);
#pragma unroll
                                            for (int dd = 0; dd < 8; ++dd) asm volatile("" : "+v"(mkb[dd]));
                                        }
                                    }
                                    emit_cvt(z - 3, t);
                                }
                            }
                        }
                        ++nm;
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    (void)dA;
                    // weight registers whose taps are done for this chunk take the next chunk's
                    if (z == 8) A[t] = lda(t);
                    if (z == 9) A[9 + t] = lda(9 + t);
                    if (z == 0 && !STREAM) A[18 + t] = lda(18 + t);
                    if constexpr (LAST) {
                        if (z >= 3 && t < 8) emit_aux(z - 3, t);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (z == 0 && !STREAM) __syncthreads();   // every wave holds this chunk's weights and is done with the chunk before
            }
            if constexpr (LAST) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    emit_cvt(7, i);
                    emit_aux(7, i);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            xpar ^= 1;
        };

        int c = 0;
        if (first) {
            chunk(0, std::true_type(), std::false_type());
            c = 1;
            first = false;
        }
        for (; c + 1 < nkc; ++c) chunk(c, std::false_type(), std::false_type());
        chunk(nkc - 1, std::false_type(), std::true_type());
        if (!nxt.valid) break;
        cur = nxt;
        vb_next += gridDim.x;
        nxt = decode(vb_next, true);
    }
}

static int launch_zs(MfmaParams p, int64_t mblocks, hipStream_t st)
{
    typedef ZsCfg C;
    p.ntd = (p.D + C::TD - 1) / C::TD;
    p.nth = (p.H + C::TH - 1) / C::TH;
    p.ntw = (p.W + C::TW - 1) / C::TW;
    p.ncg = (int)mblocks;
    p.total = (int64_t)p.N * p.ntd * p.nth * p.ntw * p.ncg;
    p.per_xcd = (p.total + 7) / 8;
    if (p.per_xcd * 8 > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_zs_kernel<0, false, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_zs_kernel<0, true, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_zs_kernel<0, false, true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_zs_kernel<2, false, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        attr_done = true;
    }
    int64_t grid = p.per_xcd * 8 < 256 ? p.per_xcd * 8 : 256;
    if (p.omask_bits) conv_mfma_zs_kernel<2, false, false><<<dim3((unsigned)grid), 256, C::LDS_BYTES, st>>>(p);
    else if (p.pool_out) conv_mfma_zs_kernel<0, false, true><<<dim3((unsigned)grid), 256, C::LDS_BYTES, st>>>(p);
    else if (p.bits_out) conv_mfma_zs_kernel<0, true, false><<<dim3((unsigned)grid), 256, C::LDS_BYTES, st>>>(p);
    else conv_mfma_zs_kernel<0, false, false><<<dim3((unsigned)grid), 256, C::LDS_BYTES, st>>>(p);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

template <class C>
static int launch_pipe(MfmaParams p, int64_t mblocks, hipStream_t st)
{
    p.ntd = (p.D + C::TD - 1) / C::TD;
    p.nth = (p.H + C::TH - 1) / C::TH;
    p.ntw = (p.W + C::TW - 1) / C::TW;
    p.ncg = (int)(mblocks / C::MB);
    p.total = (int64_t)p.N * p.ntd * p.nth * p.ntw * p.ncg;
    p.per_xcd = (p.total + 7) / 8;
    if (p.per_xcd * 8 > 0x7fffffffLL) return K3_E_UNSUPPORTED;
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_pipe_kernel<C, 0, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_pipe_kernel<C, 0, true>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_pipe_kernel<C, 1, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_mfma_pipe_kernel<C, 2, false>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES));
        attr_done = true;
    }
    // persistent workgroups, one per CU (fewer when there is less work); a multiple of 8
    int64_t grid = p.per_xcd * 8 < 256 ? p.per_xcd * 8 : 256;
    if (p.omask_bits) conv_mfma_pipe_kernel<C, 2, false><<<dim3((unsigned)grid), 256, C::LDS_BYTES, st>>>(p);
    else if (p.omask) conv_mfma_pipe_kernel<C, 1, false><<<dim3((unsigned)grid), 256, C::LDS_BYTES, st>>>(p);
    else if (p.bits_out) conv_mfma_pipe_kernel<C, 0, true><<<dim3((unsigned)grid), 256, C::LDS_BYTES, st>>>(p);
    else conv_mfma_pipe_kernel<C, 0, false><<<dim3((unsigned)grid), 256, C::LDS_BYTES, st>>>(p);
    K3_LAUNCH_CHECK();
    return K3_OK;
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

// Which kernel serves the launch: 1-4 the pipelined one-workgroup-per-CU kernel (8x8x16 tiles when
// they give every CU a tile, else 4x8x8 tiles -- the deep, small-volume levels of the network --
// taking one output block per workgroup where two would leave CUs without work), 0 the first kernel.
static int mfma_variant(const MfmaParams &p, int64_t mblocks)
{
    const int cmax = p.cd1 > p.cd2 ? p.cd1 : p.cd2;
    // the halo tile's voxel offsets and the per-lane output offsets are kept in 32 bits
    const int smax = p.c1 > p.c2 ? p.c1 : p.c2;
    // ... and the halo tile's voxel offsets in 24 bits, its byte offsets in 31 (the copies' offset arithmetic)
    const bool fits = (int64_t)10 * p.H * p.W * (cmax > 1 ? cmax : 1) < 0x7fffffffLL && p.cd1 + p.cd2 <= 1024 &&
                      (int64_t)11 * p.H * p.W < (1 << 24) && (int64_t)11 * p.H * p.W * smax * 2 < 0x7fffffffLL;
    if (!p.mask && fits) {
        const int64_t big = (int64_t)p.N * ((p.D + 7) / 8) * ((p.H + 7) / 8) * ((p.W + 15) / 16);
        const int64_t small = (int64_t)p.N * ((p.D + 3) / 4) * ((p.H + 7) / 8) * ((p.W + 7) / 8);
        const bool even = mblocks % 2 == 0;
        if (even && big * (mblocks / 2) >= 256) return 1;
        if (!even && big * mblocks >= 256) return 2;
        if (even && small * (mblocks / 2) >= 192) return 3;
        if (small * mblocks >= 48) return 4;
    }
    return 0;
}

// the plane-streaming kernel serves the launch: one 32-channel block per workgroup on 8x8x16 tiles,
// mask as bits or none, sources of equal channel counts
static bool zs_serves(const MfmaParams &p, int64_t mblocks)
{
    return mfma_variant(p, mblocks) == 2 && !p.omask && (p.c2 == 0 || p.c2 == p.c1);
}

static int launch_mfma(MfmaParams p, int64_t mchannels, hipStream_t st)
{
    int64_t mblocks = mchannels / 32;
    switch (mfma_variant(p, mblocks)) {
    case 1: return launch_pipe<PipeCfg<8, 8, 16, 2>>(p, mblocks, st);
    case 2: {
        if (zs_serves(p, mblocks)) return launch_zs(p, mblocks, st);
        return launch_pipe<PipeCfg<8, 8, 16, 1>>(p, mblocks, st);
    }
    case 3: return launch_pipe<PipeCfg<4, 8, 8, 2>>(p, mblocks, st);
    case 4: return launch_pipe<PipeCfg<4, 8, 8, 1>>(p, mblocks, st);
    default: break;
    }
    if (mblocks % 2 == 0) return launch_cfg<TileCfg<8, 8, 8, 2, 9>>(p, mblocks, st);
    return launch_cfg<TileCfg<8, 8, 8, 1, 27>>(p, mblocks, st);
}

int conv_fwd_mfma(const ConvArgs &a, hipStream_t st, bool *pooled)
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
    // the pipelined kernel writes the bit mask of its output itself; behind the first kernel a
    // small pass derives it from the stored tensor
    const bool native = mfma_variant(p, a.cout / 32) != 0;
    p.bits_out = native ? (unsigned short *)a.ybits : nullptr;
    // the pooled output leaves with the plane-streaming kernel's output planes (ReLU on, even sizes, no bit mask asked for)
    const bool pools = a.ypool && !a.ybits && a.relu && a.D % 2 == 0 && a.H % 2 == 0 && a.W % 2 == 0 && zs_serves(p, a.cout / 32);
    p.pool_out = pools ? (bf16_t *)a.ypool : nullptr;
    if (pooled) *pooled = pools;
    int rc = launch_mfma(p, a.cout, st);
    if (rc == K3_OK && a.ybits && !native) rc = launch_relu_bits(a.dtype, a.y, a.ybits, a.V() * a.cout / 16, st);
    return rc;
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
    p.omask = (const bf16_t *)a.omask;
    p.cd1 = (int)a.c1;
    p.cd2 = (int)a.c2;
    p.N = (int)a.N; p.D = (int)a.D; p.H = (int)a.H; p.W = (int)a.W;
    // mask given as bits: read by the pipelined kernel; behind the first kernel a small pass applies it
    const bool native = mfma_variant(p, cin / 32) != 0;
    p.omask_bits = native ? (const unsigned short *)a.omask_bits : nullptr;
    int rc = launch_mfma(p, cin, st);
    if (rc == K3_OK && a.omask_bits && !native) rc = launch_apply_relu_bits(a.dtype, a.dx, a.omask_bits, a.V() * a.c1 / 16, st);
    return rc;
}

}  // namespace k3
