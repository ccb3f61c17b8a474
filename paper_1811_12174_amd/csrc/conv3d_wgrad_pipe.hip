// Pipelined bf16 MFMA kernel for the 3x3x3 convolution backward-weight pass on gfx950.
//
// Same GEMM as conv3d_wgrad.hip, dW[tap][ci][co] = sum_v X[v + off_tap][ci] * G[v][co] with the
// contraction over voxels and the MFMA operands produced by the transposing LDS read, but
// organised as one persistent workgroup per CU that marches along the depth axis:
//
//  * A workgroup owns a 32-channel block of x, 32*COBN channels of g and a contiguous range
//    of (column, plane) pairs, a column being a 16x16 (h, w) patch of one sample.  One stage
//    multiplies one plane: 256 voxels = 16 K-steps.  The x planes d-1, d, d+1 (18x18 voxels
//    with the in-plane halo) sit in a ring of four LDS buffers, so every x plane is fetched
//    once per column and serves the three depth taps; g planes alternate between two buffers.
//  * While a stage is multiplied, x and g planes one or two stages ahead move from global
//    memory straight into the free LDS buffers (asynchronous 16-byte-per-lane copies); one
//    vmcnt wait and one barrier per stage.  The copies go through buffer descriptors: an item
//    outside the volume carries an offset beyond the descriptor's range and arrives as zeros,
//    a plane outside the volume (or beyond the run) gets a descriptor of size zero.  They are
//    issued one at a time between the MFMAs of the stage (a wave issues in order and is alone
//    on its SIMD: a burst of copy instructions would idle the matrix core).
//  * The four waves split the 27 taps (7, 7, 7, 6); the spare slot of the last wave
//    multiplies g by ones, which yields the bias gradient.  Inside a stage the operand
//    fragments of K-step s+1 are requested from LDS between the MFMAs of K-step s.
//  * Each workgroup writes one partial sum per (split, tap, ci, co); the partials are added
//    in a fixed order by reduce_partials_kernel (no atomics: run-to-run identical).
//
//  * Short problems (a handful of planes per workgroup) pay mostly for the partial sums: every
//    workgroup writes 27 x 32 x 32 floats whatever its share of the voxels.  The KS variant
//    therefore gives a workgroup one of the four tap groups and four times the planes: its
//    four waves split the K-steps of a plane (4 each) instead of the taps, add their
//    accumulators through LDS at the end (fixed order), and the partial sums shrink 4x.
//
// The kernel takes no ReLU mask: backward passes that need one hand over a gradient already
// masked by its producer, or use the kernel in conv3d_wgrad.hip.
#include "common.h"
#include "conv_internal.h"

namespace k3 {

namespace wp {
constexpr int TH = 16, TW = 16, HH = TH + 2, HW = TW + 2;
constexpr int XP_SLOTS = HH * HW * 4;              // 16-byte slots of one x plane (32 channels per voxel)
constexpr int XP_GROUPS = (XP_SLOTS + 63) / 64;    // 1 KB copy groups
constexpr int XP_BYTES = XP_GROUPS * 1024;
constexpr int XK = (XP_GROUPS + 3) / 4;            // copies per wave and x plane
constexpr int GP_BYTES1 = TH * TW * 64;            // one 32-channel block of a g plane
// PF = how many planes ahead of the multiplied one the copies run.  The x ring holds the three
// planes in use plus PF incoming ones, the g ring the one in use plus PF incoming ones.
constexpr int nxb(int pf) { return 3 + pf; }
constexpr int ngb(int pf) { return 1 + pf; }
constexpr int dump_off(int cobn, int pf) { return ngb(pf) * cobn * GP_BYTES1 + nxb(pf) * XP_BYTES; }
constexpr int lds_bytes(int cobn, int pf) { return dump_off(cobn, pf) + 1024; }
}  // namespace wp

struct WgradPipeParams {
    const bf16_t *x1, *x2;
    int c1, c2;
    const bf16_t *dy;
    int cout;
    float *ws;
    int64_t per_split;   // floats per split: 27*cin*cout + cout
    int N, D, H, W;
    int nth, ntw;        // columns per sample along h and w
    int P;               // planes in total: columns * D
    int S;               // splits of the plane range: split s owns planes [s*pbase + min(s, prem), ...)
    int pbase, prem;     // P / S and P % S
    int ncib, ncog;      // 32-channel blocks of x, groups of 32*COBN channels of g
    int total, per_xcd;
};

__device__ __forceinline__ bf16x8 wp_tr_pair(const unsigned char *base, int off)
{
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(base + off));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(base + off + 4 * 64));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

// One stage: the 16 K-steps of one plane.  K-step s covers rows 2*(s/2) + hb and columns
// 8*(s%2) .. +7 of the 16x16 patch; xa[t] / ga are the lane's LDS byte offsets of the tap-t x
// fragment and of the g fragment for K-step 0.  last (wave-uniform): the seventh slot is the
// ones product (its x fragment is still read, from a valid address, and dropped).
// The stage runs NK K-steps starting at the K-step the offsets xa / ga point to.  extra(e),
// e = 0 .. NE-1, is called behind evenly spaced MFMAs (the stage's copies).
template <int COBN, int NK, int NE, class Extra>
__device__ __forceinline__ void wp_stage(f32x16 (&acc)[7][COBN], const unsigned char *smem, const int (&xa)[7], int ga,
                                         bf16x8 ones, bool last, Extra extra)
{
    using namespace wp;
    constexpr int NF = COBN + 7;        // fragments per K-step
    constexpr int NM = 7 * COBN;        // MFMAs per K-step
    constexpr int STEP = NK * NM / NE;  // MFMAs between two calls of extra
    static_assert(STEP >= 1, "more copies than MFMAs");
    bf16x8 fr[2][COBN + 7];
    auto load = [&](int s, int f) __attribute__((always_inline)) -> bf16x8 {
        const int r2 = 2 * (s >> 1), q = 8 * (s & 1);
        if (f < COBN) return wp_tr_pair(smem, ga + f * GP_BYTES1 + (r2 * TW + q) * 64);
        return wp_tr_pair(smem, xa[f - COBN] + (r2 * HW + q) * 64);
    };
#pragma unroll
    for (int f = 0; f < NF; ++f) fr[0][f] = load(0, f);
#pragma unroll
    for (int s = 0; s < NK; ++s) {
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            if (s + 1 < NK) {
#pragma unroll
                for (int f = m * NF / NM; f < (m + 1) * NF / NM; ++f) fr[(s + 1) & 1][f] = load(s + 1, f);
            }
            const int t = m / COBN, c = m % COBN;
            const bf16x8 a = (t == 6 && last) ? ones : fr[s & 1][COBN + t];
            acc[t][c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, fr[s & 1][c], acc[t][c], 0, 0, 0);
            if ((s * NM + m) % STEP == 0 && (s * NM + m) / STEP < NE) extra((s * NM + m) / STEP);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

template <int COBN, int PF, bool KS>
__global__ __launch_bounds__(256, 1) void conv_wgrad_pipe_kernel(WgradPipeParams p)
{
    using namespace wp;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hb = lane >> 5, g16 = (lane >> 4) & 1, j = lane & 15;
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)smem;
    constexpr int NXB = nxb(PF), NGB = ngb(PF);
    // LDS map: the g ring first, then the ring of x planes, then the dump area of the padding
    // copies.  (Measured: with the x ring first and the g buffers behind it the same kernel ran
    // 2.8x slower for COBN = 2.)
    constexpr int GBUF = COBN * GP_BYTES1;
    constexpr int GOFF = 0;
    constexpr int XOFF = NGB * GBUF;
    constexpr int GK = COBN * 4;              // g copies per wave and plane
    constexpr int OPS = XK + GK;              // copies per wave and stage (always exactly this many)
    constexpr int NK = KS ? 4 : 16;           // K-steps of a plane a wave multiplies
    const unsigned dump = lds0 + dump_off(COBN, PF);

    // XCD-aware order: consecutive block ids go round-robin to the 8 XCDs, so the logical order
    // is cut into 8 contiguous runs; the workgroups of one split (same voxels, different channel
    // blocks) are neighbours in the logical order and share an L2.
    const unsigned logical = (blockIdx.x & 7u) * (unsigned)p.per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= (unsigned)p.per_xcd || logical >= (unsigned)p.total) return;
    // KS: the tap group varies fastest, so the four workgroups that read the same planes are neighbours
    const int tg = KS ? (int)(logical & 3u) : wv;        // tap group of this wave: taps 7 tg .. 7 tg + 6
    const unsigned lg = KS ? logical >> 2 : logical;
    const unsigned yz = (unsigned)(p.ncib * p.ncog);
    const int split = (int)(lg / yz);
    const int r = (int)(lg - (unsigned)split * yz);
    const int cib = r % p.ncib, cob0 = (r / p.ncib) * COBN;
    const int cin = p.c1 + p.c2;
    const bool first = cib * 32 < p.c1;
    const bf16_t *xsrc = first ? p.x1 : p.x2;
    const int Cx = first ? p.c1 : p.c2;
    const int chx = first ? cib * 32 : cib * 32 - p.c1;

    // ---- per-lane description of the copy items (tile independent)
    int xoff[XK], xco[XK];     // byte offset from the halo plane's first voxel / halo coords lh | lw << 8
    unsigned xsl = 0;          // slot holds a voxel of the 18x18 plane
#pragma unroll
    for (int k = 0; k < XK; ++k) {
        const int slot = (wv + 4 * k) * 64 + lane;
        const int vox = slot >> 2, part = slot & 3;
        const int lh = vox / HW, lw = vox - lh * HW;
        xoff[k] = (lh * p.W + lw) * Cx * 2 + part * 16;
        xco[k] = lh | (lw << 8);
        xsl |= ((wv + 4 * k < XP_GROUPS && vox < HH * HW) ? 1u : 0u) << k;
    }
    int goff[GK], gco[GK];
#pragma unroll
    for (int k = 0; k < GK; ++k) {
        const int slot = (wv + 4 * k) * 64 + lane;
        const int cb = slot / (TH * TW * 4), rem = slot - cb * (TH * TW * 4);
        const int vox = rem >> 2, part = rem & 3;
        const int lh = vox / TW, lw = vox - lh * TW;
        goff[k] = (lh * p.W + lw) * p.cout * 2 + ((cob0 + cb) * 32) * 2 + part * 16;
        gco[k] = lh | (lw << 8);
    }

    // ---- lane-constant parts of the transposing-read addresses and the wave's taps
    // (KS: the wave's K-steps 4 wv .. 4 wv + 3 are rows 4 wv .. 4 wv + 3 of the patch)
    const int krow = KS ? 4 * wv : 0;
    const int lane_x = XOFF + ((krow + hb) * HW + (j >> 2)) * 64 + g16 * 32 + (j & 3) * 8;
    const int lane_g = GOFF + ((krow + hb) * TW + (j >> 2)) * 64 + g16 * 32 + (j & 3) * 8;
    int tapoff[7], tapkd[7];
#pragma unroll
    for (int t = 0; t < 7; ++t) {
        int tap = tg * 7 + t;
        if (tap > 26) tap = 26;   // slot of the ones product: address unused
        tapkd[t] = tap / 9;
        tapoff[t] = lane_x + (((tap / 3) % 3) * HW + tap % 3) * 64;
    }

    // LDS offset of tap t's fragment when x plane i sits at ring position xb (one output block:
    // kept as a table; with two blocks the registers are needed elsewhere)
    int xatab[COBN == 1 ? NXB : 1][7];
    if constexpr (COBN == 1) {
#pragma unroll
        for (int xb = 0; xb < NXB; ++xb)
#pragma unroll
            for (int t = 0; t < 7; ++t) xatab[xb][t] = ((xb + tapkd[t]) % NXB) * XP_BYTES + tapoff[t];
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

    // ---- this split's plane range, walked column by column
    int pl = split * p.pbase + (split < p.prem ? split : p.prem);
    const int pl_end = pl + p.pbase + (split < p.prem ? 1 : 0);
    while (pl < pl_end) {
        const int col = (int)((unsigned)pl / (unsigned)p.D);
        const int dlo = pl - col * p.D;
        int run_end = (col + 1) * p.D;
        if (run_end > pl_end) run_end = pl_end;
        const int n_run = run_end - pl;   // planes of this run
        pl = run_end;
        const int twi = (int)((unsigned)col % (unsigned)p.ntw);
        const int q1 = (int)((unsigned)col / (unsigned)p.ntw);
        const int thi = (int)((unsigned)q1 % (unsigned)p.nth);
        const int n = (int)((unsigned)q1 / (unsigned)p.nth);
        const int h0 = thi * TH, w0 = twi * TW;

        // per-lane offsets of this column's items; beyond every descriptor's range where the item
        // lies outside the volume (in-plane test) or is padding
        unsigned xo[XK], go[GK];
#pragma unroll
        for (int k = 0; k < XK; ++k) {
            const unsigned gh = h0 + (xco[k] & 255) - 1, gw = w0 + (xco[k] >> 8) - 1;
            xo[k] = (((xsl >> k) & 1) && gh < (unsigned)p.H && gw < (unsigned)p.W) ? (unsigned)xoff[k] : 0xffffffffu;
        }
#pragma unroll
        for (int k = 0; k < GK; ++k) {
            const int gh = h0 + (gco[k] & 255), gw = w0 + (gco[k] >> 8);
            go[k] = (gh < p.H && gw < p.W) ? (unsigned)goff[k] : 0xffffffffu;
        }
        // element index of voxel (n, 0, h0, w0); planes are p.H * p.W voxels apart
        const int64_t vox0 = (((int64_t)n * p.D) * p.H + h0) * p.W + w0;
        const int64_t plane = (int64_t)p.H * p.W;

        // x plane with run index q (plane dlo - 1 + q) -> ring buffer buf; `on` false: padding copies
        struct PlaneSrc {
            __amdgpu_buffer_rsrc_t rs;
            unsigned lds;     // LDS address of this wave's first copy group in the destination buffer
            bool on;
        };
        auto x_plane = [&](int q, int buf, bool on) __attribute__((always_inline)) {
            const int d = dlo - 1 + q;
            const bool din = on && d >= 0 && d < p.D;
            // the halo plane's first voxel: one row and one column before the column's origin
            const bf16_t *base = xsrc + (vox0 + d * plane - (p.W + 1)) * Cx + chx;
            PlaneSrc s;
            s.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(base), 0, din ? 0x7ffffff0 : 0, 0x00020000);
            s.lds = lds0 + XOFF + buf * XP_BYTES + wv * 1024;
            s.on = on;
            return s;
        };
        auto x_copy = [&](const PlaneSrc &s, int k) __attribute__((always_inline)) {
            const bool grp = s.on && wv + 4 * k < XP_GROUPS;
            dma16_buf(grp ? s.lds + k * 4096 : dump, s.rs, xo[k], 0u);
        };
        // g plane with run index i (plane dlo + i)
        auto g_plane = [&](int i, int buf, bool on) __attribute__((always_inline)) {
            const bf16_t *base = p.dy + (vox0 + (dlo + i) * plane) * p.cout;
            PlaneSrc s;
            s.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(base), 0, on ? 0x7ffffff0 : 0, 0x00020000);
            s.lds = lds0 + GOFF + buf * GBUF + wv * 1024;
            s.on = on;
            return s;
        };
        auto g_copy = [&](const PlaneSrc &s, int k) __attribute__((always_inline)) {
            dma16_buf(s.on ? s.lds + k * 4096 : dump, s.rs, go[k], 0u);
        };
        auto issue_x = [&](int q, int buf, bool on) __attribute__((always_inline)) {
            const PlaneSrc s = x_plane(q, buf, on);
#pragma unroll
            for (int k = 0; k < XK; ++k) x_copy(s, k);
        };
        auto issue_g = [&](int i, int buf, bool on) __attribute__((always_inline)) {
            const PlaneSrc s = g_plane(i, buf, on);
#pragma unroll
            for (int k = 0; k < GK; ++k) g_copy(s, k);
        };

        // Prologue of the run: what stage 0 reads (x planes 0..2, g plane 0), then the planes the
        // first PF - 1 stages would have fetched.  The barrier also closes the previous run.
        // Stage i reads x planes i..i+2 and g plane i, and fetches x plane i+2+PF and g plane
        // i+PF when stage i+PF exists; at its end only the copies of the last PF-1 stages may
        // still be in flight (copies complete in issue order).
        __syncthreads();
        issue_x(0, 0, true);
        issue_x(1, 1, true);
        issue_x(2, 2, true);
        issue_g(0, 0, true);
#pragma unroll
        for (int e = 1; e < PF; ++e) {
            issue_x(2 + e, 2 + e, e < n_run);
            issue_g(e, e, e < n_run);
        }
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((PF - 1) * OPS) : "memory");
        __syncthreads();

        // The loop is unrolled over the x ring, so the ring position of x plane i is a constant in
        // each body (the taps' LDS offsets come from a table made once); the sources of the planes a
        // stage fetches advance by one plane per stage.  With a short stage (the KS variant has 28
        // MFMAs) the scalar bookkeeping of a stage otherwise outweighs its matrix work.
        int gb = 0, i = 0;   // ring buffer of g plane i; stage
        int dnext = dlo + 1 + PF;                                  // depth index of the x plane that stage i fetches
        const bf16_t *xnext = xsrc + (vox0 + dnext * plane - (p.W + 1)) * Cx + chx;
        const bf16_t *gnext = p.dy + (vox0 + (dlo + PF) * plane) * p.cout;
        const int64_t xstep = plane * Cx, gstep = plane * p.cout;
        bool more = n_run > 0;
        while (more) {
#pragma unroll
            for (int xb = 0; xb < NXB; ++xb) {
                const int xn = (xb + 2 + PF) % NXB;
                int gn = gb + PF; if (gn >= NGB) gn -= NGB;
                const bool on = i + PF < n_run;
                PlaneSrc sx, sg;
                sx.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(xnext), 0, (on && dnext >= 0 && dnext < p.D) ? 0x7ffffff0 : 0, 0x00020000);
                sx.lds = lds0 + XOFF + xn * XP_BYTES + wv * 1024;
                sx.on = on;
                sg.rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(gnext), 0, on ? 0x7ffffff0 : 0, 0x00020000);
                sg.lds = lds0 + GOFF + gn * GBUF + wv * 1024;
                sg.on = on;
                int xa[7];
#pragma unroll
                for (int t = 0; t < 7; ++t) {
                    if constexpr (COBN == 1) {
                        xa[t] = xatab[xb][t];
                    } else {
                        int bsel = xb + tapkd[t]; if (bsel >= NXB) bsel -= NXB;
                        xa[t] = bsel * XP_BYTES + tapoff[t];
                    }
                }
                const int ga = lane_g + gb * GBUF;
                wp_stage<COBN, NK, OPS>(acc, smem, xa, ga, ones, tg == 3, [&](int e) __attribute__((always_inline)) {
                    if (e < XK) x_copy(sx, e);
                    else g_copy(sg, e - XK);
                });
                asm volatile("s_waitcnt vmcnt(%0)" ::"n"((PF - 1) * OPS) : "memory");
                __syncthreads();
                if (++gb == NGB) gb = 0;
                xnext += xstep;
                gnext += gstep;
                ++dnext;
                if (++i >= n_run) {
                    more = false;
                    break;
                }
            }
        }
    }

    if constexpr (KS) {
        // the four waves hold sums over different voxels of the same taps: through LDS (the rings
        // are no longer read after the barrier that ended the last stage), wave w adds up taps w
        // and w + 4 of the group in the fixed order wave 0, 1, 2, 3
        static_assert(COBN == 1, "K split is built for one output block");
        static_assert(4 * 7 * 16 * 256 <= lds_bytes(COBN, PF), "reduction buffer fits the rings");
        f32x4 *red = reinterpret_cast<f32x4 *>(smem);
#pragma unroll
        for (int t = 0; t < 7; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                red[((wv * 7 + t) * 4 + q) * 64 + lane] = f32x4{acc[t][0][4 * q], acc[t][0][4 * q + 1], acc[t][0][4 * q + 2], acc[t][0][4 * q + 3]};
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 7; ++t) {
            if (t != wv && t != wv + 4) continue;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                f32x4 s = red[((0 * 7 + t) * 4 + q) * 64 + lane];
#pragma unroll
                for (int u = 1; u < 4; ++u) {
                    const f32x4 v = red[((u * 7 + t) * 4 + q) * 64 + lane];
                    s[0] += v[0]; s[1] += v[1]; s[2] += v[2]; s[3] += v[3];
                }
                acc[t][0][4 * q] = s[0]; acc[t][0][4 * q + 1] = s[1]; acc[t][0][4 * q + 2] = s[2]; acc[t][0][4 * q + 3] = s[3];
            }
        }
    }
    float *out = p.ws + (int64_t)split * p.per_split;
#pragma unroll
    for (int t = 0; t < 7; ++t) {
        if (KS && t != wv && t != wv + 4) continue;
        const int tap = tg * 7 + t;
#pragma unroll
        for (int c = 0; c < COBN; ++c) {
            const int co = (cob0 + c) * 32 + (lane & 31);
            if (tap <= 26) {
                // rows ci = cib*32 + (i/4)*8 + hb*4 + i%4 of this tap's [cin][cout] block
                float *o = out + ((int64_t)tap * cin + cib * 32 + hb * 4) * p.cout + co;
#pragma unroll
                for (int i = 0; i < 16; ++i) o[((i >> 2) * 8 + (i & 3)) * p.cout] = acc[t][c][i];
            } else if (cib == 0 && hb == 0) {
                out[(int64_t)27 * cin * p.cout + co] = acc[t][c][0];   // row 0 of ones^T * g
            }
        }
    }
}

static int wp_num_cus()
{
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

static constexpr int wp_pf(int cobn) { return cobn == 1 ? 2 : 1; }   // deeper read-ahead where a stage is short

// ks: with fewer than 12 planes per workgroup the workgroups take one tap group each and four
// times the planes (see the KS variant of the kernel)
static void wp_plan(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout, int *cobn, int64_t *P,
                    int *S, bool *ks)
{
    *cobn = (cout % 64 == 0) ? 2 : 1;
    *P = N * ((H + wp::TH - 1) / wp::TH) * ((W + wp::TW - 1) / wp::TW) * D;
    const int64_t yz = (cin / 32) * (cout / (32 * *cobn));
    int64_t s = wp_num_cus() / yz;   // one workgroup per CU in total
    *ks = *cobn == 1 && s >= 4 && *P < 12 * s && *P >= s / 4;
    if (*ks) s /= 4;
    if (s > *P) s = *P;
    if (s < 1) s = 1;
    *S = (int)s;
}

bool conv_wgrad_pipe_ok(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout)
{
    // byte offsets inside one plane and the plane / workgroup counts are kept in 32 bits
    const int64_t c = cin > cout ? cin : cout;
    const int64_t P = N * ((H + wp::TH - 1) / wp::TH) * ((W + wp::TW - 1) / wp::TW) * D;
    return (int64_t)(wp::HH + 1) * W * c * 2 < 0x7fffffffLL && H * W * c * 2 < 0x7fffffffLL && P < 0x3fffffffLL &&
           (cin / 32) * (cout / 32) < 0x100000LL;
}

size_t conv_wgrad_pipe_ws_bytes(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout)
{
    int cobn, S;
    int64_t P;
    bool ks;
    wp_plan(N, D, H, W, cin, cout, &cobn, &P, &S, &ks);
    return (size_t)S * (size_t)(27 * cin * cout + cout) * sizeof(float);
}

template <int COBN, bool KS>
static int launch_wgrad_pipe(const WgradPipeParams &p, hipStream_t st)
{
    constexpr int PF = wp_pf(COBN);
    constexpr int lds = wp::lds_bytes(COBN, PF);
    static_assert(lds <= 160 * 1024, "LDS budget");
    static bool attr_done = false;
    if (!attr_done) {
        K3_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&conv_wgrad_pipe_kernel<COBN, PF, KS>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        attr_done = true;
    }
    conv_wgrad_pipe_kernel<COBN, PF, KS><<<dim3((unsigned)(p.per_xcd * 8)), 256, lds, st>>>(p);
    K3_LAUNCH_CHECK();
    return K3_OK;
}

int conv_wgrad_pipe(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st)
{
    WgradPipeParams p{};
    const int64_t cin = a.c1 + a.c2;
    int cobn;
    int64_t P;
    bool ks;
    wp_plan(a.N, a.D, a.H, a.W, cin, a.cout, &cobn, &P, &p.S, &ks);
    p.P = (int)P;
    p.pbase = p.P / p.S;
    p.prem = p.P % p.S;
    p.x1 = (const bf16_t *)a.x;
    p.x2 = (const bf16_t *)a.x2;
    p.c1 = (int)a.c1;
    p.c2 = (int)a.c2;
    p.dy = (const bf16_t *)a.dy;
    p.cout = (int)a.cout;
    p.ws = ws;
    p.per_split = 27 * cin * a.cout + a.cout;
    p.N = (int)a.N; p.D = (int)a.D; p.H = (int)a.H; p.W = (int)a.W;
    p.nth = (int)((a.H + wp::TH - 1) / wp::TH);
    p.ntw = (int)((a.W + wp::TW - 1) / wp::TW);
    p.ncib = (int)(cin / 32);
    p.ncog = (int)(a.cout / (32 * cobn));
    const int64_t total = (int64_t)p.S * p.ncib * p.ncog * (ks ? 4 : 1);
    if (total > 0x3fffffffLL) return K3_E_UNSUPPORTED;
    p.total = (int)total;
    p.per_xcd = (p.total + 7) / 8;
    int rc = cobn == 2 ? launch_wgrad_pipe<2, false>(p, st)
                       : (ks ? launch_wgrad_pipe<1, true>(p, st) : launch_wgrad_pipe<1, false>(p, st));
    if (rc != K3_OK) return rc;
    return launch_reduce_partials(ws, dW, db, 27 * cin * a.cout, p.per_split, p.S, st);
}

}  // namespace k3
