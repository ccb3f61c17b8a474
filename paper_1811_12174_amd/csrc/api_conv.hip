// C-ABI entry points for the 3x3x3 convolution passes: argument validation and dispatch
// between the MFMA implicit-GEMM kernels and the direct kernels.
#include "common.h"
#include "conv_internal.h"
#include <mutex>

namespace k3 {
static thread_local int g_last_hip_error = 0;
void set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
}  // namespace k3

using namespace k3;

// Split-K partial sums of k3_conv3d_bwd_weight_static: one array per GPU, part of the loaded
// code object, held until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels, and every other use, get the device address kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[K3_STATIC_SCRATCH_BYTES];

static constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, looked up once
static std::mutex g_scratch_lock;

// Address of the current device's copy of the array (each GPU has its own, at its own address).
static int scratch_for_current_device(void **ptr)
{
    int dev = -1;
    K3_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return K3_E_UNSUPPORTED;
    std::lock_guard<std::mutex> g(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        K3_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return K3_E_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return K3_OK;
}

extern "C" {

int k3_version(void) { return 104; }
int k3_last_hip_error(void) { return g_last_hip_error; }

const char *k3_status_string(int s)
{
    switch (s) {
    case K3_OK: return "ok";
    case K3_E_BADARG: return "bad argument";
    case K3_E_SHAPE: return "shape mismatch";
    case K3_E_UNSUPPORTED: return "unsupported dtype or channel count";
    case K3_E_WORKSPACE: return "workspace too small";
    case K3_E_OOM: return "device budget or table exhausted";
    case K3_E_NOT_PINNED: return "host pointer is not page-locked";
    case K3_E_STATE: return "illegal swap-state transition";
    case K3_E_HIP: return "HIP error";
    default: return "unknown status";
    }
}

int k3_conv3d_packed_bytes(int64_t cin, int64_t cout, int dtype, size_t *bytes)
{
    if (!bytes || cin <= 0 || cout <= 0 || (dtype != K3_BF16 && dtype != K3_F32)) return K3_E_BADARG;
    // the packed form does not depend on how C_in is split over two sources
    *bytes = (dtype == K3_BF16 && cin % 32 == 0 && cout % 32 == 0) ? conv_packed_bytes(cin, cout) : 0;
    return K3_OK;
}

int k3_conv3d_pack_weights(const void *w, int64_t cin, int64_t cout, int dtype, void *packed, size_t packed_bytes,
                           void *stream)
{
    size_t need = 0;
    int rc = k3_conv3d_packed_bytes(cin, cout, dtype, &need);
    if (rc != K3_OK) return rc;
    if (need == 0) return K3_OK;
    if (!w || !packed) return K3_E_BADARG;
    if (packed_bytes < need) return K3_E_WORKSPACE;
    return conv_pack_weights(w, cin, cout, packed, (hipStream_t)stream);
}

// Validates a (two-source) input / output descriptor set and fills the common fields.
static int fill_args(ConvArgs &a, const k3_tensor *xd, const k3_tensor *x2d, const void *x2, const k3_tensor *yd)
{
    if (!desc_ok(xd) || !desc_ok(yd)) return K3_E_BADARG;
    if ((x2d == nullptr) != (x2 == nullptr)) return K3_E_BADARG;
    if (x2d && !desc_ok(x2d)) return K3_E_BADARG;
    if (!same_space(xd, yd) || xd->dtype != yd->dtype) return K3_E_SHAPE;
    if (x2d && (!same_space(xd, x2d) || x2d->dtype != xd->dtype)) return K3_E_SHAPE;
    if (xd->d > 0x3fffffff || xd->h > 0x3fffffff || xd->w > 0x3fffffff || xd->n > 0x3fffffff) return K3_E_UNSUPPORTED;
    a.dtype = xd->dtype;
    a.N = xd->n; a.D = xd->d; a.H = xd->h; a.W = xd->w;
    a.c1 = xd->c;
    a.c2 = x2d ? x2d->c : 0;
    a.cout = yd->c;
    return K3_OK;
}

static int conv_fwd_any(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2, const void *w,
                        const void *packed, const float *bias, int relu, const k3_tensor *yd, void *y, void *relu_bits,
                        void *stream, void *ypool = nullptr, bool *pooled = nullptr)
{
    ConvArgs a;
    int rc = fill_args(a, xd, x2d, x2, yd);
    if (rc != K3_OK) return rc;
    if (!x || !w || !y) return K3_E_BADARG;
    if (relu_bits && a.cout % 16 != 0) return K3_E_UNSUPPORTED;
    a.x = x; a.x2 = x2; a.w = w; a.packed = packed; a.bias = bias; a.relu = relu ? 1 : 0; a.y = y; a.ybits = relu_bits;
    a.ypool = ypool;
    if (pooled) *pooled = false;
    hipStream_t st = (hipStream_t)stream;
    if (mfma_ok(a.dtype, a.c1, a.c2, a.cout)) {
        if (!packed) return K3_E_BADARG;
        return conv_fwd_mfma(a, st, pooled);   // writes the bits itself (or runs the generic pass)
    }
    if (conv_first_ok(a.dtype, a.c1, a.c2, a.cout)) return conv_first_fwd(a, st);   // likewise
    rc = conv_fwd_direct(a, st);
    if (rc == K3_OK && relu_bits) rc = launch_relu_bits(a.dtype, y, relu_bits, a.V() * a.cout / 16, st);
    return rc;
}

int k3_conv3d_fwd(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2, const void *w,
                  const void *packed, const float *bias, int relu, const k3_tensor *yd, void *y, void *stream)
{
    return conv_fwd_any(xd, x, x2d, x2, w, packed, bias, relu, yd, y, nullptr, stream);
}

int k3_conv3d_fwd_pool(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2, const void *w,
                       const void *packed, const float *bias, int relu, const k3_tensor *yd, void *y,
                       const k3_tensor *pd, void *y_pooled, void *stream)
{
    if (!desc_ok(yd) || !desc_ok(pd) || !y_pooled) return K3_E_BADARG;
    if (yd->d % 2 || yd->h % 2 || yd->w % 2) return K3_E_SHAPE;
    if (pd->n != yd->n || pd->d * 2 != yd->d || pd->h * 2 != yd->h || pd->w * 2 != yd->w || pd->c != yd->c ||
        pd->dtype != yd->dtype)
        return K3_E_SHAPE;
    bool pooled = false;
    int rc = conv_fwd_any(xd, x, x2d, x2, w, packed, bias, relu, yd, y, nullptr, stream, y_pooled, &pooled);
    if (rc != K3_OK || pooled) return rc;
    return k3_pool3d_fwd(yd, y, pd, y_pooled, stream);   // the convolution kernel that ran does not pool: a second pass
}

int k3_relu_bits_bytes(const k3_tensor *yd, size_t *bytes)
{
    if (!desc_ok(yd) || !bytes) return K3_E_BADARG;
    if (yd->c % 16 != 0) return K3_E_UNSUPPORTED;
    *bytes = (size_t)voxels(yd) * (size_t)(yd->c / 16) * sizeof(uint16_t);
    return K3_OK;
}

int k3_conv3d_fwd_bits(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2, const void *w,
                       const void *packed, const float *bias, int relu, const k3_tensor *yd, void *y, void *relu_bits,
                       void *stream)
{
    if (!relu_bits) return K3_E_BADARG;
    return conv_fwd_any(xd, x, x2d, x2, w, packed, bias, relu, yd, y, relu_bits, stream);
}

static int conv_dgrad_any(const k3_tensor *dyd, const void *dy, const void *y_mask, const void *w, const void *packed,
                          const k3_tensor *dxd, void *dx, const k3_tensor *dx2d, void *dx2, const void *dx_mask,
                          const void *dx_mask_bits, void *stream)
{
    ConvArgs a;
    int rc = fill_args(a, dxd, dx2d, dx2, dyd);
    if (rc != K3_OK) return rc;
    if (!dy || !w || !dx) return K3_E_BADARG;
    if (dx_mask && dx_mask_bits) return K3_E_BADARG;
    if (dx_mask_bits && a.c1 % 16 != 0) return K3_E_UNSUPPORTED;
    a.dy = dy; a.ymask = y_mask; a.w = w; a.packed = packed; a.dx = dx; a.dx2 = dx2; a.omask = dx_mask;
    a.omask_bits = dx_mask_bits;
    hipStream_t st = (hipStream_t)stream;
    if (mfma_ok(a.dtype, a.c1, a.c2, a.cout)) {
        if (!packed) return K3_E_BADARG;
        return conv_dgrad_mfma(a, st);   // reads the bits itself (or runs the generic pass)
    }
    rc = conv_dgrad_direct(a, st);
    if (rc == K3_OK && dx_mask_bits) rc = launch_apply_relu_bits(a.dtype, dx, dx_mask_bits, a.V() * a.c1 / 16, st);
    return rc;
}

int k3_conv3d_bwd_data(const k3_tensor *dyd, const void *dy, const void *y_mask, const void *w, const void *packed,
                       const k3_tensor *dxd, void *dx, const k3_tensor *dx2d, void *dx2, const void *dx_mask,
                       void *stream)
{
    return conv_dgrad_any(dyd, dy, y_mask, w, packed, dxd, dx, dx2d, dx2, dx_mask, nullptr, stream);
}

int k3_conv3d_bwd_data_bits(const k3_tensor *dyd, const void *dy, const void *y_mask, const void *w, const void *packed,
                            const k3_tensor *dxd, void *dx, const k3_tensor *dx2d, void *dx2, const void *dx_mask_bits,
                            void *stream)
{
    if (!dx_mask_bits) return K3_E_BADARG;
    return conv_dgrad_any(dyd, dy, y_mask, w, packed, dxd, dx, dx2d, dx2, nullptr, dx_mask_bits, stream);
}

int k3_conv3d_bwd_weight_workspace_bytes(const k3_tensor *xd, const k3_tensor *x2d, const k3_tensor *dyd, size_t *bytes)
{
    if (!desc_ok(xd) || !desc_ok(dyd) || !bytes || (x2d && !desc_ok(x2d))) return K3_E_BADARG;
    if (!same_space(xd, dyd) || (x2d && !same_space(xd, x2d))) return K3_E_SHAPE;
    int64_t c1 = xd->c, c2 = x2d ? x2d->c : 0;
    if (mfma_ok(xd->dtype, c1, c2, dyd->c))
        *bytes = conv_wgrad_mfma_ws_bytes(xd->n, xd->d, xd->h, xd->w, c1 + c2, dyd->c);
    else if (conv_first_ok(xd->dtype, c1, c2, dyd->c))
        *bytes = conv_first_wgrad_ws_bytes(xd->n, xd->d, xd->h, xd->w, dyd->c);
    else
        *bytes = conv_wgrad_direct_ws_bytes(voxels(xd), c1 + c2, dyd->c);
    return K3_OK;
}

// Partial-sum bytes of the kernel a backward-weight call with these shapes runs on; the size
// query of the boundary reports the larger of the masked and the unmasked case.
static size_t bwd_weight_need(const k3_tensor *xd, const k3_tensor *x2d, const k3_tensor *dyd, bool masked)
{
    const int64_t c1 = xd->c, c2 = x2d ? x2d->c : 0;
    if (mfma_ok(xd->dtype, c1, c2, dyd->c))
        return conv_wgrad_mfma_ws_bytes_for(xd->n, xd->d, xd->h, xd->w, c1 + c2, dyd->c, masked);
    if (conv_first_ok(xd->dtype, c1, c2, dyd->c)) return conv_first_wgrad_ws_bytes(xd->n, xd->d, xd->h, xd->w, dyd->c);
    return conv_wgrad_direct_ws_bytes(voxels(xd), c1 + c2, dyd->c);
}

// Validation and dispatch shared by the two backward-weight entry points.
static int bwd_weight_run(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2, const k3_tensor *dyd,
                          const void *dy, const void *y_mask, float *dW, float *db, void *ws, size_t ws_bytes,
                          void *stream)
{
    ConvArgs a;
    int rc = fill_args(a, xd, x2d, x2, dyd);
    if (rc != K3_OK) return rc;
    if (!x || !dy || !dW || !ws) return K3_E_BADARG;
    if (ws_bytes < bwd_weight_need(xd, x2d, dyd, y_mask != nullptr)) return K3_E_WORKSPACE;
    a.x = x; a.x2 = x2; a.dy = dy; a.ymask = y_mask;
    if (mfma_ok(a.dtype, a.c1, a.c2, a.cout)) return conv_wgrad_mfma(a, dW, db, (float *)ws, (hipStream_t)stream);
    if (conv_first_ok(a.dtype, a.c1, a.c2, a.cout)) return conv_first_wgrad(a, dW, db, (float *)ws, (hipStream_t)stream);
    return conv_wgrad_direct(a, dW, db, (float *)ws, (hipStream_t)stream);
}

int k3_conv3d_bwd_weight(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2,
                         const k3_tensor *dyd, const void *dy, const void *y_mask, float *dW, float *db, void *ws,
                         size_t ws_bytes, void *stream)
{
    return bwd_weight_run(xd, x, x2d, x2, dyd, dy, y_mask, dW, db, ws, ws_bytes, stream);
}

int k3_conv3d_bwd_weight_static(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2,
                                const k3_tensor *dyd, const void *dy, const void *y_mask, float *dW, float *db,
                                void *stream)
{
    // shapes whose partial sums do not fit the array are refused before anything is looked up or launched
    size_t any = 0;
    int rc = k3_conv3d_bwd_weight_workspace_bytes(xd, x2d, dyd, &any);   // validates the descriptors
    if (rc != K3_OK) return rc;
    if (bwd_weight_need(xd, x2d, dyd, y_mask != nullptr) > (size_t)K3_STATIC_SCRATCH_BYTES) return K3_E_WORKSPACE;
    void *ws = nullptr;
    rc = scratch_for_current_device(&ws);
    if (rc != K3_OK) return rc;
    // every partial sum the reduction pass reads is written by this call's own first kernel, so
    // what an earlier call left in the array needs no clearing
    return bwd_weight_run(xd, x, x2d, x2, dyd, dy, y_mask, dW, db, ws, (size_t)K3_STATIC_SCRATCH_BYTES, stream);
}

}  // extern "C"
