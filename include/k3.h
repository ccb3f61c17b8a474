/*
 * k3 -- C-ABI boundary of the MI355X (gfx950) 3-D U-Net training-step kernels and the
 * Large-Model-Support (LMS) activation swap engine.
 *
 * What the calls compute follows the paper's statement of the problem: a 3-D
 * encoder/decoder segmentation network built from 3x3x3 convolution layers, 2x2x2
 * max-pooling layers, an up-sampling decoder layer and a per-voxel three-class
 * likelihood (sections 3 and 4.1), trained with activations that are parked in host
 * memory between their forward and backward use (section 2.2).
 *
 * Conventions
 *  - Every function returns an int status: K3_OK (0) or a negative K3_E_* code.  No
 *    exceptions, no aborts.  k3_last_hip_error() returns the last HIP error seen by
 *    the calling thread when the status was K3_E_HIP.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *    The caller owns every buffer it passes; the library only borrows pointers for
 *    the work it enqueues and keeps none after that work has run.
 *  - Compute calls are asynchronous: they enqueue kernels on the caller's stream
 *    (`stream` is a hipStream_t passed as void*; NULL is the default stream) and do
 *    not synchronise.
 *  - Activations are dense NDHWC (channel fastest).  3x3x3 weights are
 *    [kd][kh][kw][C_in][C_out]; transposed-conv weights [i][j][k][C_in][C_out]; head
 *    weights [C][K]; all in the activation dtype except the head (fp32).  Biases,
 *    weight gradients, bias gradients, logits and the loss are fp32.
 *  - bf16 tensors hold round-to-nearest-even values; all accumulation is fp32.
 *  - Results are run-to-run bit-identical: no floating-point atomics are used.
 */
#ifndef K3_H
#define K3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    K3_OK = 0,
    K3_E_BADARG = -1,      /* null pointer, negative size, unknown dtype */
    K3_E_SHAPE = -2,       /* descriptors disagree, odd dimension given to pooling */
    K3_E_UNSUPPORTED = -3, /* dtype / channel combination has no kernel */
    K3_E_WORKSPACE = -4,   /* workspace or packed buffer too small */
    K3_E_OOM = -5,         /* device budget or handle table exhausted */
    K3_E_NOT_PINNED = -6,  /* host pointer is not page-locked */
    K3_E_STATE = -7,       /* illegal swap-state transition */
    K3_E_HIP = -8          /* a HIP call failed; see k3_last_hip_error() */
};

enum { K3_BF16 = 1, K3_F32 = 2 };

/* Shape and element type of a dense NDHWC tensor. */
typedef struct k3_tensor {
    int64_t n, d, h, w, c;
    int32_t dtype;    /* K3_BF16 or K3_F32 */
    int32_t reserved; /* must be 0 */
} k3_tensor;

const char *k3_status_string(int status);
int k3_last_hip_error(void);
/* Library ABI version (major * 100 + minor). */
int k3_version(void);

/* ------------------------------------------------------------------ 3x3x3 convolution
 * The 3x3x3 convolutional layer of the encoder and decoder (section 4.1), stride 1,
 * zero padding 1 (cross-correlation):
 *   y[n,d,h,w,co] = act(bias[co] + sum_{kd,kh,kw,ci} x[n,d+kd-1,h+kh-1,w+kw-1,ci] * W[kd,kh,kw,ci,co])
 *
 * bf16 tensors whose channel counts are multiples of 32 run on the MFMA implicit-GEMM
 * kernels and need the weights in a packed device buffer made by k3_conv3d_pack_weights;
 * every other case (fp32, or small / odd channel counts) runs on direct kernels that
 * read the canonical weights.  k3_conv3d_packed_bytes reports 0 for the latter.
 */

/* Bytes needed for the packed form of a C_in -> C_out weight tensor (0: not needed). */
int k3_conv3d_packed_bytes(int64_t cin, int64_t cout, int dtype, size_t *bytes);

/* Builds the packed forms (forward and backward-data operand order) of canonical
 * weights w (dev) into packed (dev, caller-owned, packed_bytes long).  Must be
 * called again whenever w changes.  A no-op returning K3_OK when no packed form exists. */
int k3_conv3d_pack_weights(const void *w, int64_t cin, int64_t cout, int dtype,
                           void *packed, size_t packed_bytes, void *stream);

/* Forward pass with fused bias and optional ReLU.  The input may be given as two
 * tensors of equal n,d,h,w that are concatenated along channels, [x | x2] (the skip
 * connection of a decoder level); pass x2d = x2 = NULL for one input.  w is
 * [3][3][3][C_in][C_out] with C_in = x.c + x2.c; bias may be NULL (zero).  packed may
 * be NULL only when k3_conv3d_packed_bytes reports 0.  All pointers dev. */
int k3_conv3d_fwd(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2,
                  const void *w, const void *packed, const float *bias, int relu,
                  const k3_tensor *yd, void *y, void *stream);

/* k3_conv3d_fwd followed by the 2x2x2 max-pool of its output (the "convolution ... then
 * max-pooling" pair that ends an encoder level, section 4.1): y receives the convolution
 * output as k3_conv3d_fwd writes it, y_pooled (n, d/2, h/2, w/2, c; same dtype) what
 * k3_pool3d_fwd would compute from y, bit for bit.  Where the convolution kernel that serves
 * the shape can, the pooled planes leave with its output planes (one pass); otherwise the
 * pooling kernel runs behind it on the same stream.  d, h, w must be even (K3_E_SHAPE).
 * All pointers dev, caller-owned. */
int k3_conv3d_fwd_pool(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2,
                       const void *w, const void *packed, const float *bias, int relu,
                       const k3_tensor *yd, void *y, const k3_tensor *pd, void *y_pooled, void *stream);

/* Backward-data pass: with g = dy where y_mask > 0 else 0 (g = dy when y_mask is NULL),
 *   dx[n,d,h,w,ci] = sum_{kd,kh,kw,co} g[n,d-kd+1,h-kh+1,w-kw+1,co] * W[kd,kh,kw,ci,co].
 * y_mask is the stored forward output of the same layer (same shape and dtype as dy).
 * The result may be split along channels into two tensors [dx | dx2] (pass NULLs for
 * one output).  When dx_mask is not NULL (same shape and dtype as dx) the first output is
 * zeroed where dx_mask <= 0: dx is the gradient of a stored ReLU output, and applying that
 * layer's mask here, once, lets its backward passes run with y_mask = NULL (their fastest
 * path: a masked input cannot be copied asynchronously into LDS). */
int k3_conv3d_bwd_data(const k3_tensor *dyd, const void *dy, const void *y_mask,
                       const void *w, const void *packed,
                       const k3_tensor *dxd, void *dx, const k3_tensor *dx2d, void *dx2,
                       const void *dx_mask, void *stream);

/* One-bit-per-element form of the ReLU mask.  A stored ReLU output y with C channels
 * (C a multiple of 16, K3_E_UNSUPPORTED otherwise) has the bit tensor
 *   bits[v][j] (uint16, j < C / 16), bit i of word j set iff y[v][16 j + i] > 0,
 * k3_relu_bits_bytes reports its size.  k3_conv3d_fwd_bits is k3_conv3d_fwd that also writes
 * relu_bits (dev) for its output; k3_conv3d_bwd_data_bits is k3_conv3d_bwd_data whose mask for
 * the first destination (see dx_mask there) is given as such bits instead of as the bf16 /
 * fp32 tensor: the backward pass then reads 1/16 of the bytes.  Results are identical to the
 * tensor-mask forms. */
int k3_relu_bits_bytes(const k3_tensor *yd, size_t *bytes);
int k3_conv3d_fwd_bits(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2, const void *w,
                       const void *packed, const float *bias, int relu, const k3_tensor *yd, void *y,
                       void *relu_bits, void *stream);
int k3_conv3d_bwd_data_bits(const k3_tensor *dyd, const void *dy, const void *y_mask, const void *w,
                            const void *packed, const k3_tensor *dxd, void *dx, const k3_tensor *dx2d, void *dx2,
                            const void *dx_mask_bits, void *stream);

/* Workspace bytes k3_conv3d_bwd_weight needs for these shapes (split-K partial sums; the
 * larger of the call with and without y_mask). */
int k3_conv3d_bwd_weight_workspace_bytes(const k3_tensor *xd, const k3_tensor *x2d,
                                         const k3_tensor *dyd, size_t *bytes);

/* Backward-weight pass, with g as above and x = [x | x2]:
 *   dW[kd,kh,kw,ci,co] = sum_{n,d,h,w} x[n,d+kd-1,h+kh-1,w+kw-1,ci] * g[n,d,h,w,co]
 *   db[co]            = sum_{n,d,h,w} g[n,d,h,w,co]            (skipped when db is NULL)
 * dW and db are fp32 dev buffers that are overwritten.  The voxel sum is split into
 * slabs whose partial results go to ws (dev) and are then added in a fixed order. */
int k3_conv3d_bwd_weight(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2,
                         const k3_tensor *dyd, const void *dy, const void *y_mask,
                         float *dW, float *db, void *ws, size_t ws_bytes, void *stream);

/* k3_conv3d_bwd_weight for callers that cannot allocate device memory or pass a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the
 * split-K partial sums go to an array of K3_STATIC_SCRATCH_BYTES that is part of the library's
 * device code, one copy per GPU, held until the process ends.  The call allocates nothing and
 * frees nothing.  Same arguments, kernels and results (bit for bit) as k3_conv3d_bwd_weight
 * without ws / ws_bytes; shapes whose partial sums exceed the array return K3_E_WORKSPACE and
 * enqueue nothing (every bf16 shape with channel counts that are multiples of 32 and no y_mask
 * fits, at any volume).  The array keeps the previous call's contents; nothing in it has to
 * start at zero.  All calls on one GPU share it: calls that overlap on one GPU (different
 * streams, or threads) race and must be serialised by the caller.  The device that is current
 * at the call must be the one that owns the tensors and the stream. */
#define K3_STATIC_SCRATCH_BYTES (64u << 20)
int k3_conv3d_bwd_weight_static(const k3_tensor *xd, const void *x, const k3_tensor *x2d, const void *x2,
                                const k3_tensor *dyd, const void *dy, const void *y_mask,
                                float *dW, float *db, void *stream);

/* ------------------------------------------------------------------ 2x2x2 max pooling
 * The 2x2x2 max-pooling layer that follows the encoder convolutions (section 4.1):
 *   y[n,d,h,w,c] = max_{i,j,k in {0,1}} x[n,2d+i,2h+j,2w+k,c].
 * x.d, x.h, x.w must be even (K3_E_SHAPE otherwise). */
int k3_pool3d_fwd(const k3_tensor *xd, const void *x, const k3_tensor *yd, void *y, void *stream);

/* Backward: dx is zero except at the first maximum of each window (order i, j, k),
 * which receives that window's dy.  The arg-max is recomputed from x.  When add is not
 * NULL (same shape as dx) it is added element-wise: dx = route(dy) + add (the skip
 * connection's gradient joining the pooled path).  When relu_mask is non-zero the result
 * is then zeroed where x <= 0: x is a stored ReLU output, and applying its mask here lets
 * that layer's backward passes run without one (see k3_conv3d_bwd_data, dx_mask). */
int k3_pool3d_bwd(const k3_tensor *xd, const void *x, const k3_tensor *dyd, const void *dy,
                  const void *add, int relu_mask, void *dx, void *stream);

/* The same pair with the backward pass's routing kept as one bit per element of x instead of
 * x itself, for a pooling layer whose input is a stored ReLU output that nothing else reads
 * again (the encoder layers of section 4.1's model: the activation can then be dropped, or
 * need not be swapped, once it is pooled).  k3_pool3d_fwd_bits computes y as k3_pool3d_fwd
 * does and writes route_bits (dev; layout and size of k3_relu_bits_bytes(xd)): the bit of
 * x[n,2d+i,2h+j,2w+k,c] is set iff that element is the first maximum of its window (order
 * i, j, k) and > 0.  k3_pool3d_bwd_bits writes dx = the window's dy where the bit is set and
 * zero elsewhere, which is what k3_pool3d_bwd(x, dy, add = NULL, relu_mask = 1) computes.
 * bf16 with c a multiple of 16 only (K3_E_UNSUPPORTED otherwise); shapes as above. */
int k3_pool3d_fwd_bits(const k3_tensor *xd, const void *x, const k3_tensor *yd, void *y,
                       void *route_bits, void *stream);
int k3_pool3d_bwd_bits(const k3_tensor *xd, const void *route_bits, const k3_tensor *dyd,
                       const void *dy, void *dx, void *stream);

/* ------------------------------------------------------------------ 2x2x2 stride-2 transposed convolution
 * The decoder's up-sampling layer (section 4.1) in its learned form:
 *   y[n,2d+i,2h+j,2w+k,co] = bias[co] + sum_ci x[n,d,h,w,ci] * W[i,j,k,ci,co]
 * w is the canonical [2][2][2][C_in][C_out] tensor in the activation dtype (dev).  As for
 * the 3x3x3 convolution, bf16 tensors with channel counts that are multiples of 32 run on
 * MFMA kernels and need a packed copy of the weights (k3_upconv3d_packed_bytes reports 0
 * otherwise, and packed may then be NULL). */
int k3_upconv3d_packed_bytes(int64_t cin, int64_t cout, int dtype, size_t *bytes);
int k3_upconv3d_pack_weights(const void *w, int64_t cin, int64_t cout, int dtype,
                             void *packed, size_t packed_bytes, void *stream);
int k3_upconv3d_fwd(const k3_tensor *xd, const void *x, const void *w, const void *packed,
                    const float *bias, const k3_tensor *yd, void *y, void *stream);
/* dx[n,d,h,w,ci] = sum_{i,j,k,co} dy[n,2d+i,2h+j,2w+k,co] * W[i,j,k,ci,co]; when dx_mask is
 * not NULL (same shape and dtype as dx) dx is zeroed where dx_mask <= 0 (the ReLU mask of
 * the layer that produced the transposed conv's input, applied by the producer). */
int k3_upconv3d_bwd_data(const k3_tensor *dyd, const void *dy, const void *w, const void *packed,
                         const k3_tensor *dxd, void *dx, const void *dx_mask, void *stream);
int k3_upconv3d_bwd_weight_workspace_bytes(const k3_tensor *xd, const k3_tensor *dyd, size_t *bytes);
/* dW[i,j,k,ci,co] = sum_{n,d,h,w} x[n,d,h,w,ci] * dy[n,2d+i,2h+j,2w+k,co]; db[co] = sum dy
 * (db may be NULL).  dW, db: fp32 dev, overwritten; ws: dev workspace for partial sums. */
int k3_upconv3d_bwd_weight(const k3_tensor *xd, const void *x, const k3_tensor *dyd, const void *dy,
                           float *dW, float *db, void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------ 1x1x1 head + softmax cross-entropy
 * The per-voxel likelihood of each of K = 3 classes (section 4.1), forward and
 * backward in one pass over the activations:
 *   z[v,k] = bh[k] + sum_c a[v,c] * Wh[c,k];  p = softmax_k(z);
 *   loss = -(1/V) sum_v log p[v, label_v];    dz = (p - onehot(label)) / V;
 *   da = dz * Wh^T;  dWh = a^T * dz;  dbh = sum_v dz.
 * a: dev, ad->dtype; wh [C][3], bh [3]: fp32 dev; labels: uint8 dev, one per voxel;
 * loss: one fp32 (dev); da: dev, same shape and dtype as a; dWh [C][3], dbh [3]: fp32
 * dev; logits: optional fp32 [V][3] dev (NULL to skip).  When relu_mask is non-zero da is
 * zeroed where a <= 0 (a is a stored ReLU output; see k3_conv3d_bwd_data, dx_mask).  da may
 * be a itself: the gradient then replaces the activations, which nothing reads after this
 * call in a training step (one tensor less at the step's memory peak).  ws holds
 * per-workgroup partial sums. */
int k3_head_workspace_bytes(const k3_tensor *ad, size_t *bytes);
int k3_head_softmax_ce_fwd_bwd(const k3_tensor *ad, const void *a, const float *wh, const float *bh,
                               const uint8_t *labels, float *loss, void *da, int relu_mask,
                               float *dWh, float *dbh, float *logits, void *ws, size_t ws_bytes,
                               void *stream);
/* The same with class-weighted voxels (section 4.1: the weight of voxels is adjusted for the
 * class imbalance of the training set): voxel v counts w_v = class_w[label_v],
 *   loss = -(1/V) sum_v w_v log p[v, label_v];   dz = w_v (p - onehot(label)) / V.
 * The normalisation by the voxel count V (not by the sum of the weights) is a reading: the
 * paper does not give it.  class_w: three fp32 values, dev. */
int k3_head_softmax_wce_fwd_bwd(const k3_tensor *ad, const void *a, const float *wh, const float *bh,
                                const uint8_t *labels, const float *class_w, float *loss, void *da,
                                int relu_mask, float *dWh, float *dbh, float *logits, void *ws,
                                size_t ws_bytes, void *stream);
/* Inference read-out (section 4.1: the classification emitted is the class with the
 * maximum likelihood): classes[v] = argmax_k z[v,k] of the head's logits, lowest k on ties,
 * decided on the fp32 logits the kernel computes; logits: optional fp32 [V][3] (NULL to
 * skip).  a: dev, ad->dtype; wh [C][3], bh [3] (may be NULL): fp32 dev; classes: uint8 dev. */
int k3_head_classify(const k3_tensor *ad, const void *a, const float *wh, const float *bh, uint8_t *classes,
                     float *logits, void *stream);

/* ------------------------------------------------------------------ Dice coefficient
 * The Dice coefficient the paper lists among the figures compared between training runs
 * (section 3.1), per class, between the classified and the labelled voxel sets:
 *   counts[t][p] = number of voxels with label t classified as p  (3 x 3, uint64, row-major);
 *   dice[k] = 2 counts[k][k] / (sum_p counts[k][p] + sum_t counts[t][k]), 1 when that
 *   denominator is 0 (a class neither set contains).
 * classes, labels: uint8 dev, one per voxel, values above 2 count as class 2; counts: dev,
 * 9 uint64, overwritten; dice: dev, 3 fp32, or NULL to get the counts only.  voxels = 0 gives
 * zero counts and dice = 1.  Exact integer counting: the result does not depend on order. */
int k3_dice_coefficients(const uint8_t *classes, const uint8_t *labels, int64_t voxels, uint64_t *counts,
                         float *dice, void *stream);

/* ------------------------------------------------------------------ up-sampling layer
 * The up-sampling layer that follows each decoder convolution of the section-4.1 model,
 * read as nearest-neighbour up-sampling by 2 per axis (the paper does not name the
 * interpolation):  y[n, 2d+i, 2h+j, 2w+k, c] = x[n, d, h, w, c] for i, j, k in {0, 1}.
 * Backward (the adjoint): dx[n,d,h,w,c] = sum_{i,j,k} dy[n, 2d+i, 2h+j, 2w+k, c], summed in
 * fp32 in a fixed order; when x_mask is not NULL it is the stored ReLU output x and dx is
 * zeroed where x <= 0 (see k3_conv3d_bwd_data, dx_mask).  Descriptors: x / dx are
 * (n, d, h, w, c), y / dy are (n, 2d, 2h, 2w, c), same dtype (K3_E_SHAPE otherwise).
 * All pointers dev; x_mask has the shape of dx. */
int k3_upsample3d_fwd(const k3_tensor *xd, const void *x, const k3_tensor *yd, void *y, void *stream);
int k3_upsample3d_bwd(const k3_tensor *dyd, const void *dy, const void *x_mask, const k3_tensor *dxd, void *dx,
                      void *stream);

/* ------------------------------------------------------------------ weight update
 * Stochastic gradient descent, the weight-update algorithm the paper's training runs on
 * the GPU (section 1), with the usual momentum and weight-decay terms (both may be 0,
 * which gives plain SGD), on a flat vector of n fp32 parameters:
 *   v <- momentum * v + (g + weight_decay * w);   w <- w - lr * v.
 * w (master weights), v (momentum buffer) are updated in place; g is read only.  When
 * w_bf16 is not NULL it receives the updated weights rounded to bf16 (round to nearest
 * even), the working copy the bf16 kernels read.  All pointers dev; n = 0 is a no-op.
 * Any alignment is accepted (16-byte aligned vectors take the wide path).  NaN
 * hyper-parameters return K3_E_BADARG. */
int k3_sgd_momentum_step(int64_t n, float *w, float *v, const float *g, float lr, float momentum,
                         float weight_decay, void *w_bf16, void *stream);

/* ------------------------------------------------------------------ measurement aids
 * The machine rates the benchmark quotes its kernels against, measured on the box it runs on
 * (not part of the training path; the caller times them with events on `stream`).
 * k3_probe_mfma_bf16: `blocks` workgroups of 4 waves each run `iters` rounds of four independent
 * register-resident bf16 32x32x16 MFMAs; *flops (host, may be NULL) receives the FLOPs of the
 * launch; sink (dev, blocks * 256 floats) receives one value per lane so the loop is kept.
 * k3_probe_copy: grid-stride device copy of `bytes` (a multiple of 16; src, dst dev, 16-byte
 * aligned, not overlapping) by `blocks` workgroups of 256 lanes, 16 bytes per lane and round. */
int k3_probe_mfma_bf16(int64_t iters, int blocks, float *sink, double *flops, void *stream);
int k3_probe_copy(const void *src, void *dst, size_t bytes, int blocks, void *stream);

/* ------------------------------------------------------------------ LMS swap engine
 * Tensor swapping between device and host memory so that only the tensors a training
 * step currently needs stay on the GPU (section 2.2): a finished forward activation
 * is copied to page-locked host memory on a dedicated copy stream and its device block
 * can be reused; before its backward consumer runs it is copied back.
 *
 * A handle walks RESIDENT -> OUT_IN_FLIGHT -> ON_HOST -> IN_IN_FLIGHT -> RESIDENT; calls
 * that do not fit the current state return K3_E_STATE.  The context owns two copy
 * streams (device-to-host, host-to-device) and its events.  Host buffers are owned by
 * the caller, must be page-locked (K3_E_NOT_PINNED otherwise) and must stay valid
 * until the handle is released.  Calls on one context must come from one thread. */
typedef struct k3_lms k3_lms;

/* device_budget_bytes: cap on the bytes of device blocks accounted through
 * k3_lms_account_alloc / _free (0 = unlimited). */
int k3_lms_create(uint64_t device_budget_bytes, k3_lms **ctx);
int k3_lms_destroy(k3_lms *ctx);

/* Page-locked host memory helpers (hipHostMalloc / hipHostFree). */
int k3_lms_host_alloc(size_t bytes, void **host_ptr);
int k3_lms_host_free(void *host_ptr);

/* Device-budget accounting for blocks the caller allocates: _alloc fails with
 * K3_E_OOM (and accounts nothing) when the budget would be exceeded. */
int k3_lms_account_alloc(k3_lms *ctx, uint64_t bytes);
int k3_lms_account_free(k3_lms *ctx, uint64_t bytes);

/* Starts the device-to-host copy of bytes at dev_ptr into host_ptr.  The copy waits
 * for everything enqueued so far on compute_stream (the producers and forward readers
 * of the tensor).  Returns a new handle in OUT_IN_FLIGHT. */
int k3_lms_swap_out(k3_lms *ctx, const void *dev_ptr, size_t bytes, void *host_ptr,
                    void *compute_stream, int *handle);
/* 1 in *done once the swap-out copy has finished (handle moves to ON_HOST), else 0; also
 * after k3_lms_release_after it reports the copy itself, not the hand-over of the block. */
int k3_lms_swap_out_done(k3_lms *ctx, int handle, int *done);
/* Makes `stream` wait for the swap-out copy, so that work enqueued on it afterwards
 * may overwrite or free the device block.  The handle stays OUT_IN_FLIGHT until the copy
 * has finished (then ON_HOST); a prefetch may be started at once (it waits for the copy). */
int k3_lms_release_after(k3_lms *ctx, int handle, void *stream);
/* Starts the host-to-device copy of the tensor into dev_ptr (a block of at least the
 * swapped size).  The copy waits for work already enqueued on consumer_stream (earlier
 * users of that block), and consumer_stream is made to wait for the copy, so kernels
 * enqueued on it afterwards see the data.  Handle: ON_HOST -> IN_IN_FLIGHT. */
int k3_lms_prefetch_in(k3_lms *ctx, int handle, void *dev_ptr, void *consumer_stream);
/* As k3_lms_prefetch_in, but no stream is made to wait: the copy starts once the work
 * already enqueued on block_stream (earlier users of the block) has run, and overlaps
 * whatever is enqueued afterwards.  Every stream that reads the tensor must be given
 * k3_lms_wait_in before its first reader is enqueued. */
int k3_lms_prefetch_start(k3_lms *ctx, int handle, void *dev_ptr, void *block_stream);
/* Makes `stream` wait for the prefetch copy of `handle` (for consumers on other streams,
 * and after k3_lms_prefetch_start). */
int k3_lms_wait_in(k3_lms *ctx, int handle, void *stream);
/* Drops the device copy of a tensor that was brought back and only read since: the host
 * copy of the earlier swap-out is still its value, so nothing is copied.  `stream` is
 * made to wait for the copy-in first (a no-op once it finished), so that work enqueued
 * on it afterwards may reuse the block.  IN_IN_FLIGHT / RESIDENT -> ON_HOST. */
int k3_lms_evict(k3_lms *ctx, int handle, void *stream);
/* Drops the handle; a copy still in flight (in either direction, also after
 * k3_lms_release_after) is waited for first, so the host buffer may be reused or freed
 * once this returns. */
int k3_lms_release(k3_lms *ctx, int handle);
/* Blocks the host until both copy streams are idle. */
int k3_lms_sync(k3_lms *ctx);

typedef struct k3_lms_stats {
    uint64_t bytes_out, bytes_in;           /* bytes copied in each direction */
    uint64_t n_out, n_in;                   /* copies started */
    uint64_t device_bytes, device_peak;     /* accounted device bytes now / high-water mark */
    uint64_t live_handles;
} k3_lms_stats;
int k3_lms_get_stats(k3_lms *ctx, k3_lms_stats *out);
/* Measurement aid: with timing on (off by default) every copy is bracketed by a pair of timed
 * events on its copy stream.  k3_lms_copy_busy_ms returns the accumulated time, in
 * milliseconds since the context was created, that the device-to-host and the host-to-device
 * copy stream spent copying (copies of one direction run one after the other, so the sum of
 * their durations is that stream's busy time); copies still in flight are not counted yet. */
int k3_lms_set_copy_timing(k3_lms *ctx, int on);
/* Debug switch (off by default): every device block whose tensor has gone to the host
 * (k3_lms_release_after, k3_lms_evict) is overwritten with 0xFF bytes -- NaN in bf16 and
 * fp32 -- on the stream that was just ordered behind the copy, so that a kernel which still
 * reads the block after the swap shows up in the results.  Blocks already handed over when
 * the switch is turned on are not touched. */
int k3_lms_set_poison(k3_lms *ctx, int on);
int k3_lms_copy_busy_ms(k3_lms *ctx, double *out_ms, double *in_ms);
int k3_lms_handle_state(k3_lms *ctx, int handle, int *state);

enum { K3_LMS_RESIDENT = 0, K3_LMS_OUT_IN_FLIGHT = 1, K3_LMS_ON_HOST = 2, K3_LMS_IN_IN_FLIGHT = 3 };

#ifdef __cplusplus
}
#endif
#endif /* K3_H */
