/*
 * CPU oracle for the 3-D U-Net training-step operators.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call into this file; it exists so that the GPU
 * kernels can be compared, element by element, with the plain definitions.
 *
 * The paper (sections 3 and 4.1) names the operators only: 3x3x3 convolution
 * layers, 2x2x2 max-pooling layers, an up-sampling ("inverse") decoder layer and a
 * per-voxel three-class likelihood.  Each function below is the textbook definition
 * of that operator, or of its exact gradient, evaluated by direct loops in double
 * precision: no tiling, no reordering beyond a natural loop nest, no fast paths.
 * OpenMP is applied to the outermost (n, d, h) loops only.
 *
 * Conventions: activations are NDHWC (channel fastest), 3x3x3 weights are
 * [kd][kh][kw][C_in][C_out], transposed-conv weights [i][j][k][C_in][C_out], head
 * weights [C][K].  Convolution means cross-correlation with zero padding 1 and
 * stride 1 ("same" size).  All sizes are 64-bit.
 *
 * Every function here is pinned by tests that do not go through this file's own
 * arithmetic: closed forms, shift kernels, adjoint/bilinear identities, finite
 * differences, an independently structured numpy evaluation, and PyTorch's CPU
 * operators as a library special case.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef int64_t i64;

#define IDX5(n, d, h, w, c, D, H, W, C) (((((i64)(n) * (D) + (d)) * (H) + (h)) * (W) + (w)) * (C) + (c))

/* y[n,d,h,w,co] = act(b[co] + sum_{kd,kh,kw,ci} x[n,d+kd-1,h+kh-1,w+kw-1,ci] * W[kd,kh,kw,ci,co]),
 * out-of-range x reads as zero; act is ReLU when relu != 0, identity otherwise.
 * (3x3x3 convolutional layer, paper section 4.1.) */
void orc_conv3d_fwd(const double *x, const double *wt, const double *b, double *y,
                    i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co, int relu)
{
    i64 ndh = N * D * H;
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < ndh; ++r) {
        i64 n = r / (D * H), d = (r / H) % D, h = r % H;
        for (i64 w = 0; w < W; ++w)
            for (i64 co = 0; co < Co; ++co) {
                double acc = b ? b[co] : 0.0;
                for (int kd = 0; kd < 3; ++kd)
                    for (int kh = 0; kh < 3; ++kh)
                        for (int kw = 0; kw < 3; ++kw) {
                            i64 dd = d + kd - 1, hh = h + kh - 1, ww = w + kw - 1;
                            if (dd < 0 || dd >= D || hh < 0 || hh >= H || ww < 0 || ww >= W) continue;
                            const double *xp = x + IDX5(n, dd, hh, ww, 0, D, H, W, Ci);
                            const double *wp = wt + (((i64)(kd * 3 + kh) * 3 + kw) * Ci) * Co + co;
                            for (i64 ci = 0; ci < Ci; ++ci) acc += xp[ci] * wp[ci * Co];
                        }
                if (relu && !(acc > 0.0)) acc = 0.0;
                y[IDX5(n, d, h, w, co, D, H, W, Co)] = acc;
            }
    }
}

/* Same sum as orc_conv3d_fwd but only at the listed voxels: pts holds npts rows of
 * (n, d, h, w); out is [npts][Co].  Used to sample very large tensors. */
void orc_conv3d_fwd_points(const double *x, const double *wt, const double *b, double *out,
                           const i64 *pts, i64 npts,
                           i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co, int relu)
{
    (void)N;
#pragma omp parallel for schedule(static)
    for (i64 p = 0; p < npts; ++p) {
        i64 n = pts[4 * p], d = pts[4 * p + 1], h = pts[4 * p + 2], w = pts[4 * p + 3];
        for (i64 co = 0; co < Co; ++co) {
            double acc = b ? b[co] : 0.0;
            for (int kd = 0; kd < 3; ++kd)
                for (int kh = 0; kh < 3; ++kh)
                    for (int kw = 0; kw < 3; ++kw) {
                        i64 dd = d + kd - 1, hh = h + kh - 1, ww = w + kw - 1;
                        if (dd < 0 || dd >= D || hh < 0 || hh >= H || ww < 0 || ww >= W) continue;
                        const double *xp = x + IDX5(n, dd, hh, ww, 0, D, H, W, Ci);
                        const double *wp = wt + (((i64)(kd * 3 + kh) * 3 + kw) * Ci) * Co + co;
                        for (i64 ci = 0; ci < Ci; ++ci) acc += xp[ci] * wp[ci * Co];
                    }
            if (relu && !(acc > 0.0)) acc = 0.0;
            out[p * Co + co] = acc;
        }
    }
}

/* g = dy where y > 0, else 0 (gradient of ReLU read off the stored output). */
void orc_relu_bwd(const double *dy, const double *y, double *g, i64 count)
{
#pragma omp parallel for schedule(static)
    for (i64 i = 0; i < count; ++i) g[i] = (y[i] > 0.0) ? dy[i] : 0.0;
}

/* dx[n,d,h,w,ci] = sum_{kd,kh,kw,co} g[n,d-kd+1,h-kh+1,w-kw+1,co] * W[kd,kh,kw,ci,co]
 * (g = 0 out of range): the exact gradient of the forward sum with respect to x. */
void orc_conv3d_bwd_data(const double *g, const double *wt, double *dx,
                         i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
    i64 ndh = N * D * H;
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < ndh; ++r) {
        i64 n = r / (D * H), d = (r / H) % D, h = r % H;
        for (i64 w = 0; w < W; ++w)
            for (i64 ci = 0; ci < Ci; ++ci) {
                double acc = 0.0;
                for (int kd = 0; kd < 3; ++kd)
                    for (int kh = 0; kh < 3; ++kh)
                        for (int kw = 0; kw < 3; ++kw) {
                            i64 dd = d - kd + 1, hh = h - kh + 1, ww = w - kw + 1;
                            if (dd < 0 || dd >= D || hh < 0 || hh >= H || ww < 0 || ww >= W) continue;
                            const double *gp = g + IDX5(n, dd, hh, ww, 0, D, H, W, Co);
                            const double *wp = wt + (((i64)(kd * 3 + kh) * 3 + kw) * Ci + ci) * Co;
                            for (i64 co = 0; co < Co; ++co) acc += gp[co] * wp[co];
                        }
                dx[IDX5(n, d, h, w, ci, D, H, W, Ci)] = acc;
            }
    }
}

/* Same sum as orc_conv3d_bwd_data but only at the listed voxels: pts holds npts rows of
 * (n, d, h, w); out is [npts][Ci].  Used to sample very large tensors. */
void orc_conv3d_bwd_data_points(const double *g, const double *wt, double *out, const i64 *pts, i64 npts,
                                i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
    (void)N;
#pragma omp parallel for schedule(static)
    for (i64 p = 0; p < npts; ++p) {
        i64 n = pts[4 * p], d = pts[4 * p + 1], h = pts[4 * p + 2], w = pts[4 * p + 3];
        for (i64 ci = 0; ci < Ci; ++ci) {
            double acc = 0.0;
            for (int kd = 0; kd < 3; ++kd)
                for (int kh = 0; kh < 3; ++kh)
                    for (int kw = 0; kw < 3; ++kw) {
                        i64 dd = d - kd + 1, hh = h - kh + 1, ww = w - kw + 1;
                        if (dd < 0 || dd >= D || hh < 0 || hh >= H || ww < 0 || ww >= W) continue;
                        const double *gp = g + IDX5(n, dd, hh, ww, 0, D, H, W, Co);
                        const double *wp = wt + (((i64)(kd * 3 + kh) * 3 + kw) * Ci + ci) * Co;
                        for (i64 co = 0; co < Co; ++co) acc += gp[co] * wp[co];
                    }
            out[p * Ci + ci] = acc;
        }
    }
}

/* dW[kd,kh,kw,ci,co] = sum_{n,d,h,w} x[n,d+kd-1,h+kh-1,w+kw-1,ci] * g[n,d,h,w,co];
 * db[co] = sum_{n,d,h,w} g[n,d,h,w,co].  Parallel over the 27*Ci output rows so the
 * voxel sum of each entry is accumulated by one thread in a fixed order. */
void orc_conv3d_bwd_weight(const double *x, const double *g, double *dW, double *db,
                           i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
    i64 rows = 27 * Ci;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 r = 0; r < rows; ++r) {
        int t = (int)(r / Ci);
        i64 ci = r % Ci;
        int kd = t / 9, kh = (t / 3) % 3, kw = t % 3;
        double *acc = dW + r * Co;
        for (i64 co = 0; co < Co; ++co) acc[co] = 0.0;
        for (i64 n = 0; n < N; ++n)
            for (i64 d = 0; d < D; ++d) {
                i64 dd = d + kd - 1;
                if (dd < 0 || dd >= D) continue;
                for (i64 h = 0; h < H; ++h) {
                    i64 hh = h + kh - 1;
                    if (hh < 0 || hh >= H) continue;
                    for (i64 w = 0; w < W; ++w) {
                        i64 ww = w + kw - 1;
                        if (ww < 0 || ww >= W) continue;
                        double xv = x[IDX5(n, dd, hh, ww, ci, D, H, W, Ci)];
                        const double *gp = g + IDX5(n, d, h, w, 0, D, H, W, Co);
                        for (i64 co = 0; co < Co; ++co) acc[co] += xv * gp[co];
                    }
                }
            }
    }
    if (db) {
        for (i64 co = 0; co < Co; ++co) db[co] = 0.0;
        i64 V = N * D * H * W;
        for (i64 v = 0; v < V; ++v)
            for (i64 co = 0; co < Co; ++co) db[co] += g[v * Co + co];
    }
}

/* The same voxel sum for a list of single entries: ent holds nent rows of
 * (tap, ci, co) with tap = (kd*3+kh)*3+kw; out is [nent]. */
void orc_conv3d_bwd_weight_entries(const double *x, const double *g, double *out,
                                   const i64 *ent, i64 nent,
                                   i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 e = 0; e < nent; ++e) {
        int t = (int)ent[3 * e];
        i64 ci = ent[3 * e + 1], co = ent[3 * e + 2];
        int kd = t / 9, kh = (t / 3) % 3, kw = t % 3;
        double acc = 0.0;
        for (i64 n = 0; n < N; ++n)
            for (i64 d = 0; d < D; ++d)
                for (i64 h = 0; h < H; ++h)
                    for (i64 w = 0; w < W; ++w) {
                        i64 dd = d + kd - 1, hh = h + kh - 1, ww = w + kw - 1;
                        if (dd < 0 || dd >= D || hh < 0 || hh >= H || ww < 0 || ww >= W) continue;
                        acc += x[IDX5(n, dd, hh, ww, ci, D, H, W, Ci)] * g[IDX5(n, d, h, w, co, D, H, W, Co)];
                    }
        out[e] = acc;
    }
}

/* y[n,d,h,w,c] = max over the 2x2x2 window x[n,2d+i,2h+j,2w+k,c] (2x2x2 max pooling,
 * paper section 4.1).  D, H, W are the INPUT sizes and must be even. */
void orc_pool3d_fwd(const double *x, double *y, i64 N, i64 D, i64 H, i64 W, i64 C)
{
    i64 Do = D / 2, Ho = H / 2, Wo = W / 2, ndh = N * Do * Ho;
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < ndh; ++r) {
        i64 n = r / (Do * Ho), d = (r / Ho) % Do, h = r % Ho;
        for (i64 w = 0; w < Wo; ++w)
            for (i64 c = 0; c < C; ++c) {
                double m = x[IDX5(n, 2 * d, 2 * h, 2 * w, c, D, H, W, C)];
                for (int i = 0; i < 2; ++i)
                    for (int j = 0; j < 2; ++j)
                        for (int k = 0; k < 2; ++k) {
                            double v = x[IDX5(n, 2 * d + i, 2 * h + j, 2 * w + k, c, D, H, W, C)];
                            if (v > m) m = v;
                        }
                y[IDX5(n, d, h, w, c, Do, Ho, Wo, C)] = m;
            }
    }
}

/* dx is zero except at the first maximum (lexicographic (i,j,k) order) of each window,
 * which receives dy of that window. */
void orc_pool3d_bwd(const double *x, const double *dy, double *dx, i64 N, i64 D, i64 H, i64 W, i64 C)
{
    i64 Do = D / 2, Ho = H / 2, Wo = W / 2, ndh = N * Do * Ho;
    memset(dx, 0, sizeof(double) * (size_t)(N * D * H * W * C));
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < ndh; ++r) {
        i64 n = r / (Do * Ho), d = (r / Ho) % Do, h = r % Ho;
        for (i64 w = 0; w < Wo; ++w)
            for (i64 c = 0; c < C; ++c) {
                int bi = 0, bj = 0, bk = 0;
                double m = x[IDX5(n, 2 * d, 2 * h, 2 * w, c, D, H, W, C)];
                for (int i = 0; i < 2; ++i)
                    for (int j = 0; j < 2; ++j)
                        for (int k = 0; k < 2; ++k) {
                            double v = x[IDX5(n, 2 * d + i, 2 * h + j, 2 * w + k, c, D, H, W, C)];
                            if (v > m) { m = v; bi = i; bj = j; bk = k; }
                        }
                dx[IDX5(n, 2 * d + bi, 2 * h + bj, 2 * w + bk, c, D, H, W, C)] = dy[IDX5(n, d, h, w, c, Do, Ho, Wo, C)];
            }
    }
}

/* 2x2x2 stride-2 transposed convolution (the decoder's up-sampling layer, paper
 * section 4.1, in the learned form the workload fixes):
 * y[n,2d+i,2h+j,2w+k,co] = b[co] + sum_ci x[n,d,h,w,ci] * W[i,j,k,ci,co].
 * D, H, W are the INPUT sizes. */
void orc_upconv3d_fwd(const double *x, const double *wt, const double *b, double *y,
                      i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
    i64 ndh = N * D * H;
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < ndh; ++r) {
        i64 n = r / (D * H), d = (r / H) % D, h = r % H;
        for (i64 w = 0; w < W; ++w)
            for (int i = 0; i < 2; ++i)
                for (int j = 0; j < 2; ++j)
                    for (int k = 0; k < 2; ++k)
                        for (i64 co = 0; co < Co; ++co) {
                            double acc = b ? b[co] : 0.0;
                            const double *xp = x + IDX5(n, d, h, w, 0, D, H, W, Ci);
                            const double *wp = wt + ((i64)((i * 2 + j) * 2 + k) * Ci) * Co + co;
                            for (i64 ci = 0; ci < Ci; ++ci) acc += xp[ci] * wp[ci * Co];
                            y[IDX5(n, 2 * d + i, 2 * h + j, 2 * w + k, co, 2 * D, 2 * H, 2 * W, Co)] = acc;
                        }
    }
}

/* dx[n,d,h,w,ci] = sum_{i,j,k,co} dy[n,2d+i,2h+j,2w+k,co] * W[i,j,k,ci,co]. */
void orc_upconv3d_bwd_data(const double *dy, const double *wt, double *dx,
                           i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
    i64 ndh = N * D * H;
#pragma omp parallel for schedule(static)
    for (i64 r = 0; r < ndh; ++r) {
        i64 n = r / (D * H), d = (r / H) % D, h = r % H;
        for (i64 w = 0; w < W; ++w)
            for (i64 ci = 0; ci < Ci; ++ci) {
                double acc = 0.0;
                for (int i = 0; i < 2; ++i)
                    for (int j = 0; j < 2; ++j)
                        for (int k = 0; k < 2; ++k) {
                            const double *gp = dy + IDX5(n, 2 * d + i, 2 * h + j, 2 * w + k, 0, 2 * D, 2 * H, 2 * W, Co);
                            const double *wp = wt + ((i64)((i * 2 + j) * 2 + k) * Ci + ci) * Co;
                            for (i64 co = 0; co < Co; ++co) acc += gp[co] * wp[co];
                        }
                dx[IDX5(n, d, h, w, ci, D, H, W, Ci)] = acc;
            }
    }
}

/* dW[i,j,k,ci,co] = sum_{n,d,h,w} x[n,d,h,w,ci] * dy[n,2d+i,2h+j,2w+k,co]; db[co] = sum dy. */
void orc_upconv3d_bwd_weight(const double *x, const double *dy, double *dW, double *db,
                             i64 N, i64 D, i64 H, i64 W, i64 Ci, i64 Co)
{
    i64 rows = 8 * Ci;
#pragma omp parallel for schedule(dynamic, 1)
    for (i64 r = 0; r < rows; ++r) {
        int t = (int)(r / Ci);
        i64 ci = r % Ci;
        int i = t / 4, j = (t / 2) % 2, k = t % 2;
        double *acc = dW + r * Co;
        for (i64 co = 0; co < Co; ++co) acc[co] = 0.0;
        for (i64 n = 0; n < N; ++n)
            for (i64 d = 0; d < D; ++d)
                for (i64 h = 0; h < H; ++h)
                    for (i64 w = 0; w < W; ++w) {
                        double xv = x[IDX5(n, d, h, w, ci, D, H, W, Ci)];
                        const double *gp = dy + IDX5(n, 2 * d + i, 2 * h + j, 2 * w + k, 0, 2 * D, 2 * H, 2 * W, Co);
                        for (i64 co = 0; co < Co; ++co) acc[co] += xv * gp[co];
                    }
    }
    if (db) {
        for (i64 co = 0; co < Co; ++co) db[co] = 0.0;
        i64 V = N * D * H * W * 8;
        for (i64 v = 0; v < V; ++v)
            for (i64 co = 0; co < Co; ++co) db[co] += dy[v * Co + co];
    }
}

/* Per-voxel class likelihoods and their training loss (paper section 4.1: a
 * likelihood for each of three classes; the workload fixes softmax + mean cross-entropy):
 *   z[v,k] = b[k] + sum_c a[v,c] * Wh[c,k];  p = softmax_k(z) (max-subtracted);
 *   loss = -(1/V) sum_v log p[v,label_v];  dz = (p - onehot(label)) / V;
 *   da = dz * Wh^T;  dWh = a^T * dz;  dbh = sum_v dz.
 * Any of logits, da, dWh, dbh may be NULL. */
void orc_head_softmax_ce(const double *a, const double *wh, const double *bh, const uint8_t *labels,
                         double *loss, double *logits, double *da, double *dWh, double *dbh,
                         i64 V, i64 C, i64 K)
{
    double total = 0.0;
    double *z = (double *)malloc(sizeof(double) * (size_t)K);
    double *dz = (double *)malloc(sizeof(double) * (size_t)K);
    if (dWh) for (i64 i = 0; i < C * K; ++i) dWh[i] = 0.0;
    if (dbh) for (i64 k = 0; k < K; ++k) dbh[k] = 0.0;
    for (i64 v = 0; v < V; ++v) {
        const double *av = a + v * C;
        double zmax = -INFINITY;
        for (i64 k = 0; k < K; ++k) {
            double s = bh ? bh[k] : 0.0;
            for (i64 c = 0; c < C; ++c) s += av[c] * wh[c * K + k];
            z[k] = s;
            if (s > zmax) zmax = s;
            if (logits) logits[v * K + k] = s;
        }
        double den = 0.0;
        for (i64 k = 0; k < K; ++k) den += exp(z[k] - zmax);
        double logden = log(den);
        int lab = labels[v];
        total += -(z[lab] - zmax - logden);
        for (i64 k = 0; k < K; ++k) {
            double p = exp(z[k] - zmax - logden);
            dz[k] = (p - (k == lab ? 1.0 : 0.0)) / (double)V;
        }
        if (da)
            for (i64 c = 0; c < C; ++c) {
                double s = 0.0;
                for (i64 k = 0; k < K; ++k) s += dz[k] * wh[c * K + k];
                da[v * C + c] = s;
            }
        if (dWh)
            for (i64 c = 0; c < C; ++c)
                for (i64 k = 0; k < K; ++k) dWh[c * K + k] += av[c] * dz[k];
        if (dbh)
            for (i64 k = 0; k < K; ++k) dbh[k] += dz[k];
    }
    *loss = total / (double)V;
    free(z);
    free(dz);
}
