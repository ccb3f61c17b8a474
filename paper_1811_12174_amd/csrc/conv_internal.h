// Internal argument bundle and launcher declarations shared by the conv3d sources.
#pragma once
#include "common.h"

namespace k3 {

struct ConvArgs {
    int dtype = 0;
    int64_t N = 0, D = 0, H = 0, W = 0;
    int64_t c1 = 0, c2 = 0;   // input channels of the first / second source (or destination)
    int64_t cout = 0;
    // forward / weight gradient inputs
    const void *x = nullptr, *x2 = nullptr;
    // canonical and packed weights
    const void *w = nullptr, *packed = nullptr;
    const float *bias = nullptr;
    int relu = 0;
    void *y = nullptr;
    // backward inputs / outputs
    const void *dy = nullptr, *ymask = nullptr;
    void *dx = nullptr, *dx2 = nullptr;
    const void *omask = nullptr;   // optional mask applied to dx (first destination) by the producer
    const void *omask_bits = nullptr;   // the same mask as one bit per element (alternative to omask)
    void *ybits = nullptr;              // optional: bit mask of the forward output (set where y > 0)
    void *ypool = nullptr;              // optional: 2x2x2 max-pool of the forward output (the kernel may write it itself)
    int64_t V() const { return N * D * H * W; }
};

// true when the bf16 MFMA implicit-GEMM kernels cover this channel configuration
static inline bool mfma_ok(int dtype, int64_t c1, int64_t c2, int64_t cout)
{
    return dtype == K3_BF16 && c1 % 32 == 0 && c2 % 32 == 0 && cout % 32 == 0;
}

int conv_fwd_direct(const ConvArgs &a, hipStream_t st);
int conv_dgrad_direct(const ConvArgs &a, hipStream_t st);
int conv_wgrad_direct(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st);
size_t conv_wgrad_direct_ws_bytes(int64_t V, int64_t cin, int64_t cout);

size_t conv_packed_bytes(int64_t cin, int64_t cout);
int conv_pack_weights(const void *w, int64_t cin, int64_t cout, void *packed, hipStream_t st);
// *pooled (when not null) reports whether the kernel wrote a.ypool itself
int conv_fwd_mfma(const ConvArgs &a, hipStream_t st, bool *pooled = nullptr);
int conv_dgrad_mfma(const ConvArgs &a, hipStream_t st);
int conv_wgrad_mfma(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st);
size_t conv_wgrad_mfma_ws_bytes(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout);
size_t conv_wgrad_mfma_ws_bytes_for(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout, bool masked);

bool conv_wgrad_pipe_ok(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout);
size_t conv_wgrad_pipe_ws_bytes(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cin, int64_t cout);
int conv_wgrad_pipe(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st);

bool conv_first_ok(int dtype, int64_t c1, int64_t c2, int64_t cout);
int conv_first_fwd(const ConvArgs &a, hipStream_t st);
int conv_first_wgrad(const ConvArgs &a, float *dW, float *db, float *ws, hipStream_t st);
size_t conv_first_wgrad_ws_bytes(int64_t N, int64_t D, int64_t H, int64_t W, int64_t cout);

// one uint16 word per 16 consecutive channels: bit i set iff element 16 * word + i is > 0
int launch_relu_bits(int dtype, const void *y, void *bits, int64_t nwords, hipStream_t st);
// zeroes the elements of t whose bit is clear
int launch_apply_relu_bits(int dtype, void *t, const void *bits, int64_t nwords, hipStream_t st);

int launch_reduce_partials(const float *ws, float *dW, float *db, int64_t countW, int64_t count, int nsplit,
                           hipStream_t st);

}  // namespace k3
