// HIP backend of the swap engine and the k3_lms_* C-ABI entry points.  Copies run on two
// dedicated non-blocking streams at the default priority (one per direction, so both DMA
// directions can be busy at once) and are fenced with timing-disabled events.
#include <new>
#include <vector>

#include "common.h"
#include "lms_engine.h"

namespace {

// debug aid of the swap engine: a block whose tensor has gone to the host is overwritten
__global__ __launch_bounds__(256) void lms_poison_kernel(unsigned char *p, size_t bytes)
{
    const size_t stride = (size_t)gridDim.x * 256 * 16;
    for (size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 16; i < bytes; i += stride) {
        if (i + 16 <= bytes && (((uintptr_t)p + i) & 15) == 0) {
            *reinterpret_cast<uint4 *>(p + i) = make_uint4(0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu);
        } else {
            for (size_t j = i; j < bytes && j < i + 16; ++j) p[j] = 0xff;
        }
    }
}

struct HipBackend : k3lms::Backend {
    int last = 0;
    // optional timing of the copies (off by default): a timed event pair around every copy; the
    // copies of a direction run one after the other on one stream, so the sum of the pairs is the
    // time that direction's copy engine was busy
    struct Timed { hipEvent_t t0, t1; int dir; };
    bool timing = false;
    std::vector<Timed> pending;
    std::vector<hipEvent_t> spare;
    double busy_ms[2] = {0.0, 0.0};
    hipEvent_t timed_event()
    {
        if (!spare.empty()) { hipEvent_t e = spare.back(); spare.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
        return e;
    }
    void collect()   // adds the pairs whose copy has finished
    {
        size_t keep = 0;
        for (size_t i = 0; i < pending.size(); ++i) {
            Timed &t = pending[i];
            float ms = 0.f;
            hipError_t r = hipEventElapsedTime(&ms, t.t0, t.t1);
            if (r == hipSuccess) {
                busy_ms[t.dir] += ms;
                spare.push_back(t.t0);
                spare.push_back(t.t1);
            } else {
                (void)hipGetLastError();   // not ready yet
                pending[keep++] = t;
            }
        }
        pending.resize(keep);
    }
    int timed_copy(void *dst, const void *src, size_t bytes, hipMemcpyKind kind, hipStream_t st, int dir)
    {
        if (!timing) return chk(hipMemcpyAsync(dst, src, bytes, kind, st));
        hipEvent_t t0 = timed_event(), t1 = timed_event();
        if (!t0 || !t1) return chk(hipMemcpyAsync(dst, src, bytes, kind, st));
        if (chk(hipEventRecord(t0, st))) return 1;
        if (chk(hipMemcpyAsync(dst, src, bytes, kind, st))) return 1;
        if (chk(hipEventRecord(t1, st))) return 1;
        pending.push_back(Timed{t0, t1, dir});
        if (pending.size() > 256) collect();
        return 0;
    }
    ~HipBackend()
    {
        for (Timed &t : pending) { (void)hipEventDestroy(t.t0); (void)hipEventDestroy(t.t1); }
        for (hipEvent_t e : spare) (void)hipEventDestroy(e);
    }
    int chk(hipError_t e)
    {
        if (e != hipSuccess) {
            last = (int)e;
            k3::set_hip_error(e);
            return 1;
        }
        return 0;
    }
    int stream_create(k3lms::stream_t *s) override
    {
        hipStream_t st;
        if (chk(hipStreamCreateWithFlags(&st, hipStreamNonBlocking))) return 1;
        *s = st;
        return 0;
    }
    int stream_destroy(k3lms::stream_t s) override { return chk(hipStreamDestroy((hipStream_t)s)); }
    int stream_sync(k3lms::stream_t s) override { return chk(hipStreamSynchronize((hipStream_t)s)); }
    int event_create(k3lms::event_t *e) override
    {
        hipEvent_t ev;
        if (chk(hipEventCreateWithFlags(&ev, hipEventDisableTiming))) return 1;
        *e = ev;
        return 0;
    }
    int event_destroy(k3lms::event_t e) override { return chk(hipEventDestroy((hipEvent_t)e)); }
    int event_record(k3lms::event_t e, k3lms::stream_t s) override { return chk(hipEventRecord((hipEvent_t)e, (hipStream_t)s)); }
    int stream_wait_event(k3lms::stream_t s, k3lms::event_t e) override
    {
        return chk(hipStreamWaitEvent((hipStream_t)s, (hipEvent_t)e, 0));
    }
    int event_query(k3lms::event_t e, bool *done) override
    {
        hipError_t r = hipEventQuery((hipEvent_t)e);
        if (r == hipSuccess) { *done = true; return 0; }
        if (r == hipErrorNotReady) { *done = false; (void)hipGetLastError(); return 0; }
        return chk(r);
    }
    int event_sync(k3lms::event_t e) override { return chk(hipEventSynchronize((hipEvent_t)e)); }
    int copy_d2h(void *host, const void *dev, size_t bytes, k3lms::stream_t s) override
    {
        return timed_copy(host, dev, bytes, hipMemcpyDeviceToHost, (hipStream_t)s, 0);
    }
    int copy_h2d(void *dev, const void *host, size_t bytes, k3lms::stream_t s) override
    {
        return timed_copy(dev, const_cast<void *>(host), bytes, hipMemcpyHostToDevice, (hipStream_t)s, 1);
    }
    int fill_poison(void *dev, size_t bytes, k3lms::stream_t s) override
    {
        if (bytes == 0) return 0;
        size_t blocks = (bytes + 4095) / 4096;
        if (blocks > 8192) blocks = 8192;
        lms_poison_kernel<<<dim3((unsigned)blocks), 256, 0, (hipStream_t)s>>>((unsigned char *)dev, bytes);
        return chk(hipGetLastError());
    }
    bool is_pinned(const void *host, size_t bytes) override
    {
        hipPointerAttribute_t at;
        hipError_t r = hipPointerGetAttributes(&at, host);
        if (r != hipSuccess) { (void)hipGetLastError(); return false; }
        if (at.type != hipMemoryTypeHost) return false;
        // the last byte must belong to a page-locked allocation too
        r = hipPointerGetAttributes(&at, (const char *)host + bytes - 1);
        if (r != hipSuccess) { (void)hipGetLastError(); return false; }
        return at.type == hipMemoryTypeHost;
    }
};

int map_status(int s)
{
    switch (s) {
    case k3lms::OK: return K3_OK;
    case k3lms::E_BADARG: return K3_E_BADARG;
    case k3lms::E_OOM: return K3_E_OOM;
    case k3lms::E_NOT_PINNED: return K3_E_NOT_PINNED;
    case k3lms::E_STATE: return K3_E_STATE;
    default: return K3_E_HIP;
    }
}

}  // namespace

struct k3_lms {
    HipBackend be;
    k3lms::Engine eng;
    explicit k3_lms(uint64_t budget) : eng(&be, budget) {}
};

extern "C" {

int k3_lms_create(uint64_t device_budget_bytes, k3_lms **ctx)
{
    if (!ctx) return K3_E_BADARG;
    k3_lms *c = new (std::nothrow) k3_lms(device_budget_bytes);
    if (!c) return K3_E_OOM;
    int rc = c->eng.init();
    if (rc) {
        delete c;
        return map_status(rc);
    }
    *ctx = c;
    return K3_OK;
}

int k3_lms_destroy(k3_lms *ctx)
{
    if (!ctx) return K3_E_BADARG;
    delete ctx;
    return K3_OK;
}

int k3_lms_host_alloc(size_t bytes, void **host_ptr)
{
    if (!host_ptr || bytes == 0) return K3_E_BADARG;
    K3_HIP(hipHostMalloc(host_ptr, bytes, hipHostMallocDefault));
    return K3_OK;
}

int k3_lms_host_free(void *host_ptr)
{
    if (!host_ptr) return K3_E_BADARG;
    K3_HIP(hipHostFree(host_ptr));
    return K3_OK;
}

int k3_lms_account_alloc(k3_lms *ctx, uint64_t bytes) { return ctx ? map_status(ctx->eng.account_alloc(bytes)) : K3_E_BADARG; }
int k3_lms_account_free(k3_lms *ctx, uint64_t bytes) { return ctx ? map_status(ctx->eng.account_free(bytes)) : K3_E_BADARG; }

int k3_lms_swap_out(k3_lms *ctx, const void *dev_ptr, size_t bytes, void *host_ptr, void *compute_stream, int *handle)
{
    return ctx ? map_status(ctx->eng.swap_out(dev_ptr, bytes, host_ptr, compute_stream, handle)) : K3_E_BADARG;
}
int k3_lms_swap_out_done(k3_lms *ctx, int handle, int *done) { return ctx ? map_status(ctx->eng.swap_out_done(handle, done)) : K3_E_BADARG; }
int k3_lms_release_after(k3_lms *ctx, int handle, void *stream) { return ctx ? map_status(ctx->eng.release_after(handle, stream)) : K3_E_BADARG; }
int k3_lms_prefetch_in(k3_lms *ctx, int handle, void *dev_ptr, void *consumer_stream)
{
    return ctx ? map_status(ctx->eng.prefetch_in(handle, dev_ptr, consumer_stream)) : K3_E_BADARG;
}
int k3_lms_prefetch_start(k3_lms *ctx, int handle, void *dev_ptr, void *block_stream)
{
    return ctx ? map_status(ctx->eng.prefetch_start(handle, dev_ptr, block_stream)) : K3_E_BADARG;
}
int k3_lms_evict(k3_lms *ctx, int handle, void *stream) { return ctx ? map_status(ctx->eng.evict(handle, stream)) : K3_E_BADARG; }
int k3_lms_wait_in(k3_lms *ctx, int handle, void *stream) { return ctx ? map_status(ctx->eng.wait_in(handle, stream)) : K3_E_BADARG; }
int k3_lms_release(k3_lms *ctx, int handle) { return ctx ? map_status(ctx->eng.release(handle)) : K3_E_BADARG; }
int k3_lms_sync(k3_lms *ctx) { return ctx ? map_status(ctx->eng.sync()) : K3_E_BADARG; }
int k3_lms_handle_state(k3_lms *ctx, int handle, int *state) { return ctx ? map_status(ctx->eng.handle_state(handle, state)) : K3_E_BADARG; }

int k3_lms_set_poison(k3_lms *ctx, int on)
{
    if (!ctx) return K3_E_BADARG;
    ctx->eng.set_poison(on != 0);
    return K3_OK;
}

int k3_lms_set_copy_timing(k3_lms *ctx, int on)
{
    if (!ctx) return K3_E_BADARG;
    ctx->be.timing = on != 0;
    return K3_OK;
}

int k3_lms_copy_busy_ms(k3_lms *ctx, double *out_ms, double *in_ms)
{
    if (!ctx || !out_ms || !in_ms) return K3_E_BADARG;
    ctx->be.collect();
    *out_ms = ctx->be.busy_ms[0];
    *in_ms = ctx->be.busy_ms[1];
    return K3_OK;
}

int k3_lms_get_stats(k3_lms *ctx, k3_lms_stats *out)
{
    if (!ctx || !out) return K3_E_BADARG;
    const k3lms::Stats &s = ctx->eng.stats();
    out->bytes_out = s.bytes_out; out->bytes_in = s.bytes_in; out->n_out = s.n_out; out->n_in = s.n_in;
    out->device_bytes = s.device_bytes; out->device_peak = s.device_peak; out->live_handles = s.live_handles;
    return K3_OK;
}

}  // extern "C"
