// See lms_engine.h.  Ordering rules implemented here:
//  swap-out : ev_ready recorded on the compute stream -> D2H stream waits for it -> copy ->
//             ev_out recorded on the D2H stream.  The device block may be reused by a stream
//             only after that stream waited for ev_out (release_after).
//  prefetch : ev_ready recorded on the consumer stream (earlier users of the destination
//             block) -> H2D stream waits for it and for ev_out -> copy -> ev_in recorded on
//             the H2D stream -> the consumer stream waits for ev_in (prefetch_in at once,
//             prefetch_start leaves that wait to a later wait_in so the copy overlaps the
//             kernels enqueued in between).
//  evict    : a tensor that came back and was only read goes ON_HOST again without a copy.
//  A handle stays OUT_IN_FLIGHT until its copy-out has really finished, also after release_after
//  handed the device block to a stream: swap_out_done and handle_state report the copy, and
//  release waits for it, so the host buffer is safe to reuse once the handle is released.
#include "lms_engine.h"

namespace k3lms {

#define BE(call)                         \
    do {                                 \
        if ((call) != 0) return E_BACKEND; \
    } while (0)

Engine::Engine(Backend *be, uint64_t budget) : be_(be), budget_(budget) {}

Engine::~Engine()
{
    if (d2h_) be_->stream_sync(d2h_);
    if (h2d_) be_->stream_sync(h2d_);
    for (Slot &s : slots_) {
        if (s.ev_ready) be_->event_destroy(s.ev_ready);
        if (s.ev_out) be_->event_destroy(s.ev_out);
        if (s.ev_in) be_->event_destroy(s.ev_in);
    }
    if (d2h_) be_->stream_destroy(d2h_);
    if (h2d_) be_->stream_destroy(h2d_);
}

int Engine::init()
{
    BE(be_->stream_create(&d2h_));
    BE(be_->stream_create(&h2d_));
    return OK;
}

int Engine::account_alloc(uint64_t bytes)
{
    if (budget_ && stats_.device_bytes + bytes > budget_) return E_OOM;
    stats_.device_bytes += bytes;
    if (stats_.device_bytes > stats_.device_peak) stats_.device_peak = stats_.device_bytes;
    return OK;
}

int Engine::account_free(uint64_t bytes)
{
    if (bytes > stats_.device_bytes) return E_BADARG;
    stats_.device_bytes -= bytes;
    return OK;
}

Engine::Slot *Engine::get(int handle)
{
    if (handle < 0 || handle >= (int)slots_.size()) return nullptr;
    Slot *s = &slots_[handle];
    return s->state == FREE_SLOT ? nullptr : s;
}

// Moves a slot out of an in-flight state once its copy has finished.
int Engine::refresh(Slot &s)
{
    bool done = false;
    if (s.state == OUT_IN_FLIGHT) {
        BE(be_->event_query(s.ev_out, &done));
        if (done) s.state = ON_HOST;
    } else if (s.state == IN_IN_FLIGHT) {
        BE(be_->event_query(s.ev_in, &done));
        if (done) s.state = RESIDENT;
    }
    return OK;
}

int Engine::swap_out(const void *dev, size_t bytes, void *host, stream_t compute, int *handle)
{
    if (!dev || !host || !handle || bytes == 0) return E_BADARG;
    if (!be_->is_pinned(host, bytes)) return E_NOT_PINNED;
    int h;
    if (!free_.empty()) {
        h = free_.back();
        free_.pop_back();
    } else {
        if ((int)slots_.size() >= kMaxHandles) return E_OOM;
        slots_.emplace_back();
        h = (int)slots_.size() - 1;
    }
    Slot &s = slots_[h];
    if (!s.ev_ready) {
        if (be_->event_create(&s.ev_ready) || be_->event_create(&s.ev_out) || be_->event_create(&s.ev_in)) {
            free_.push_back(h);
            return E_BACKEND;
        }
    }
    s.dev = dev; s.host = host; s.bytes = bytes;
    s.handed = false;
    int rc = 0;
    rc |= be_->event_record(s.ev_ready, compute);
    rc |= be_->stream_wait_event(d2h_, s.ev_ready);
    rc |= be_->copy_d2h(host, dev, bytes, d2h_);
    rc |= be_->event_record(s.ev_out, d2h_);
    if (rc) {
        free_.push_back(h);
        return E_BACKEND;
    }
    s.state = OUT_IN_FLIGHT;
    stats_.bytes_out += bytes;
    stats_.n_out += 1;
    stats_.live_handles += 1;
    *handle = h;
    return OK;
}

int Engine::swap_out_done(int handle, int *done)
{
    Slot *s = get(handle);
    if (!s || !done) return E_BADARG;
    if (s->state == RESIDENT) return E_STATE;
    int rc = refresh(*s);
    if (rc) return rc;
    *done = s->state != OUT_IN_FLIGHT;
    return OK;
}

int Engine::release_after(int handle, stream_t st)
{
    Slot *s = get(handle);
    if (!s) return E_BADARG;
    if (s->state != OUT_IN_FLIGHT && s->state != ON_HOST) return E_STATE;
    BE(be_->stream_wait_event(st, s->ev_out));   // st is ordered after the copy from here on
    if (poison_ && s->dev) BE(be_->fill_poison(const_cast<void *>(s->dev), s->bytes, st));
    s->handed = true;
    s->dev = nullptr;
    return refresh(*s);   // ON_HOST only once the copy has really finished
}

int Engine::prefetch_start(int handle, void *dev, stream_t block_stream)
{
    Slot *s = get(handle);
    if (!s || !dev) return E_BADARG;
    if (s->state == OUT_IN_FLIGHT) {
        int rc = refresh(*s);
        if (rc) return rc;
    }
    // a copy-out still in flight is fine once the block was handed over: the copy-in waits for it
    if (s->state != ON_HOST && !(s->state == OUT_IN_FLIGHT && s->handed)) return E_STATE;
    BE(be_->event_record(s->ev_ready, block_stream));
    BE(be_->stream_wait_event(h2d_, s->ev_ready));
    BE(be_->stream_wait_event(h2d_, s->ev_out));  // no-op when the swap-out already finished
    BE(be_->copy_h2d(dev, s->host, s->bytes, h2d_));
    BE(be_->event_record(s->ev_in, h2d_));
    s->dev = dev;
    s->state = IN_IN_FLIGHT;
    stats_.bytes_in += s->bytes;
    stats_.n_in += 1;
    return OK;
}

int Engine::prefetch_in(int handle, void *dev, stream_t consumer)
{
    int rc = prefetch_start(handle, dev, consumer);
    if (rc) return rc;
    BE(be_->stream_wait_event(consumer, slots_[handle].ev_in));
    return OK;
}

int Engine::evict(int handle, stream_t st)
{
    Slot *s = get(handle);
    if (!s) return E_BADARG;
    if (s->state != IN_IN_FLIGHT && s->state != RESIDENT) return E_STATE;
    // work enqueued on st from here on (the next user of the block) runs after the copy-in
    BE(be_->stream_wait_event(st, s->ev_in));
    if (poison_ && s->dev) BE(be_->fill_poison(const_cast<void *>(s->dev), s->bytes, st));
    s->state = ON_HOST;  // the host copy made by the swap-out is still the tensor's value
    s->dev = nullptr;
    return OK;
}

int Engine::wait_in(int handle, stream_t st)
{
    Slot *s = get(handle);
    if (!s) return E_BADARG;
    if (s->state != IN_IN_FLIGHT && s->state != RESIDENT) return E_STATE;
    BE(be_->stream_wait_event(st, s->ev_in));
    return OK;
}

int Engine::release(int handle)
{
    Slot *s = get(handle);
    if (!s) return E_BADARG;
    if (s->state == OUT_IN_FLIGHT) BE(be_->event_sync(s->ev_out));
    if (s->state == IN_IN_FLIGHT) BE(be_->event_sync(s->ev_in));
    s->state = FREE_SLOT;
    s->handed = false;
    s->dev = nullptr;
    s->host = nullptr;
    s->bytes = 0;
    free_.push_back(handle);
    stats_.live_handles -= 1;
    return OK;
}

int Engine::sync()
{
    BE(be_->stream_sync(d2h_));
    BE(be_->stream_sync(h2d_));
    return OK;
}

int Engine::handle_state(int handle, int *state)
{
    Slot *s = get(handle);
    if (!s || !state) return E_BADARG;
    int rc = refresh(*s);
    if (rc) return rc;
    *state = s->state;
    return OK;
}

}  // namespace k3lms
