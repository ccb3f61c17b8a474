// Host-memory mock backend for the swap engine's CPU tests.  "Device" memory is ordinary
// host memory.  Streams are FIFO queues of deferred operations that only run when the test
// pumps them (mock_pump) or something synchronises, so the tests can observe in-flight
// states and verify that every copy is fenced by the right events.
#include <cstdint>
#include <cstring>
#include <deque>
#include <functional>
#include <map>
#include <string>
#include <set>
#include <vector>

#include "lms_engine.h"

using namespace k3lms;

namespace {

struct MockEvent {
    uint64_t recorded = 0;   // generation of the last record call
    uint64_t completed = 0;  // generation that has completed
};

struct Op {
    enum Kind { RECORD, WAIT, COPY } kind;
    MockEvent *ev = nullptr;
    uint64_t gen = 0;
    void *dst = nullptr;
    const void *src = nullptr;
    size_t bytes = 0;
};

struct MockStream {
    std::deque<Op> q;
};

struct MockBackend : Backend {
    std::set<MockStream *> streams;
    std::set<const void *> pinned_bases;
    std::map<const void *, size_t> pinned;
    std::vector<std::string> log;
    int fail_copies = 0;

    // runs queued operations until every stream is empty or blocked on an unfinished event
    bool step_stream(MockStream *s)
    {
        bool progressed = false;
        while (!s->q.empty()) {
            Op &op = s->q.front();
            if (op.kind == Op::WAIT) {
                if (op.ev->completed < op.gen) break;
            } else if (op.kind == Op::RECORD) {
                op.ev->completed = op.gen;
            } else {
                memcpy(op.dst, op.src, op.bytes);
            }
            s->q.pop_front();
            progressed = true;
        }
        return progressed;
    }
    void pump()
    {
        bool again = true;
        while (again) {
            again = false;
            for (MockStream *s : streams) again |= step_stream(s);
        }
    }
    int stream_create(stream_t *s) override
    {
        MockStream *m = new MockStream;
        streams.insert(m);
        *s = m;
        return 0;
    }
    int stream_destroy(stream_t s) override
    {
        streams.erase((MockStream *)s);
        delete (MockStream *)s;
        return 0;
    }
    int stream_sync(stream_t s) override
    {
        pump();
        return ((MockStream *)s)->q.empty() ? 0 : 1;  // non-empty after pumping = deadlock
    }
    int event_create(event_t *e) override { *e = new MockEvent; return 0; }
    int event_destroy(event_t e) override { delete (MockEvent *)e; return 0; }
    int event_record(event_t e, stream_t s) override
    {
        MockEvent *ev = (MockEvent *)e;
        ev->recorded += 1;
        Op op; op.kind = Op::RECORD; op.ev = ev; op.gen = ev->recorded;
        ((MockStream *)s)->q.push_back(op);
        return 0;
    }
    int stream_wait_event(stream_t s, event_t e) override
    {
        MockEvent *ev = (MockEvent *)e;
        Op op; op.kind = Op::WAIT; op.ev = ev; op.gen = ev->recorded;  // waits for the latest record so far
        ((MockStream *)s)->q.push_back(op);
        return 0;
    }
    int event_query(event_t e, bool *done) override
    {
        MockEvent *ev = (MockEvent *)e;
        *done = ev->completed >= ev->recorded;
        return 0;
    }
    int event_sync(event_t e) override
    {
        pump();
        MockEvent *ev = (MockEvent *)e;
        return ev->completed >= ev->recorded ? 0 : 1;
    }
    int copy_d2h(void *host, const void *dev, size_t bytes, stream_t s) override
    {
        if (fail_copies) return 1;
        Op op; op.kind = Op::COPY; op.dst = host; op.src = dev; op.bytes = bytes;
        ((MockStream *)s)->q.push_back(op);
        return 0;
    }
    int copy_h2d(void *dev, const void *host, size_t bytes, stream_t s) override
    {
        if (fail_copies) return 1;
        Op op; op.kind = Op::COPY; op.dst = dev; op.src = host; op.bytes = bytes;
        ((MockStream *)s)->q.push_back(op);
        return 0;
    }
    int fill_poison(void *dev, size_t bytes, stream_t s) override
    {
        char *src = new char[bytes];   // leaked: the deferred copy reads it when the stream is pumped
        memset(src, 0xFF, bytes);
        Op op; op.kind = Op::COPY; op.dst = dev; op.src = src; op.bytes = bytes;
        ((MockStream *)s)->q.push_back(op);
        return 0;
    }
    bool is_pinned(const void *host, size_t bytes) override
    {
        for (auto &kv : pinned) {
            const char *b = (const char *)kv.first;
            if ((const char *)host >= b && (const char *)host + bytes <= b + kv.second) return true;
        }
        return false;
    }
};

struct Ctx {
    MockBackend be;
    Engine eng;
    explicit Ctx(uint64_t budget) : eng(&be, budget) {}
};

}  // namespace

extern "C" {
void *mock_create(uint64_t budget)
{
    Ctx *c = new Ctx(budget);
    if (c->eng.init()) { delete c; return nullptr; }
    return c;
}
void mock_destroy(void *c) { delete (Ctx *)c; }
void *mock_stream_create(void *c) { stream_t s; ((Ctx *)c)->be.stream_create(&s); return s; }
void mock_pin(void *c, const void *p, size_t n) { ((Ctx *)c)->be.pinned[p] = n; }
void mock_pump(void *c) { ((Ctx *)c)->be.pump(); }
void mock_fail_copies(void *c, int on) { ((Ctx *)c)->be.fail_copies = on; }
// a "kernel" on a compute stream: a deferred memset, so ordering against copies is observable
void mock_enqueue_fill(void *c, void *stream, void *dst, int value, size_t n)
{
    (void)c;
    // implemented as a copy from a leaked constant buffer to keep the Op struct simple
    char *src = new char[n];
    memset(src, value, n);
    Op op; op.kind = Op::COPY; op.dst = dst; op.src = src; op.bytes = n;
    ((MockStream *)stream)->q.push_back(op);
}
int mock_stream_pending(void *stream) { return (int)((MockStream *)stream)->q.size(); }

int mock_account_alloc(void *c, uint64_t b) { return ((Ctx *)c)->eng.account_alloc(b); }
int mock_account_free(void *c, uint64_t b) { return ((Ctx *)c)->eng.account_free(b); }
int mock_swap_out(void *c, const void *dev, size_t n, void *host, void *stream, int *h) { return ((Ctx *)c)->eng.swap_out(dev, n, host, stream, h); }
int mock_swap_out_done(void *c, int h, int *done) { return ((Ctx *)c)->eng.swap_out_done(h, done); }
int mock_release_after(void *c, int h, void *stream) { return ((Ctx *)c)->eng.release_after(h, stream); }
int mock_prefetch_in(void *c, int h, void *dev, void *stream) { return ((Ctx *)c)->eng.prefetch_in(h, dev, stream); }
int mock_prefetch_start(void *c, int h, void *dev, void *stream) { return ((Ctx *)c)->eng.prefetch_start(h, dev, stream); }
int mock_evict(void *c, int h, void *stream) { return ((Ctx *)c)->eng.evict(h, stream); }
int mock_wait_in(void *c, int h, void *stream) { return ((Ctx *)c)->eng.wait_in(h, stream); }
int mock_release(void *c, int h) { return ((Ctx *)c)->eng.release(h); }
int mock_sync(void *c) { return ((Ctx *)c)->eng.sync(); }
void mock_set_poison(void *c, int on) { ((Ctx *)c)->eng.set_poison(on != 0); }
int mock_state(void *c, int h, int *s) { return ((Ctx *)c)->eng.handle_state(h, s); }
void mock_stats(void *c, uint64_t *out)
{
    const Stats &s = ((Ctx *)c)->eng.stats();
    out[0] = s.bytes_out; out[1] = s.bytes_in; out[2] = s.n_out; out[3] = s.n_in;
    out[4] = s.device_bytes; out[5] = s.device_peak; out[6] = s.live_handles;
}
}
