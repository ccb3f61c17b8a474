// Swap-engine logic of the LMS scheme (paper section 2.2): which copies are issued, on
// which stream, fenced by which events, and the per-tensor state machine.  This file has
// no GPU dependency: all device work goes through the Backend interface, so the same
// logic runs against HIP in the library and against a host-memory mock in the CPU tests.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

namespace k3lms {

enum Status {
    OK = 0, E_BADARG = -1, E_OOM = -5, E_NOT_PINNED = -6, E_STATE = -7, E_BACKEND = -8
};
enum State { RESIDENT = 0, OUT_IN_FLIGHT = 1, ON_HOST = 2, IN_IN_FLIGHT = 3, FREE_SLOT = -1 };

typedef void *stream_t;
typedef void *event_t;

struct Backend {
    virtual ~Backend() {}
    virtual int stream_create(stream_t *s) = 0;
    virtual int stream_destroy(stream_t s) = 0;
    virtual int stream_sync(stream_t s) = 0;
    virtual int event_create(event_t *e) = 0;
    virtual int event_destroy(event_t e) = 0;
    virtual int event_record(event_t e, stream_t s) = 0;
    virtual int stream_wait_event(stream_t s, event_t e) = 0;
    virtual int event_query(event_t e, bool *done) = 0;
    virtual int event_sync(event_t e) = 0;
    virtual int copy_d2h(void *host, const void *dev, size_t bytes, stream_t s) = 0;
    virtual int copy_h2d(void *dev, const void *host, size_t bytes, stream_t s) = 0;
    virtual bool is_pinned(const void *host, size_t bytes) = 0;
    // debug aid: overwrite a device block with 0xFF bytes on stream s (see Engine::set_poison)
    virtual int fill_poison(void *dev, size_t bytes, stream_t s) = 0;
};

struct Stats {
    uint64_t bytes_out = 0, bytes_in = 0, n_out = 0, n_in = 0;
    uint64_t device_bytes = 0, device_peak = 0, live_handles = 0;
};

class Engine {
public:
    Engine(Backend *be, uint64_t device_budget_bytes);
    ~Engine();
    int init();  // creates the two copy streams
    int account_alloc(uint64_t bytes);
    int account_free(uint64_t bytes);
    int swap_out(const void *dev, size_t bytes, void *host, stream_t compute, int *handle);
    int swap_out_done(int handle, int *done);
    int release_after(int handle, stream_t s);
    int prefetch_in(int handle, void *dev, stream_t consumer);
    int prefetch_start(int handle, void *dev, stream_t block_stream);
    int evict(int handle, stream_t s);
    int wait_in(int handle, stream_t s);
    int release(int handle);
    int sync();
    int handle_state(int handle, int *state);
    // Debug switch: every device block whose tensor has gone to the host (release_after, evict) is
    // overwritten with 0xFF bytes (a bf16 / fp32 NaN pattern) on the stream that was just ordered
    // behind the copy, so a kernel that still reads the block after the swap is found out.
    void set_poison(bool on) { poison_ = on; }
    const Stats &stats() const { return stats_; }
    static const int kMaxHandles = 1 << 16;

private:
    struct Slot {
        int state = FREE_SLOT;
        const void *dev = nullptr;
        void *host = nullptr;
        size_t bytes = 0;
        bool handed = false;         // release_after gave the device block back while the copy-out may still run
        event_t ev_ready = nullptr;  // recorded on the compute stream before a copy may start
        event_t ev_out = nullptr;    // end of the device-to-host copy
        event_t ev_in = nullptr;     // end of the host-to-device copy
    };
    Slot *get(int handle);
    int refresh(Slot &s);
    Backend *be_;
    uint64_t budget_;
    bool poison_ = false;
    stream_t d2h_ = nullptr, h2d_ = nullptr;
    std::vector<Slot> slots_;
    std::vector<int> free_;
    Stats stats_;
};

}  // namespace k3lms
