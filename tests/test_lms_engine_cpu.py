"""Host-only tests of the swap engine's state machine and event fencing.

The engine source (csrc/lms_engine.cpp, no GPU dependency) is compiled with g++ against a
mock backend whose streams only advance when pumped, so in-flight states, ordering against
"kernels" on the compute stream and every error path can be forced from the host.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1811_12174_amd", "csrc")
OK, E_BADARG, E_OOM, E_NOT_PINNED, E_STATE, E_BACKEND = 0, -1, -5, -6, -7, -8
RESIDENT, OUT_IN_FLIGHT, ON_HOST, IN_IN_FLIGHT = 0, 1, 2, 3


@pytest.fixture(scope="module")
def mock(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("lmsmock") / "liblms_mock.so")
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-I" + CSRC, "-o", so,
                           os.path.join(ROOT, "tests", "lms_mock", "lms_mock.cpp"), os.path.join(CSRC, "lms_engine.cpp")])
    L = ctypes.CDLL(so)
    L.mock_create.restype = ctypes.c_void_p
    L.mock_create.argtypes = [ctypes.c_uint64]
    L.mock_stream_create.restype = ctypes.c_void_p
    L.mock_stream_create.argtypes = [ctypes.c_void_p]
    for name in ("mock_destroy", "mock_pump"):
        getattr(L, name).argtypes = [ctypes.c_void_p]
    L.mock_pin.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t]
    L.mock_fail_copies.argtypes = [ctypes.c_void_p, ctypes.c_int]
    L.mock_enqueue_fill.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t]
    L.mock_stream_pending.argtypes = [ctypes.c_void_p]
    L.mock_account_alloc.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
    L.mock_account_free.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
    L.mock_swap_out.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)]
    L.mock_swap_out_done.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    L.mock_release_after.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    L.mock_prefetch_in.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    L.mock_wait_in.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    L.mock_prefetch_start.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    L.mock_evict.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
    L.mock_release.argtypes = [ctypes.c_void_p, ctypes.c_int]
    L.mock_sync.argtypes = [ctypes.c_void_p]
    L.mock_state.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    L.mock_stats.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint64)]
    L.mock_set_poison.argtypes = [ctypes.c_void_p, ctypes.c_int]
    return L


class Env:
    def __init__(self, L, budget=0, n=4096):
        self.L = L
        self.c = L.mock_create(budget)
        self.compute = L.mock_stream_create(self.c)
        self.dev = np.arange(n, dtype=np.uint8) * 7 % 251
        self.dev = self.dev.astype(np.uint8)
        self.orig = self.dev.copy()
        self.host = np.zeros(n, dtype=np.uint8)
        L.mock_pin(self.c, self.host.ctypes.data, n)
        self.n = n

    def state(self, h):
        s = ctypes.c_int(-9)
        assert self.L.mock_state(self.c, h, ctypes.byref(s)) == OK
        return s.value

    def stats(self):
        a = (ctypes.c_uint64 * 7)()
        self.L.mock_stats(self.c, a)
        return list(a)

    def close(self):
        self.L.mock_destroy(self.c)


def test_round_trip_and_states(mock):
    e = Env(mock)
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert e.state(h.value) == OUT_IN_FLIGHT
    done = ctypes.c_int(5)
    assert mock.mock_swap_out_done(e.c, h.value, ctypes.byref(done)) == OK and done.value == 0
    assert not np.array_equal(e.host, e.orig)           # nothing ran yet
    mock.mock_pump(e.c)
    assert np.array_equal(e.host, e.orig)
    assert mock.mock_swap_out_done(e.c, h.value, ctypes.byref(done)) == OK and done.value == 1
    assert e.state(h.value) == ON_HOST
    # poison the device block, then bring the tensor back
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK
    e.dev[:] = 0xFF
    assert mock.mock_prefetch_in(e.c, h.value, e.dev.ctypes.data, e.compute) == OK
    assert e.state(h.value) == IN_IN_FLIGHT
    mock.mock_pump(e.c)
    assert e.state(h.value) == RESIDENT
    assert np.array_equal(e.dev, e.orig)
    assert mock.mock_release(e.c, h.value) == OK
    st = e.stats()
    assert st[0] == e.n and st[1] == e.n and st[2] == 1 and st[3] == 1 and st[6] == 0
    e.close()


def test_copy_waits_for_producer_and_consumer_waits_for_copy(mock):
    """The D2H copy must see what the compute stream wrote before swap_out; a kernel enqueued
    after prefetch_in must run after the H2D copy; the H2D copy must not overtake earlier
    users of the destination block."""
    e = Env(mock)
    mock.mock_enqueue_fill(e.c, e.compute, e.dev.ctypes.data, 0x11, e.n)     # producer kernel, not run yet
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK
    mock.mock_enqueue_fill(e.c, e.compute, e.dev.ctypes.data, 0x22, e.n)     # reuses the block after release
    mock.mock_pump(e.c)
    assert np.all(e.host == 0x11)      # copy saw the producer's data, not the later overwrite
    assert np.all(e.dev == 0x22)
    mock.mock_enqueue_fill(e.c, e.compute, e.dev.ctypes.data, 0x33, e.n)     # earlier user of the destination
    assert mock.mock_prefetch_in(e.c, h.value, e.dev.ctypes.data, e.compute) == OK
    probe = np.zeros(e.n, dtype=np.uint8)
    # "consumer kernel": copies dev -> probe on the compute stream after the prefetch
    mock.mock_enqueue_fill(e.c, e.compute, probe.ctypes.data, 0, 1)          # keeps the queue non-trivial
    mock.mock_pump(e.c)
    assert np.all(e.dev == 0x11)       # H2D copy landed after the 0x33 fill
    assert mock.mock_stream_pending(e.compute) == 0
    e.close()


def test_prefetch_before_swap_out_finished_is_ordered(mock):
    e = Env(mock)
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK      # ON_HOST without a host-side wait
    dst = np.zeros(e.n, dtype=np.uint8)
    assert mock.mock_prefetch_in(e.c, h.value, dst.ctypes.data, e.compute) == OK
    mock.mock_pump(e.c)
    assert np.array_equal(dst, e.orig)
    e.close()


def test_illegal_transitions(mock):
    e = Env(mock)
    h = ctypes.c_int(-1)
    dst = np.zeros(e.n, dtype=np.uint8)
    assert mock.mock_prefetch_in(e.c, 0, dst.ctypes.data, e.compute) == E_BADARG       # never swapped
    assert mock.mock_release(e.c, 3) == E_BADARG
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_prefetch_in(e.c, h.value, dst.ctypes.data, e.compute) == E_STATE   # copy still in flight, block not released
    assert mock.mock_wait_in(e.c, h.value, e.compute) == E_STATE
    mock.mock_pump(e.c)
    assert mock.mock_prefetch_in(e.c, h.value, dst.ctypes.data, e.compute) == OK
    assert mock.mock_prefetch_in(e.c, h.value, dst.ctypes.data, e.compute) == E_STATE   # double prefetch
    assert mock.mock_release_after(e.c, h.value, e.compute) == E_STATE
    mock.mock_pump(e.c)
    assert mock.mock_release(e.c, h.value) == OK
    assert mock.mock_release(e.c, h.value) == E_BADARG                                  # double release
    done = ctypes.c_int(0)
    assert mock.mock_swap_out_done(e.c, h.value, ctypes.byref(done)) == E_BADARG
    e.close()


def test_not_pinned_and_bad_args(mock):
    e = Env(mock)
    h = ctypes.c_int(-1)
    loose = np.zeros(e.n, dtype=np.uint8)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, loose.ctypes.data, e.compute, ctypes.byref(h)) == E_NOT_PINNED
    # a range that starts pinned but runs past the registered block
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data + 1, e.compute, ctypes.byref(h)) == E_NOT_PINNED
    assert mock.mock_swap_out(e.c, None, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == E_BADARG
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, 0, e.host.ctypes.data, e.compute, ctypes.byref(h)) == E_BADARG
    assert e.stats()[6] == 0
    e.close()


def test_backend_failure_leaves_no_handle(mock):
    e = Env(mock)
    h = ctypes.c_int(-1)
    mock.mock_fail_copies(e.c, 1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == E_BACKEND
    assert e.stats()[6] == 0
    mock.mock_fail_copies(e.c, 0)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert h.value == 0         # the failed attempt's slot was recycled
    e.close()


def test_device_budget(mock):
    e = Env(mock, budget=1000)
    assert mock.mock_account_alloc(e.c, 600) == OK
    assert mock.mock_account_alloc(e.c, 500) == E_OOM
    assert e.stats()[4] == 600
    assert mock.mock_account_free(e.c, 600) == OK
    assert mock.mock_account_alloc(e.c, 1000) == OK
    assert mock.mock_account_free(e.c, 2000) == E_BADARG
    assert e.stats()[5] == 1000
    e.close()


def test_release_while_in_flight_waits(mock):
    e = Env(mock)
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_release(e.c, h.value) == OK        # synchronises on the copy first
    assert np.array_equal(e.host, e.orig)
    e.close()


def test_many_handles_recycle(mock):
    e = Env(mock, n=64 * 16)
    hs = []
    for i in range(16):
        h = ctypes.c_int(-1)
        assert mock.mock_swap_out(e.c, e.dev.ctypes.data + 64 * i, 64, e.host.ctypes.data + 64 * i, e.compute, ctypes.byref(h)) == OK
        hs.append(h.value)
    assert sorted(hs) == list(range(16))
    assert mock.mock_sync(e.c) == OK
    assert np.array_equal(e.host, e.orig)
    for h in hs:
        assert mock.mock_release(e.c, h) == OK
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, 64, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert h.value in hs
    e.close()


def test_prefetch_start_overlaps_until_wait_in(mock):
    """prefetch_start does not fence the compute stream: a kernel enqueued after it but before
    wait_in may run before the copy lands, one enqueued after wait_in may not."""
    e = Env(mock)
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    mock.mock_pump(e.c)
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK
    dst = np.zeros(e.n, dtype=np.uint8)
    mock.mock_enqueue_fill(e.c, e.compute, dst.ctypes.data, 0x44, e.n)        # earlier user of the block
    assert mock.mock_prefetch_start(e.c, h.value, dst.ctypes.data, e.compute) == OK
    assert e.state(h.value) == IN_IN_FLIGHT
    assert mock.mock_wait_in(e.c, h.value, e.compute) == OK
    probe = np.zeros(1, dtype=np.uint8)
    mock.mock_enqueue_fill(e.c, e.compute, probe.ctypes.data, 1, 1)           # "consumer"
    mock.mock_pump(e.c)
    assert np.array_equal(dst, e.orig)      # the copy landed after the 0x44 fill, not before
    assert probe[0] == 1 and e.state(h.value) == RESIDENT
    assert mock.mock_release(e.c, h.value) == OK
    e.close()


def test_evict_keeps_the_host_copy_and_allows_a_second_prefetch(mock):
    e = Env(mock)
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_evict(e.c, h.value, e.compute) == E_STATE                # still going out
    mock.mock_pump(e.c)
    assert mock.mock_evict(e.c, h.value, e.compute) == E_STATE                # ON_HOST: nothing to drop
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK
    first = np.zeros(e.n, dtype=np.uint8)
    assert mock.mock_prefetch_start(e.c, h.value, first.ctypes.data, e.compute) == OK
    # evicted while the copy-in is still in flight: the stream is fenced behind the copy, so a
    # later overwrite of the block cannot be overtaken by it
    assert mock.mock_evict(e.c, h.value, e.compute) == OK
    assert e.state(h.value) == ON_HOST
    mock.mock_enqueue_fill(e.c, e.compute, first.ctypes.data, 0x55, e.n)      # block reused
    mock.mock_pump(e.c)
    assert np.all(first == 0x55)
    second = np.zeros(e.n, dtype=np.uint8)
    assert mock.mock_prefetch_in(e.c, h.value, second.ctypes.data, e.compute) == OK
    mock.mock_pump(e.c)
    assert np.array_equal(second, e.orig)
    st = e.stats()
    assert st[0] == e.n and st[1] == 2 * e.n and st[2] == 1 and st[3] == 2   # one copy out, two in
    assert mock.mock_evict(e.c, h.value, e.compute) == OK                     # RESIDENT -> ON_HOST
    assert mock.mock_evict(e.c, 999, e.compute) == E_BADARG
    assert mock.mock_release(e.c, h.value) == OK
    e.close()


def test_release_after_keeps_reporting_the_copy_until_it_has_finished(mock):
    """release_after hands the device block to a stream; the copy-out may still be running.  The
    handle must keep saying so (swap_out_done, handle_state), and release must wait for the copy:
    a caller that reuses the host buffer after release would otherwise be overwritten by it."""
    e = Env(mock)
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK
    done = ctypes.c_int(5)
    assert mock.mock_swap_out_done(e.c, h.value, ctypes.byref(done)) == OK and done.value == 0
    assert e.state(h.value) == OUT_IN_FLIGHT
    assert not np.array_equal(e.host, e.orig)           # the copy has not run
    assert mock.mock_release(e.c, h.value) == OK        # waits for it
    assert np.array_equal(e.host, e.orig)
    # the same with the copy finishing in between
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK
    mock.mock_pump(e.c)
    assert mock.mock_swap_out_done(e.c, h.value, ctypes.byref(done)) == OK and done.value == 1
    assert e.state(h.value) == ON_HOST
    assert mock.mock_release(e.c, h.value) == OK
    e.close()


def test_poison_mode_overwrites_blocks_whose_tensor_went_to_the_host(mock):
    e = Env(mock)
    mock.mock_set_poison(e.c, 1)
    h = ctypes.c_int(-1)
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK
    assert np.array_equal(e.dev, e.orig)                # ordered behind the copy: nothing ran yet
    mock.mock_pump(e.c)
    assert np.array_equal(e.host, e.orig)               # the copy saw the data, then the block was poisoned
    assert np.all(e.dev == 0xFF)
    back = np.zeros(e.n, dtype=np.uint8)
    assert mock.mock_prefetch_in(e.c, h.value, back.ctypes.data, e.compute) == OK
    mock.mock_pump(e.c)
    assert np.array_equal(back, e.orig)
    assert mock.mock_evict(e.c, h.value, e.compute) == OK   # dropped again without a copy: poisoned too
    mock.mock_pump(e.c)
    assert np.all(back == 0xFF)
    again = np.zeros(e.n, dtype=np.uint8)
    assert mock.mock_prefetch_in(e.c, h.value, again.ctypes.data, e.compute) == OK
    mock.mock_pump(e.c)
    assert np.array_equal(again, e.orig)
    assert mock.mock_release(e.c, h.value) == OK
    # switched off: blocks are left alone
    mock.mock_set_poison(e.c, 0)
    e.dev[:] = e.orig
    assert mock.mock_swap_out(e.c, e.dev.ctypes.data, e.n, e.host.ctypes.data, e.compute, ctypes.byref(h)) == OK
    assert mock.mock_release_after(e.c, h.value, e.compute) == OK
    mock.mock_pump(e.c)
    assert np.array_equal(e.dev, e.orig)
    assert mock.mock_release(e.c, h.value) == OK
    e.close()
