"""ctypes binding of libk3.so (see include/k3.h).  Argument marshalling only.

Tensors are torch tensors used purely as device-memory handles: NDHWC, contiguous,
torch.bfloat16 or torch.float32.  Every function enqueues work on the current torch
HIP stream and returns without synchronising.
"""
import ctypes
import os

import torch  # loads the HIP runtime the library links against; also owns device memory

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libk3.so")

BF16, F32 = 1, 2
OK = 0
E_BADARG, E_SHAPE, E_UNSUPPORTED, E_WORKSPACE, E_OOM, E_NOT_PINNED, E_STATE, E_HIP = -1, -2, -3, -4, -5, -6, -7, -8
LMS_RESIDENT, LMS_OUT_IN_FLIGHT, LMS_ON_HOST, LMS_IN_IN_FLIGHT = 0, 1, 2, 3


class K3Error(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_string(status)})")


class TensorDesc(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int64), ("d", ctypes.c_int64), ("h", ctypes.c_int64), ("w", ctypes.c_int64),
                ("c", ctypes.c_int64), ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class LmsStats(ctypes.Structure):
    _fields_ = [("bytes_out", ctypes.c_uint64), ("bytes_in", ctypes.c_uint64), ("n_out", ctypes.c_uint64),
                ("n_in", ctypes.c_uint64), ("device_bytes", ctypes.c_uint64), ("device_peak", ctypes.c_uint64),
                ("live_handles", ctypes.c_uint64)]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        L.k3_status_string.restype = ctypes.c_char_p
        L.k3_status_string.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_string(status):
    return lib().k3_status_string(int(status)).decode()


def version():
    return lib().k3_version()


def last_hip_error():
    return lib().k3_last_hip_error()


def _check(status, what):
    if status != OK:
        raise K3Error(status, what)


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def desc(t):
    """Descriptor of a contiguous NDHWC torch tensor."""
    if t.dim() != 5 or not t.is_contiguous():
        raise ValueError("expected a contiguous 5-d NDHWC tensor")
    n, d, h, w, c = t.shape
    return TensorDesc(n, d, h, w, c, _dtype_code(t), 0)


def _p(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _d(t):
    return None if t is None else ctypes.byref(desc(t))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


# ------------------------------------------------------------------ 3x3x3 convolution
def conv3d_packed_bytes(cin, cout, dtype):
    out = ctypes.c_size_t(0)
    _check(lib().k3_conv3d_packed_bytes(ctypes.c_int64(cin), ctypes.c_int64(cout), ctypes.c_int(dtype),
                                        ctypes.byref(out)), "k3_conv3d_packed_bytes")
    return out.value


def conv3d_pack_weights(w, packed):
    """w: [3,3,3,cin,cout] device tensor; packed: uint8 device tensor of conv3d_packed_bytes or None."""
    cin, cout = w.shape[3], w.shape[4]
    nbytes = 0 if packed is None else packed.numel() * packed.element_size()
    _check(lib().k3_conv3d_pack_weights(_p(w), ctypes.c_int64(cin), ctypes.c_int64(cout), ctypes.c_int(_dtype_code(w)),
                                        _p(packed), ctypes.c_size_t(nbytes), _stream()), "k3_conv3d_pack_weights")


def conv3d_fwd(x, w, packed, bias, relu, y, x2=None):
    _check(lib().k3_conv3d_fwd(_d(x), _p(x), _d(x2), _p(x2), _p(w), _p(packed), _p(bias), ctypes.c_int(int(relu)),
                               _d(y), _p(y), _stream()), "k3_conv3d_fwd")


def relu_bits_bytes(y):
    out = ctypes.c_size_t(0)
    _check(lib().k3_relu_bits_bytes(_d(y), ctypes.byref(out)), "k3_relu_bits_bytes")
    return out.value


def conv3d_fwd_bits(x, w, packed, bias, relu, y, relu_bits, x2=None):
    """conv3d_fwd that also writes the one-bit-per-element mask of y into relu_bits (see relu_bits_bytes)."""
    _check(lib().k3_conv3d_fwd_bits(_d(x), _p(x), _d(x2), _p(x2), _p(w), _p(packed), _p(bias), ctypes.c_int(int(relu)),
                                    _d(y), _p(y), _p(relu_bits), _stream()), "k3_conv3d_fwd_bits")


def conv3d_fwd_pool(x, w, packed, bias, relu, y, y_pooled, x2=None):
    """conv3d_fwd plus the 2x2x2 max-pool of its output into y_pooled."""
    _check(lib().k3_conv3d_fwd_pool(_d(x), _p(x), _d(x2), _p(x2), _p(w), _p(packed), _p(bias), ctypes.c_int(int(relu)),
                                    _d(y), _p(y), _d(y_pooled), _p(y_pooled), _stream()), "k3_conv3d_fwd_pool")


def conv3d_bwd_data(dy, y_mask, w, packed, dx, dx2=None, dx_mask=None):
    _check(lib().k3_conv3d_bwd_data(_d(dy), _p(dy), _p(y_mask), _p(w), _p(packed), _d(dx), _p(dx), _d(dx2), _p(dx2),
                                    _p(dx_mask), _stream()), "k3_conv3d_bwd_data")


def conv3d_bwd_data_bits(dy, y_mask, w, packed, dx, dx_mask_bits, dx2=None):
    """conv3d_bwd_data with the mask of dx given as bits."""
    _check(lib().k3_conv3d_bwd_data_bits(_d(dy), _p(dy), _p(y_mask), _p(w), _p(packed), _d(dx), _p(dx), _d(dx2), _p(dx2),
                                         _p(dx_mask_bits), _stream()), "k3_conv3d_bwd_data_bits")


def conv3d_bwd_weight_workspace_bytes(x, dy, x2=None):
    out = ctypes.c_size_t(0)
    _check(lib().k3_conv3d_bwd_weight_workspace_bytes(_d(x), _d(x2), _d(dy), ctypes.byref(out)),
           "k3_conv3d_bwd_weight_workspace_bytes")
    return out.value


def conv3d_bwd_weight(x, dy, y_mask, dW, db, ws, x2=None):
    _check(lib().k3_conv3d_bwd_weight(_d(x), _p(x), _d(x2), _p(x2), _d(dy), _p(dy), _p(y_mask), _p(dW), _p(db),
                                      _p(ws), ctypes.c_size_t(ws.numel() * ws.element_size()), _stream()),
           "k3_conv3d_bwd_weight")


STATIC_SCRATCH_BYTES = 64 << 20


def conv3d_bwd_weight_static(x, dy, y_mask, dW, db, x2=None):
    """conv3d_bwd_weight whose partial sums go to the library's own static device array (allocates nothing)."""
    _check(lib().k3_conv3d_bwd_weight_static(_d(x), _p(x), _d(x2), _p(x2), _d(dy), _p(dy), _p(y_mask), _p(dW), _p(db),
                                             _stream()), "k3_conv3d_bwd_weight_static")


# ------------------------------------------------------------------ pooling
def pool3d_fwd(x, y):
    _check(lib().k3_pool3d_fwd(_d(x), _p(x), _d(y), _p(y), _stream()), "k3_pool3d_fwd")


def pool3d_bwd(x, dy, add, dx, relu_mask=False):
    _check(lib().k3_pool3d_bwd(_d(x), _p(x), _d(dy), _p(dy), _p(add), ctypes.c_int(int(relu_mask)), _p(dx), _stream()),
           "k3_pool3d_bwd")


def pool3d_fwd_bits(x, y, route_bits):
    """pool3d_fwd that also writes one routing bit per element of x (size: relu_bits_bytes(x))."""
    _check(lib().k3_pool3d_fwd_bits(_d(x), _p(x), _d(y), _p(y), _p(route_bits), _stream()), "k3_pool3d_fwd_bits")


def pool3d_bwd_bits(route_bits, dy, dx):
    """pool3d_bwd(x, dy, None, dx, relu_mask=True) from the bits pool3d_fwd_bits wrote for x."""
    _check(lib().k3_pool3d_bwd_bits(_d(dx), _p(route_bits), _d(dy), _p(dy), _p(dx), _stream()), "k3_pool3d_bwd_bits")


# ------------------------------------------------------------------ transposed convolution
def upconv3d_packed_bytes(cin, cout, dtype):
    out = ctypes.c_size_t(0)
    _check(lib().k3_upconv3d_packed_bytes(ctypes.c_int64(cin), ctypes.c_int64(cout), ctypes.c_int(dtype),
                                          ctypes.byref(out)), "k3_upconv3d_packed_bytes")
    return out.value


def upconv3d_pack_weights(w, packed):
    cin, cout = w.shape[3], w.shape[4]
    nbytes = 0 if packed is None else packed.numel() * packed.element_size()
    _check(lib().k3_upconv3d_pack_weights(_p(w), ctypes.c_int64(cin), ctypes.c_int64(cout),
                                          ctypes.c_int(_dtype_code(w)), _p(packed), ctypes.c_size_t(nbytes), _stream()),
           "k3_upconv3d_pack_weights")


def upconv3d_fwd(x, w, packed, bias, y):
    _check(lib().k3_upconv3d_fwd(_d(x), _p(x), _p(w), _p(packed), _p(bias), _d(y), _p(y), _stream()), "k3_upconv3d_fwd")


def upconv3d_bwd_data(dy, w, packed, dx, dx_mask=None):
    _check(lib().k3_upconv3d_bwd_data(_d(dy), _p(dy), _p(w), _p(packed), _d(dx), _p(dx), _p(dx_mask), _stream()),
           "k3_upconv3d_bwd_data")


def upconv3d_bwd_weight_workspace_bytes(x, dy):
    out = ctypes.c_size_t(0)
    _check(lib().k3_upconv3d_bwd_weight_workspace_bytes(_d(x), _d(dy), ctypes.byref(out)),
           "k3_upconv3d_bwd_weight_workspace_bytes")
    return out.value


def upconv3d_bwd_weight(x, dy, dW, db, ws):
    _check(lib().k3_upconv3d_bwd_weight(_d(x), _p(x), _d(dy), _p(dy), _p(dW), _p(db), _p(ws),
                                        ctypes.c_size_t(ws.numel() * ws.element_size()), _stream()),
           "k3_upconv3d_bwd_weight")


# ------------------------------------------------------------------ head
def head_workspace_bytes(a):
    out = ctypes.c_size_t(0)
    _check(lib().k3_head_workspace_bytes(_d(a), ctypes.byref(out)), "k3_head_workspace_bytes")
    return out.value


def head_softmax_ce_fwd_bwd(a, wh, bh, labels, loss, da, dWh, dbh, logits, ws, relu_mask=False):
    _check(lib().k3_head_softmax_ce_fwd_bwd(_d(a), _p(a), _p(wh), _p(bh), _p(labels), _p(loss), _p(da),
                                            ctypes.c_int(int(relu_mask)), _p(dWh),
                                            _p(dbh), _p(logits), _p(ws),
                                            ctypes.c_size_t(ws.numel() * ws.element_size()), _stream()),
           "k3_head_softmax_ce_fwd_bwd")


def head_softmax_wce_fwd_bwd(a, wh, bh, labels, class_w, loss, da, dWh, dbh, logits, ws, relu_mask=False):
    _check(lib().k3_head_softmax_wce_fwd_bwd(_d(a), _p(a), _p(wh), _p(bh), _p(labels), _p(class_w), _p(loss), _p(da),
                                             ctypes.c_int(int(relu_mask)), _p(dWh), _p(dbh), _p(logits), _p(ws),
                                             ctypes.c_size_t(ws.numel() * ws.element_size()), _stream()),
           "k3_head_softmax_wce_fwd_bwd")


def head_classify(a, wh, bh, classes, logits=None):
    _check(lib().k3_head_classify(_d(a), _p(a), _p(wh), _p(bh), _p(classes), _p(logits), _stream()), "k3_head_classify")


def upsample3d_fwd(x, y):
    _check(lib().k3_upsample3d_fwd(_d(x), _p(x), _d(y), _p(y), _stream()), "k3_upsample3d_fwd")


def upsample3d_bwd(dy, dx, x_mask=None):
    _check(lib().k3_upsample3d_bwd(_d(dy), _p(dy), _p(x_mask), _d(dx), _p(dx), _stream()), "k3_upsample3d_bwd")


def dice_coefficients(classes, labels, counts, dice=None):
    """classes, labels: uint8 tensors of equal size; counts: int64[9] device tensor; dice: float32[3] or None."""
    n = classes.numel()
    assert labels.numel() == n and counts.numel() == 9 and counts.element_size() == 8
    _check(lib().k3_dice_coefficients(_p(classes), _p(labels), ctypes.c_int64(n), _p(counts), _p(dice), _stream()),
           "k3_dice_coefficients")


def sgd_momentum_step(w, v, g, lr, momentum=0.0, weight_decay=0.0, w_bf16=None):
    n = w.numel()
    assert v.numel() == n and g.numel() == n and (w_bf16 is None or w_bf16.numel() == n)
    _check(lib().k3_sgd_momentum_step(ctypes.c_int64(n), _p(w), _p(v), _p(g), ctypes.c_float(lr),
                                      ctypes.c_float(momentum), ctypes.c_float(weight_decay),
                                      _p(w_bf16) if w_bf16 is not None else None, _stream()),
           "k3_sgd_momentum_step")


# ------------------------------------------------------------------ measurement aids
def probe_mfma_bf16(iters, blocks, sink):
    """Launches the register-resident MFMA loop; returns the FLOPs of the launch."""
    fl = ctypes.c_double(0.0)
    _check(lib().k3_probe_mfma_bf16(ctypes.c_int64(iters), ctypes.c_int(blocks), _p(sink), ctypes.byref(fl), _stream()),
           "k3_probe_mfma_bf16")
    return fl.value


def probe_copy(src, dst, blocks):
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().k3_probe_copy(_p(src), _p(dst), ctypes.c_size_t(nbytes), ctypes.c_int(blocks), _stream()), "k3_probe_copy")


# ------------------------------------------------------------------ LMS swap engine
def lms_create(device_budget_bytes=0):
    ctx = ctypes.c_void_p(0)
    _check(lib().k3_lms_create(ctypes.c_uint64(device_budget_bytes), ctypes.byref(ctx)), "k3_lms_create")
    return ctx


def lms_destroy(ctx):
    _check(lib().k3_lms_destroy(ctx), "k3_lms_destroy")


def lms_host_alloc(nbytes):
    ptr = ctypes.c_void_p(0)
    _check(lib().k3_lms_host_alloc(ctypes.c_size_t(nbytes), ctypes.byref(ptr)), "k3_lms_host_alloc")
    return ptr.value


def lms_host_free(ptr):
    _check(lib().k3_lms_host_free(ctypes.c_void_p(ptr)), "k3_lms_host_free")


def lms_account_alloc(ctx, nbytes):
    _check(lib().k3_lms_account_alloc(ctx, ctypes.c_uint64(nbytes)), "k3_lms_account_alloc")


def lms_account_free(ctx, nbytes):
    _check(lib().k3_lms_account_free(ctx, ctypes.c_uint64(nbytes)), "k3_lms_account_free")


def lms_swap_out(ctx, dev_ptr, nbytes, host_ptr, compute_stream=None):
    h = ctypes.c_int(-1)
    s = _stream() if compute_stream is None else ctypes.c_void_p(compute_stream)
    _check(lib().k3_lms_swap_out(ctx, ctypes.c_void_p(dev_ptr), ctypes.c_size_t(nbytes), ctypes.c_void_p(host_ptr), s,
                                 ctypes.byref(h)), "k3_lms_swap_out")
    return h.value


def lms_swap_out_done(ctx, handle):
    done = ctypes.c_int(0)
    _check(lib().k3_lms_swap_out_done(ctx, ctypes.c_int(handle), ctypes.byref(done)), "k3_lms_swap_out_done")
    return bool(done.value)


def lms_release_after(ctx, handle, stream=None):
    s = _stream() if stream is None else ctypes.c_void_p(stream)
    _check(lib().k3_lms_release_after(ctx, ctypes.c_int(handle), s), "k3_lms_release_after")


def lms_prefetch_in(ctx, handle, dev_ptr, consumer_stream=None):
    s = _stream() if consumer_stream is None else ctypes.c_void_p(consumer_stream)
    _check(lib().k3_lms_prefetch_in(ctx, ctypes.c_int(handle), ctypes.c_void_p(dev_ptr), s), "k3_lms_prefetch_in")


def lms_prefetch_start(ctx, handle, dev_ptr, block_stream=None):
    st = _stream() if block_stream is None else ctypes.c_void_p(block_stream)
    _check(lib().k3_lms_prefetch_start(ctx, int(handle), ctypes.c_void_p(dev_ptr), st), "k3_lms_prefetch_start")


def lms_evict(ctx, handle, stream=None):
    st = _stream() if stream is None else ctypes.c_void_p(stream)
    _check(lib().k3_lms_evict(ctx, int(handle), st), "k3_lms_evict")


def lms_wait_in(ctx, handle, stream=None):
    s = _stream() if stream is None else ctypes.c_void_p(stream)
    _check(lib().k3_lms_wait_in(ctx, ctypes.c_int(handle), s), "k3_lms_wait_in")


def lms_release(ctx, handle):
    _check(lib().k3_lms_release(ctx, ctypes.c_int(handle)), "k3_lms_release")


def lms_sync(ctx):
    _check(lib().k3_lms_sync(ctx), "k3_lms_sync")


def lms_get_stats(ctx):
    st = LmsStats()
    _check(lib().k3_lms_get_stats(ctx, ctypes.byref(st)), "k3_lms_get_stats")
    return {k: getattr(st, k) for k, _ in LmsStats._fields_}


def lms_set_copy_timing(ctx, on):
    _check(lib().k3_lms_set_copy_timing(ctx, ctypes.c_int(1 if on else 0)), "k3_lms_set_copy_timing")


def lms_set_poison(ctx, on):
    _check(lib().k3_lms_set_poison(ctx, ctypes.c_int(1 if on else 0)), "k3_lms_set_poison")


def lms_copy_busy_ms(ctx):
    """(device-to-host, host-to-device) busy milliseconds of the copy streams since the context was created."""
    a, b = ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib().k3_lms_copy_busy_ms(ctx, ctypes.byref(a), ctypes.byref(b)), "k3_lms_copy_busy_ms")
    return a.value, b.value


def lms_handle_state(ctx, handle):
    s = ctypes.c_int(-1)
    _check(lib().k3_lms_handle_state(ctx, ctypes.c_int(handle), ctypes.byref(s)), "k3_lms_handle_state")
    return s.value
