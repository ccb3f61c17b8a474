"""CPU oracle (fp64 direct loops) for the 3-D U-Net step operators.

TEST INFRASTRUCTURE ONLY.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product path never does.  It
shares no code with the GPU library.  The arithmetic lives in oracle.c (built
with gcc into liboracle.so by `oracle.build()`); this file only marshals numpy
arrays.  See oracle.c for the definitions and what pins them.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None

_i64 = ctypes.c_int64
_dp = ctypes.POINTER(ctypes.c_double)


def build(force=True):
    """Compile oracle.c with gcc (-O2, OpenMP over the outer loops only)."""
    src = os.path.join(_HERE, "oracle.c")
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(src):
        return _SO
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                           "-o", _SO, src, "-lm"])
    global _lib
    _lib = None
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        _lib = ctypes.CDLL(_SO)
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(_dp)


def _opt(a):
    if a is None:
        return None, None
    return _d(a)


def bf16_to_f64(bits):
    """bf16 bit patterns (uint16) -> float64, exact."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_bf16(a):
    """float64 -> nearest-even bf16 value of its float32 rounding, as float64.

    Mirrors a GPU that accumulates in fp32 and stores bf16 (storage emulation for
    chained comparisons)."""
    f = np.ascontiguousarray(a, dtype=np.float64).astype(np.float32)
    u = f.view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
    return r.view(np.float32).astype(np.float64)


def conv3d_fwd(x, w, b=None, relu=False):
    N, D, H, W, Ci = x.shape
    Co = w.shape[4]
    assert w.shape == (3, 3, 3, Ci, Co)
    x, xp = _d(x); w, wp = _d(w); b, bp = _opt(b)
    y = np.empty((N, D, H, W, Co), dtype=np.float64)
    _load().orc_conv3d_fwd(xp, wp, bp, y.ctypes.data_as(_dp), _i64(N), _i64(D), _i64(H), _i64(W),
                           _i64(Ci), _i64(Co), ctypes.c_int(int(relu)))
    return y


def conv3d_fwd_points(x, w, b, relu, pts):
    N, D, H, W, Ci = x.shape
    Co = w.shape[4]
    x, xp = _d(x); w, wp = _d(w); b, bp = _opt(b)
    pts = np.ascontiguousarray(pts, dtype=np.int64)
    out = np.empty((pts.shape[0], Co), dtype=np.float64)
    _load().orc_conv3d_fwd_points(xp, wp, bp, out.ctypes.data_as(_dp),
                                  pts.ctypes.data_as(ctypes.POINTER(_i64)), _i64(pts.shape[0]),
                                  _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co),
                                  ctypes.c_int(int(relu)))
    return out


def relu_bwd(dy, y):
    dy, dp_ = _d(dy); y, yp = _d(y)
    g = np.empty_like(dy)
    _load().orc_relu_bwd(dp_, yp, g.ctypes.data_as(_dp), _i64(dy.size))
    return g


def conv3d_bwd_data(g, w):
    N, D, H, W, Co = g.shape
    Ci = w.shape[3]
    assert w.shape == (3, 3, 3, Ci, Co)
    g, gp = _d(g); w, wp = _d(w)
    dx = np.empty((N, D, H, W, Ci), dtype=np.float64)
    _load().orc_conv3d_bwd_data(gp, wp, dx.ctypes.data_as(_dp), _i64(N), _i64(D), _i64(H), _i64(W),
                                _i64(Ci), _i64(Co))
    return dx


def conv3d_bwd_data_points(g, w, pts):
    """Backward-data at the listed voxels only: [npts, C_in].  Pinned against conv3d_bwd_data in
    tests/test_oracle_conv.py."""
    N, D, H, W, Co = g.shape
    Ci = w.shape[3]
    assert w.shape == (3, 3, 3, Ci, Co)
    g, gp = _d(g); w, wp = _d(w)
    pts = np.ascontiguousarray(pts, dtype=np.int64)
    out = np.empty((pts.shape[0], Ci), dtype=np.float64)
    _load().orc_conv3d_bwd_data_points(gp, wp, out.ctypes.data_as(_dp), pts.ctypes.data_as(ctypes.POINTER(_i64)),
                                       _i64(pts.shape[0]), _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return out


def conv3d_bwd_weight(x, g):
    N, D, H, W, Ci = x.shape
    Co = g.shape[4]
    assert g.shape[:4] == x.shape[:4]
    x, xp = _d(x); g, gp = _d(g)
    dW = np.empty((3, 3, 3, Ci, Co), dtype=np.float64)
    db = np.empty((Co,), dtype=np.float64)
    _load().orc_conv3d_bwd_weight(xp, gp, dW.ctypes.data_as(_dp), db.ctypes.data_as(_dp),
                                  _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return dW, db


def conv3d_bwd_weight_entries(x, g, entries):
    N, D, H, W, Ci = x.shape
    Co = g.shape[4]
    x, xp = _d(x); g, gp = _d(g)
    ent = np.ascontiguousarray(entries, dtype=np.int64)
    out = np.empty((ent.shape[0],), dtype=np.float64)
    _load().orc_conv3d_bwd_weight_entries(xp, gp, out.ctypes.data_as(_dp),
                                          ent.ctypes.data_as(ctypes.POINTER(_i64)), _i64(ent.shape[0]),
                                          _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return out


def pool3d_fwd(x):
    N, D, H, W, C = x.shape
    assert D % 2 == 0 and H % 2 == 0 and W % 2 == 0
    x, xp = _d(x)
    y = np.empty((N, D // 2, H // 2, W // 2, C), dtype=np.float64)
    _load().orc_pool3d_fwd(xp, y.ctypes.data_as(_dp), _i64(N), _i64(D), _i64(H), _i64(W), _i64(C))
    return y


def pool3d_bwd(x, dy):
    N, D, H, W, C = x.shape
    assert dy.shape == (N, D // 2, H // 2, W // 2, C)
    x, xp = _d(x); dy, dyp = _d(dy)
    dx = np.empty_like(x)
    _load().orc_pool3d_bwd(xp, dyp, dx.ctypes.data_as(_dp), _i64(N), _i64(D), _i64(H), _i64(W), _i64(C))
    return dx


def upconv3d_fwd(x, w, b=None):
    N, D, H, W, Ci = x.shape
    Co = w.shape[4]
    assert w.shape == (2, 2, 2, Ci, Co)
    x, xp = _d(x); w, wp = _d(w); b, bp = _opt(b)
    y = np.empty((N, 2 * D, 2 * H, 2 * W, Co), dtype=np.float64)
    _load().orc_upconv3d_fwd(xp, wp, bp, y.ctypes.data_as(_dp), _i64(N), _i64(D), _i64(H), _i64(W),
                             _i64(Ci), _i64(Co))
    return y


def upconv3d_bwd_data(dy, w):
    N, D2, H2, W2, Co = dy.shape
    Ci = w.shape[3]
    D, H, W = D2 // 2, H2 // 2, W2 // 2
    dy, dyp = _d(dy); w, wp = _d(w)
    dx = np.empty((N, D, H, W, Ci), dtype=np.float64)
    _load().orc_upconv3d_bwd_data(dyp, wp, dx.ctypes.data_as(_dp), _i64(N), _i64(D), _i64(H), _i64(W),
                                  _i64(Ci), _i64(Co))
    return dx


def upconv3d_bwd_weight(x, dy):
    N, D, H, W, Ci = x.shape
    Co = dy.shape[4]
    assert dy.shape[:4] == (N, 2 * D, 2 * H, 2 * W)
    x, xp = _d(x); dy, dyp = _d(dy)
    dW = np.empty((2, 2, 2, Ci, Co), dtype=np.float64)
    db = np.empty((Co,), dtype=np.float64)
    _load().orc_upconv3d_bwd_weight(xp, dyp, dW.ctypes.data_as(_dp), db.ctypes.data_as(_dp),
                                    _i64(N), _i64(D), _i64(H), _i64(W), _i64(Ci), _i64(Co))
    return dW, db


def head_softmax_ce(a, wh, bh, labels):
    """Returns dict(loss, logits, da, dW, db); a is [..., C], labels uint8 with a's leading shape."""
    C = a.shape[-1]
    K = wh.shape[1]
    V = a.size // C
    a_, ap = _d(a); wh, whp = _d(wh); bh, bhp = _opt(bh)
    lab = np.ascontiguousarray(labels, dtype=np.uint8).reshape(-1)
    assert lab.size == V
    loss = ctypes.c_double(0.0)
    logits = np.empty((V, K), dtype=np.float64)
    da = np.empty_like(a_)
    dW = np.empty((C, K), dtype=np.float64)
    db = np.empty((K,), dtype=np.float64)
    _load().orc_head_softmax_ce(ap, whp, bhp, lab.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)),
                                ctypes.byref(loss), logits.ctypes.data_as(_dp), da.ctypes.data_as(_dp),
                                dW.ctypes.data_as(_dp), db.ctypes.data_as(_dp), _i64(V), _i64(C), _i64(K))
    return {"loss": loss.value, "logits": logits.reshape(a.shape[:-1] + (K,)), "da": da, "dW": dW, "db": db}


def sgd_momentum_step(w, v, g, lr, momentum=0.0, weight_decay=0.0):
    """One step of stochastic gradient descent (the weight-update algorithm of section 1) with
    the textbook momentum and weight-decay terms, fp64, out of place:
        v' = momentum * v + (g + weight_decay * w);   w' = w - lr * v'.
    momentum = weight_decay = 0 is plain SGD, w' = w - lr * g.  Returns (w', v').
    Pinned in tests/test_oracle_sgd.py by closed forms (geometric momentum sum under a constant
    gradient, the exact contraction factor on a quadratic) and a two-step hand computation."""
    w = np.asarray(w, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    v2 = momentum * v + (g + weight_decay * w)
    return w - lr * v2, v2


def relu_bits(y):
    """Bit mask of a stored ReLU output: one uint16 word per 16 consecutive channels of a voxel,
    bit i of word j set iff y[..., 16 j + i] > 0 (the derivative of ReLU as section 4.1's layers
    use it in the backward pass, one bit per element).  y: [..., C] with C a multiple of 16;
    returns [..., C // 16] uint16.  Pinned in tests/test_oracle_conv.py against relu_bwd."""
    y = np.asarray(y, dtype=np.float64)
    C = y.shape[-1]
    assert C % 16 == 0
    pos = (y > 0).reshape(y.shape[:-1] + (C // 16, 16))
    out = np.zeros(pos.shape[:-1], dtype=np.uint32)
    for i in range(16):
        out |= pos[..., i].astype(np.uint32) << i
    return out.astype(np.uint16)


def apply_relu_bits(dy, bits):
    """dy with every element zeroed whose bit is clear (the inverse reading of relu_bits)."""
    dy = np.asarray(dy, dtype=np.float64)
    C = dy.shape[-1]
    keep = np.zeros(dy.shape, dtype=bool).reshape(dy.shape[:-1] + (C // 16, 16))
    b = np.asarray(bits).astype(np.uint32)
    for i in range(16):
        keep[..., i] = ((b >> i) & 1).astype(bool)
    return dy * keep.reshape(dy.shape)


def _windows(a):
    """[N, D, H, W, C] -> [N, D/2, H/2, W/2, 8, C]: the eight elements of each 2x2x2 window in the
    order (i, j, k), i the depth offset."""
    N, D, H, W, C = a.shape
    return a.reshape(N, D // 2, 2, H // 2, 2, W // 2, 2, C).transpose(0, 1, 3, 5, 2, 4, 6, 7).reshape(
        N, D // 2, H // 2, W // 2, 8, C)


def _unwindows(a):
    N, Do, Ho, Wo, _, C = a.shape
    return a.reshape(N, Do, Ho, Wo, 2, 2, 2, C).transpose(0, 1, 4, 2, 5, 3, 6, 7).reshape(N, 2 * Do, 2 * Ho, 2 * Wo, C)


def pool3d_route_bits(x):
    """Routing of the 2x2x2 max-pool's backward pass (section 4.1) as one bit per element of x, in
    the layout of relu_bits: the bit is set iff the element is the first maximum of its window
    (order i, j, k) and > 0, i.e. where the pooled gradient arrives and passes the ReLU that
    produced x.  Pinned in tests/test_oracle_pool_upconv_head.py against pool3d_bwd + relu_bwd."""
    x = np.asarray(x, dtype=np.float64)
    xw = _windows(x)
    first = np.argmax(xw, axis=4)                       # numpy: the first of equal maxima
    hit = np.arange(8).reshape(1, 1, 1, 1, 8, 1) == first[:, :, :, :, None, :]
    hit &= (np.max(xw, axis=4) > 0)[:, :, :, :, None, :]
    return relu_bits(_unwindows(hit).astype(np.float64))


def pool3d_bwd_bits(bits, dy):
    """dx[n, 2d+i, 2h+j, 2w+k, c] = dy[n, d, h, w, c] where the element's routing bit is set, else 0."""
    dy = np.asarray(dy, dtype=np.float64)
    spread = _unwindows(np.repeat(dy[:, :, :, :, None, :], 8, axis=4))
    return apply_relu_bits(spread, bits)

