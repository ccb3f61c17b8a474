"""GPU parity of the 3x3x3 convolution passes against the fp64 oracle, through the C-ABI."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu

# (N, D, H, W, c1, c2, cout, dtype): spans direct and MFMA paths, several tiles, ragged tails
FWD_CASES = [
    (1, 16, 16, 16, 4, 0, 8, "f32"),       # workload config 1
    (2, 5, 6, 7, 3, 2, 5, "f32"),          # odd sizes, two sources, direct
    (1, 9, 10, 11, 1, 0, 32, "bf16"),      # single-channel first layer kernels
    (2, 6, 5, 7, 1, 0, 64, "bf16"),        # first layer, two samples (borders between samples)
    (2, 9, 11, 19, 1, 0, 128, "bf16"),     # first layer of the encoder/decoder model: 128 channels (two 64-channel wgrad passes)
    (1, 5, 6, 7, 3, 2, 5, "bf16"),         # direct kernels in bf16
    (1, 16, 16, 16, 32, 0, 32, "bf16"),    # MFMA, MB=1, 8 tiles
    (1, 12, 20, 9, 32, 0, 64, "bf16"),     # MFMA, MB=2, ragged tiles
    (2, 8, 8, 16, 64, 0, 32, "bf16"),      # several K chunks
    (1, 10, 8, 8, 32, 32, 32, "bf16"),     # two sources (decoder conv1)
    (1, 4, 4, 4, 128, 0, 128, "bf16"),     # volume smaller than a tile, 2 channel groups
    (1, 2, 2, 2, 64, 64, 64, "bf16"),      # bottleneck-like
    (1, 7, 20, 35, 32, 0, 64, "bf16"),     # several 16x16 columns with ragged edges, odd depth
    (2, 3, 17, 16, 64, 32, 32, "bf16"),    # two sources, one row past a column, two samples
    (1, 40, 16, 18, 32, 0, 32, "bf16"),    # long depth run
    (3, 36, 44, 50, 32, 0, 32, "bf16"),    # plane-streaming kernel (32 output channels, a tile per CU and more): ragged on every axis
    (2, 32, 40, 48, 32, 32, 96, "bf16"),   # plane-streaming forward: two sources, four chunks, three output blocks
    (2, 32, 40, 48, 32, 64, 32, "bf16"),   # plane-streaming backward-data into two destinations (three blocks)
    (3, 36, 44, 50, 64, 32, 32, "bf16"),   # sources of unequal width: the pipelined kernel with one block per workgroup, 8x8x16 tiles
]


def _mk(case, seed0):
    N, D, H, W, c1, c2, co, dt = case
    x = synth.activations(seed0, (N, D, H, W, c1), dt)
    x2 = synth.activations(seed0 + 1, (N, D, H, W, c2), dt) if c2 else None
    w = synth.conv_weights(seed0 + 2, c1 + c2, co, dt)
    b = (synth.normal(synth.SEED, seed0 + 3, (co,), np.float64) * 0.5).astype(np.float32)
    return x, x2, w, b


@pytest.mark.parametrize("case", FWD_CASES, ids=lambda c: "x".join(map(str, c)))
@pytest.mark.parametrize("relu", [0, 1])
def test_conv_fwd(orc, case, relu):
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, rel_l2, packed_for, TOL
    N, D, H, W, c1, c2, co, dt = case
    x, x2, w, b = _mk(case, 10)
    xd, wd, bd = to_dev(x, dt), to_dev(w, dt), torch.from_numpy(b).cuda()
    x2d = to_dev(x2, dt) if c2 else None
    y = empty((N, D, H, W, co), dt)
    y.fill_(float("nan"))
    k3.conv3d_fwd(xd, wd, packed_for(wd), bd, relu, y, x2=x2d)
    torch.cuda.synchronize()
    xin = x if not c2 else np.concatenate([x, x2], axis=-1)
    ref = orc.conv3d_fwd(xin.astype(np.float64), w.astype(np.float64), b.astype(np.float64), relu=bool(relu))
    got = to_f64(y)
    assert np.isfinite(got).all()
    err = rel_l2(got, ref)
    assert err < TOL[dt], err
    if dt == "bf16":
        # one bf16 rounding of an fp32 accumulation: anything above 4e-3 means a structural bug
        assert err < 4e-3, err
        assert rel_l2(got, orc.round_bf16(ref)) < 2e-3


@pytest.mark.parametrize("case", FWD_CASES, ids=lambda c: "x".join(map(str, c)))
@pytest.mark.parametrize("masked", [0, 1, 2])
def test_conv_bwd_data(orc, case, masked):
    """masked = 1: ReLU mask on the incoming gradient; 2: mask applied to the produced gradient."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, rel_l2, packed_for, TOL
    N, D, H, W, c1, c2, co, dt = case
    _, _, w, _ = _mk(case, 20)
    dy = synth.activations(24, (N, D, H, W, co), dt)
    ym = synth.activations(25, (N, D, H, W, co), dt)
    ym[ym < 0.3] = 0.0       # plenty of exact zeros and negatives, like a stored ReLU output
    wd, dyd, ymd = to_dev(w, dt), to_dev(dy, dt), to_dev(ym, dt)
    dx = empty((N, D, H, W, c1), dt)
    dx2 = empty((N, D, H, W, c2), dt) if c2 else None
    om = synth.activations(26, (N, D, H, W, c1), dt)
    om[om < 0.2] = 0.0
    omd = to_dev(om, dt)
    k3.conv3d_bwd_data(dyd, ymd if masked == 1 else None, wd, packed_for(wd), dx, dx2=dx2,
                       dx_mask=omd if masked == 2 else None)
    torch.cuda.synchronize()
    g = dy.astype(np.float64)
    if masked == 1:
        g = orc.relu_bwd(g, ym.astype(np.float64))
    ref = orc.conv3d_bwd_data(g, w.astype(np.float64))
    if masked == 2:
        ref[..., :c1] = orc.relu_bwd(ref[..., :c1], om.astype(np.float64))
    got = to_f64(dx) if not c2 else np.concatenate([to_f64(dx), to_f64(dx2)], axis=-1)
    err = rel_l2(got, ref)
    assert err < TOL[dt], err
    if dt == "bf16":
        assert err < 4e-3, err


@pytest.mark.parametrize("case", FWD_CASES, ids=lambda c: "x".join(map(str, c)))
@pytest.mark.parametrize("masked", [0, 1])
def test_conv_bwd_weight(orc, case, masked):
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, rel_l2, TOL
    N, D, H, W, c1, c2, co, dt = case
    x, x2, _, _ = _mk(case, 30)
    dy = synth.activations(34, (N, D, H, W, co), dt)
    ym = synth.activations(35, (N, D, H, W, co), dt)
    ym[ym < 0.3] = 0.0
    xd, dyd, ymd = to_dev(x, dt), to_dev(dy, dt), to_dev(ym, dt)
    x2d = to_dev(x2, dt) if c2 else None
    dW = torch.full((3, 3, 3, c1 + c2, co), float("nan"), device="cuda")
    db = torch.full((co,), float("nan"), device="cuda")
    ws = torch.empty(max(1, k3.conv3d_bwd_weight_workspace_bytes(xd, dyd, x2=x2d)), device="cuda", dtype=torch.uint8)
    k3.conv3d_bwd_weight(xd, dyd, ymd if masked else None, dW, db, ws, x2=x2d)
    torch.cuda.synchronize()
    g = dy.astype(np.float64)
    if masked:
        g = orc.relu_bwd(g, ym.astype(np.float64))
    xin = x if not c2 else np.concatenate([x, x2], axis=-1)
    rW, rb = orc.conv3d_bwd_weight(xin.astype(np.float64), g)
    # fp32 accumulation of exact products: far inside either tolerance
    assert rel_l2(to_f64(dW), rW) < 1e-5
    assert rel_l2(to_f64(db), rb) < 1e-5
    # run-to-run identical
    dW2 = torch.empty_like(dW)
    k3.conv3d_bwd_weight(xd, dyd, ymd if masked else None, dW2, db, ws, x2=x2d)
    torch.cuda.synchronize()
    assert torch.equal(dW, dW2)


def test_identity_kernel_is_bit_exact_bf16():
    """Centre-tap identity weights reproduce the bf16 input bit for bit (MFMA path)."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, empty, packed_for
    C = 32
    x = to_dev(synth.activations(40, (1, 9, 8, 10, C), "bf16"), "bf16")
    w = np.zeros((3, 3, 3, C, C), dtype=np.float32)
    w[1, 1, 1] = np.eye(C)
    wd = to_dev(w, "bf16")
    y = empty(x.shape, "bf16")
    k3.conv3d_fwd(x, wd, packed_for(wd), None, 0, y)
    torch.cuda.synchronize()
    assert torch.equal(x.view(torch.int16), y.view(torch.int16))


def test_shift_kernels_bf16_mfma():
    """One-hot kernels at each tap shift the input exactly, zero filled at every face."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, packed_for
    C = 32
    xs = synth.activations(41, (1, 9, 10, 11, C), "bf16")
    x = to_dev(xs, "bf16")
    for tap in (0, 2, 6, 8, 13, 18, 20, 24, 26, 4, 10, 22):
        kd, kh, kw = tap // 9, (tap // 3) % 3, tap % 3
        w = np.zeros((3, 3, 3, C, C), dtype=np.float32)
        w[kd, kh, kw] = np.eye(C)
        wd = to_dev(w, "bf16")
        y = empty(x.shape, "bf16")
        k3.conv3d_fwd(x, wd, packed_for(wd), None, 0, y)
        torch.cuda.synchronize()
        exp = np.zeros_like(xs)
        D, H, W = xs.shape[1:4]

        def rng_(s, n):
            return slice(max(0, -s), n - max(0, s)), slice(max(0, s), n - max(0, -s))
        (od, id_), (oh, ih), (ow, iw) = rng_(kd - 1, D), rng_(kh - 1, H), rng_(kw - 1, W)
        exp[:, od, oh, ow] = xs[:, id_, ih, iw]
        assert np.array_equal(to_f64(y), exp.astype(np.float64)), tap


def test_error_codes():
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import empty
    x = empty((1, 4, 4, 4, 32), "bf16")
    y = empty((1, 4, 4, 5, 32), "bf16")
    w = empty((3, 3, 3, 32, 32), "bf16")
    with pytest.raises(k3.K3Error) as e:
        k3.conv3d_fwd(x, w, None, None, 0, y)
    assert e.value.status == k3.E_SHAPE
    y = empty((1, 4, 4, 4, 32), "bf16")
    with pytest.raises(k3.K3Error) as e:
        k3.conv3d_fwd(x, w, None, None, 0, y)      # MFMA shape without packed weights
    assert e.value.status == k3.E_BADARG
    dW = torch.empty((3, 3, 3, 32, 32), device="cuda")
    ws = torch.empty(16, device="cuda", dtype=torch.uint8)
    with pytest.raises(k3.K3Error) as e:
        k3.conv3d_bwd_weight(x, y, None, dW, None, ws)
    assert e.value.status == k3.E_WORKSPACE


BITS_CASES = [
    (1, 16, 16, 16, 32, 0, 32),      # pipelined kernel, one output block per workgroup, 4x8x8 tiles
    (1, 12, 20, 35, 32, 0, 64),      # ragged tiles, two blocks per workgroup
    (2, 9, 10, 11, 1, 0, 64),        # first layer (im2col kernel writes the bits)
    (1, 6, 7, 9, 1, 0, 48),          # first layer, thread-per-channel kernel + generic bits pass
    (1, 10, 8, 8, 32, 32, 32),       # two sources forward / two destinations backward (mask on the first)
    (1, 4, 4, 4, 128, 0, 128),       # small volume: first MFMA kernel + generic passes
    (1, 5, 6, 7, 3, 2, 16),          # direct kernels
    (3, 36, 44, 50, 32, 0, 32),      # plane-streaming kernel writes / reads the bits, ragged tiles, two tiles per workgroup
    (2, 32, 40, 48, 32, 64, 32),     # plane-streaming backward-data: mask on the first of two destinations
]


@pytest.mark.parametrize("N,D,H,W,c1,c2,co", BITS_CASES)
def test_relu_bit_masks(orc, N, D, H, W, c1, c2, co):
    """The forward pass's bit mask is exactly the oracle's mask of the stored output, and
    backward-data with the mask given as bits is bit-identical to backward-data with the mask
    given as the tensor (and so inherits its parity with the oracle)."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, packed_for
    cin = c1 + c2
    x = synth.activations(20, (N, D, H, W, cin), "bf16")
    w = synth.conv_weights(21, cin, co, "bf16")
    b = (synth.normal(synth.SEED, 22, (co,), np.float64) * 0.3).astype(np.float32)
    xd, wd, bd = to_dev(x, "bf16"), to_dev(w, "bf16"), torch.from_numpy(b).cuda()
    x1 = xd[..., :c1].contiguous()
    x2 = xd[..., c1:].contiguous() if c2 else None
    pk = packed_for(wd)
    y0, y1 = empty((N, D, H, W, co), "bf16"), empty((N, D, H, W, co), "bf16")
    k3.conv3d_fwd(x1, wd, pk, bd, 1, y0, x2=x2)
    bits = torch.full((N, D, H, W, co // 16), -1, device="cuda", dtype=torch.int16)
    assert k3.relu_bits_bytes(y1) == bits.numel() * 2
    k3.conv3d_fwd_bits(x1, wd, pk, bd, 1, y1, bits, x2=x2)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    assert np.array_equal(bits.cpu().numpy().view(np.uint16), orc.relu_bits(to_f64(y1)))
    # backward through a layer whose first input is a stored ReLU output with the shape of x1
    if c1 % 16 == 0:
        m = torch.relu(x1)
        mbits = torch.from_numpy(orc.relu_bits(to_f64(m)).view(np.int16)).cuda()
        g = to_dev(synth.activations(23, (N, D, H, W, co), "bf16"), "bf16")
        dxa, dxb = empty(x1.shape, "bf16"), empty(x1.shape, "bf16")
        dx2a = empty(x2.shape, "bf16") if c2 else None
        dx2b = empty(x2.shape, "bf16") if c2 else None
        k3.conv3d_bwd_data(g, None, wd, pk, dxa, dx2=dx2a, dx_mask=m)
        k3.conv3d_bwd_data_bits(g, None, wd, pk, dxb, mbits, dx2=dx2b)
        torch.cuda.synchronize()
        assert torch.equal(dxa, dxb)
        assert c2 == 0 or torch.equal(dx2a, dx2b)
        assert np.array_equal(to_f64(dxb), orc.apply_relu_bits(to_f64(dxb), mbits.cpu().numpy().view(np.uint16)))


POOL_CASES = [
    (3, 36, 44, 50, 32, 0, 32, "bf16", 1),    # plane-streaming kernel pools itself: ragged tiles, two tiles per workgroup
    (2, 32, 40, 48, 32, 32, 96, "bf16", 1),   # ... two sources, three output blocks
    (3, 36, 44, 50, 32, 0, 32, "bf16", 0),    # no ReLU: the pooling kernel runs behind the convolution
    (1, 16, 16, 16, 32, 0, 32, "bf16", 1),    # small tiles: second pass
    (1, 12, 20, 36, 32, 0, 64, "bf16", 1),    # two blocks per workgroup: second pass
    (1, 16, 16, 16, 4, 0, 8, "f32", 1),       # direct kernels
]


@pytest.mark.parametrize("case", POOL_CASES, ids=lambda c: "x".join(map(str, c)))
def test_conv_fwd_pool(orc, case):
    """The fused call writes exactly what the convolution followed by the pooling call writes, and
    the pooled tensor is the oracle's pool of the stored output."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, packed_for
    N, D, H, W, c1, c2, co, dt, relu = case
    x, x2, w, b = _mk(case[:8], 40)
    xd, wd, bd = to_dev(x, dt), to_dev(w, dt), torch.from_numpy(b).cuda()
    x2d = to_dev(x2, dt) if c2 else None
    pk = packed_for(wd)
    y0, y1 = empty((N, D, H, W, co), dt), empty((N, D, H, W, co), dt)
    p0, p1 = empty((N, D // 2, H // 2, W // 2, co), dt), empty((N, D // 2, H // 2, W // 2, co), dt)
    y1.fill_(float("nan")); p1.fill_(float("nan"))
    k3.conv3d_fwd(xd, wd, pk, bd, relu, y0, x2=x2d)
    k3.pool3d_fwd(y0, p0)
    k3.conv3d_fwd_pool(xd, wd, pk, bd, relu, y1, p1, x2=x2d)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    assert torch.equal(p0, p1)
    assert np.array_equal(to_f64(p1), orc.pool3d_fwd(to_f64(y1)))


def test_conv_fwd_pool_rejects_odd_sizes():
    import torch
    from paper_1811_12174_amd import k3
    x = torch.zeros((1, 6, 7, 8, 32), device="cuda", dtype=torch.bfloat16)
    w = torch.zeros((3, 3, 3, 32, 32), device="cuda", dtype=torch.bfloat16)
    from gpu_util import packed_for
    y = torch.empty_like(x)
    p = torch.empty((1, 3, 3, 4, 32), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(k3.K3Error) as e:
        k3.conv3d_fwd_pool(x, w, packed_for(w), None, 1, y, p)
    assert e.value.status == k3.E_SHAPE


# ------------------------------------------------------------------ exact arithmetic: structure pinned with zero tolerance
# (N, D, H, W, c1, c2, cout): one shape per MFMA kernel variant, bench-sized where that selects the kernel
EXACT_CASES = [
    (1, 64, 64, 64, 32, 0, 32),     # plane-streaming kernel, the benchmark's layer (K-split weight gradient)
    (1, 40, 36, 50, 64, 0, 64),     # pipelined kernel, two output blocks, ragged 8x8x16 tiles
    (2, 20, 24, 24, 32, 32, 64),    # two sources / two destinations
    (1, 16, 16, 16, 128, 0, 128),   # 4x8x8 tiles
    (1, 12, 20, 9, 32, 0, 64),      # small-volume kernel
    (1, 24, 20, 36, 1, 0, 64),      # single-channel first layer
]


@pytest.mark.parametrize("case", EXACT_CASES, ids=lambda c: "x".join(map(str, c)))
def test_integer_valued_tensors_give_exact_results(orc, case):
    """With inputs in {-1, 0, 1} and sparse weights in {-1, 0, 1} (at most 200 non-zero weights
    per output channel, per input channel for backward-data) every product and every partial sum is
    a small integer: exact in bf16 operands, exact in fp32 accumulation in any order, and the
    result (|y| <= 200 < 2^8) is exact in the bf16 output.  The kernels must therefore match the
    fp64 oracle bit for bit -- at every voxel, corner, edge and tile border, for every tap at once.
    A bf16-rounded output with ordinary inputs hides structural slips smaller than its rounding
    (about 2e-3); here nothing is rounded, so there is nothing to hide behind."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, packed_for
    N, D, H, W, c1, c2, co = case
    cin = c1 + c2
    rng = np.random.default_rng(1811 + cin + co + D)
    x = rng.integers(-1, 2, size=(N, D, H, W, cin)).astype(np.float32)
    g = rng.integers(-1, 2, size=(N, D, H, W, co)).astype(np.float32)
    w = np.zeros((27, cin, co), dtype=np.float32)
    # at most 200 non-zeros in every column (the 27 * cin weights of one output channel) and, where
    # backward-data runs, in every row group (the 27 * co weights of one input channel): up to 100
    # per column placed at random, fewer when co > cin so that a row group gets 100 on average
    # and never more than 200 (checked below)
    per_col = min(27 * cin, 100 if (co <= cin or c1 == 1) else 100 * cin // co)
    for o in range(co):
        idx = rng.choice(27 * cin, size=per_col, replace=False)
        w.reshape(27 * cin, co)[idx, o] = rng.choice([-1.0, 1.0], size=idx.size)
    assert np.abs(w).sum(axis=(0, 1)).max() <= 200 and (c1 == 1 or np.abs(w).sum(axis=(0, 2)).max() <= 200)
    w = w.reshape(3, 3, 3, cin, co)
    b = rng.integers(-3, 4, size=(co,)).astype(np.float32)
    xd, gd, wd, bd = to_dev(x, "bf16"), to_dev(g, "bf16"), to_dev(w, "bf16"), torch.from_numpy(b).cuda()
    x1 = xd[..., :c1].contiguous()
    x2 = xd[..., c1:].contiguous() if c2 else None
    pk = packed_for(wd)
    X, G, Wt = x.astype(np.float64), g.astype(np.float64), w.astype(np.float64)

    y = empty((N, D, H, W, co), "bf16")
    bits = torch.empty((N, D, H, W, co // 16), device="cuda", dtype=torch.int16)
    k3.conv3d_fwd_bits(x1, wd, pk, bd, 1, y, bits, x2=x2)
    torch.cuda.synchronize()
    ref = orc.conv3d_fwd(X, Wt, b.astype(np.float64), relu=True)
    assert np.array_equal(to_f64(y), ref)
    assert np.array_equal(bits.cpu().numpy().view(np.uint16), orc.relu_bits(ref))

    if c1 > 1:
        dx1 = empty((N, D, H, W, c1), "bf16")
        dx2 = empty((N, D, H, W, c2), "bf16") if c2 else None
        k3.conv3d_bwd_data(gd, None, wd, pk, dx1, dx2=dx2, dx_mask=x1)
        torch.cuda.synchronize()
        ref = orc.conv3d_bwd_data(G, Wt)
        ref[..., :c1] *= X[..., :c1] > 0
        got = to_f64(dx1) if not c2 else np.concatenate([to_f64(dx1), to_f64(dx2)], axis=-1)
        assert np.array_equal(got, ref)

    dW, db = torch.empty((3, 3, 3, cin, co), device="cuda"), torch.empty(co, device="cuda")
    ws = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(x1, gd, x2=x2), device="cuda", dtype=torch.uint8)
    k3.conv3d_bwd_weight(x1, gd, None, dW, db, ws, x2=x2)
    torch.cuda.synchronize()
    rW, rb = orc.conv3d_bwd_weight(X, G)      # integer sums below 2^24: exact in fp32
    assert np.array_equal(to_f64(dW), rW)
    assert np.array_equal(to_f64(db), rb)
