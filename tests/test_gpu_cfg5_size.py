"""GPU parity at workload config 5's size: tensors of 4 x 320^3 voxels x 64 channels (8.4 Gi
elements, 16.8 GB) need 64-bit element offsets in every kernel that touches them.

Every kernel of the base-64 U-Net step that sees such a tensor runs here at that size: the
single-source and the two-source 3x3x3 convolution (forward, masked backward-data into one and
into two destinations, backward-weight), the ReLU bit-mask writer and reader, the single-channel
first layer (forward, backward-weight), max-pool forward / backward, the transposed convolution
(forward, backward-data, backward-weight) and the head.

The oracle cannot run at that size in full, so:
  * local results (convolution, pooling, transposed convolution, head gradient) are checked on
    crops cut out on the device with their halo, placed at the first voxels, at the last voxels
    (element offsets beyond 2^33) and in between;
  * global sums (weight gradients, loss) are checked in two steps: the oracle sums ONE sample,
    which the GPU reproduces when run on that sample alone (its data lies beyond element 2^32 of
    the tensor), and the full-size GPU result must equal the sum of the four single-sample GPU
    results (the mean, for the loss).
Inputs are seeded N(0,1) tensors generated on the device sample by sample (a host generator
would need minutes for 8.4 Gi values); the oracle reads the very same bytes back.
"""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu

N, S, C = 4, 320, 64
E = 10   # crop edge
# Bound between the full-size weight gradient and the sum of the four single-sample ones.  Each
# entry is a sum of 1.3e8 products of N(0,1) values accumulated in fp32 (as the workload fixes):
# partial sums of magnitude ~1e3 carry a rounding random walk of ~1e-2 each, ~0.1 over the 128
# partials of an entry whose value is ~1e4, i.e. ~8e-6 relative for either side of the comparison
# (measured between the two: 1.1e-5).  Single-sample results keep the 1e-5 bound against the oracle.
TOL_SUM = 3e-5
CORNERS = [(0, 0, 0, 0), (N - 1, S - E, S - E, S - E), (N - 1, 0, S - E, 0), (2, 155, 3, 301), (3, S - E, 160, 8),
           (1, 64, 128, 256), (N - 1, S - E, S - E, 0)]


def rel(got, ref):
    from gpu_util import rel_l2
    return rel_l2(got, ref, depth=2)


def f64(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def halo_crop(t, n, d0, h0, w0, edge=E, size=S):
    """Crop [d0, d0+edge) x ... of sample n with a one-voxel halo where the volume has one: the
    oracle's zero padding then only acts on faces that are faces of the volume.  Returns the crop
    (float64, with a leading sample axis) and the slices of the inner block inside it."""
    lo = [max(c - 1, 0) for c in (d0, h0, w0)]
    hi = [min(c + edge + 1, size) for c in (d0, h0, w0)]
    crop = f64(t[n, lo[0]:hi[0], lo[1]:hi[1], lo[2]:hi[2]])[None]
    inner = tuple(slice(c - l, c - l + edge) for c, l in zip((d0, h0, w0), lo))
    return crop, inner


def block(t, n, d0, h0, w0, edge=E):
    return f64(t[n, d0:d0 + edge, h0:h0 + edge, w0:w0 + edge])


def wgrad_entries(cin, cout, count, seed):
    rng = np.random.default_rng(seed)
    ent = [(t, int(rng.integers(cin)), int(rng.integers(cout))) for t in range(27)]   # every tap once
    while len(ent) < count:
        ent.append((int(rng.integers(27)), int(rng.integers(cin)), int(rng.integers(cout))))
    return np.array(ent, dtype=np.int64)


class Big:
    """x and g: 4 x 320^3 x 64 bf16 each, N(0,1), seeded; host float64 copies of sample 3 on demand."""

    def __init__(self):
        import torch
        gen = torch.Generator(device="cuda")
        gen.manual_seed(181112174)
        self.x = torch.empty((N, S, S, S, C), device="cuda", dtype=torch.bfloat16)
        self.g = torch.empty((N, S, S, S, C), device="cuda", dtype=torch.bfloat16)
        for n in range(N):
            self.x[n] = torch.randn((S, S, S, C), device="cuda", generator=gen).to(torch.bfloat16)
            self.g[n] = torch.randn((S, S, S, C), device="cuda", generator=gen).to(torch.bfloat16)
        self.gen = gen
        self._x3 = self._g3 = None

    def X3(self):
        if self._x3 is None:
            self._x3 = f64(self.x[3])[None]
        return self._x3

    def G3(self):
        if self._g3 is None:
            self._g3 = f64(self.g[3])[None]
        return self._g3


@pytest.fixture(scope="module")
def big():
    import torch
    free, _ = torch.cuda.mem_get_info()
    if free < 150e9:
        pytest.skip("needs ~120 GB of free device memory")
    b = Big()
    yield b
    del b
    import gc
    gc.collect()
    torch.cuda.empty_cache()


def _weights(seed, cin, cout):
    import torch
    from gpu_util import to_dev, packed_for
    wh = synth.conv_weights(seed, cin, cout, "bf16")
    bh = (synth.normal(synth.SEED, seed + 1, (cout,), np.float64) * 0.3).astype(np.float32)
    wd = to_dev(wh, "bf16")
    return wh.astype(np.float64), bh.astype(np.float64), wd, torch.from_numpy(bh).cuda(), packed_for(wd)


def _sum_of_single_sample_runs(run_one, shape_w, shape_b):
    """Sum over the four samples of the single-sample GPU results, in float64."""
    import torch
    tot_w, tot_b = np.zeros(shape_w), np.zeros(shape_b)
    one_w, one_b = None, None
    for n in range(N):
        dW, db = run_one(n)
        torch.cuda.synchronize()
        tot_w += f64(dW)
        tot_b += f64(db)
        if n == 3:
            one_w, one_b = f64(dW), f64(db)
    return tot_w, tot_b, one_w, one_b


def test_single_source_conv(orc, big):
    """Forward, backward-data with the producer-side mask as tensor and as bits, backward-weight."""
    import torch
    from paper_1811_12174_amd import k3
    x, g = big.x, big.g
    Wt, bh, wd, b, pk = _weights(90, C, C)
    y = torch.empty_like(x)
    ybits = torch.empty((N, S, S, S, C // 16), device="cuda", dtype=torch.int16)
    k3.conv3d_fwd_bits(x, wd, pk, b, 1, y, ybits)
    dx = torch.empty_like(x)
    k3.conv3d_bwd_data(g, None, wd, pk, dx, dx_mask=x)
    torch.cuda.synchronize()
    for (n, d0, h0, w0) in CORNERS:
        xc, inner = halo_crop(x, n, d0, h0, w0)
        gc_, _ = halo_crop(g, n, d0, h0, w0)
        ref = orc.conv3d_fwd(xc, Wt, bh, relu=True)[0][inner]
        got = block(y, n, d0, h0, w0)
        assert rel(got, ref) < 4e-3, ("fwd", n, d0, h0, w0)
        bits = ybits[n, d0:d0 + E, h0:h0 + E, w0:w0 + E].cpu().numpy().view(np.uint16)
        assert np.array_equal(bits, orc.relu_bits(got)), ("bits", n, d0, h0, w0)
        ref = orc.conv3d_bwd_data(gc_, Wt)[0][inner] * (xc[0][inner] > 0)
        assert rel(block(dx, n, d0, h0, w0), ref) < 4e-3, ("dgrad", n, d0, h0, w0)
    # the mask as bits: the writer's bits of x, then the bit-reading pass must reproduce dx exactly
    del y
    xbits = torch.empty((N, S, S, S, C // 16), device="cuda", dtype=torch.int16)
    for n in range(N):   # bits of the stored tensor x itself (an identity-free route: compare > 0 on the device)
        pos = (x[n] > 0).view(S, S, S, C // 16, 16).to(torch.int32)
        wts = (1 << torch.arange(16, device="cuda", dtype=torch.int32))
        xbits[n] = (pos * wts).sum(dim=-1).to(torch.int16)
        del pos
    assert np.array_equal(xbits[3, :4, :4, :4].cpu().numpy().view(np.uint16), orc.relu_bits(f64(x[3, :4, :4, :4])))
    dxb = torch.empty_like(x)
    k3.conv3d_bwd_data_bits(g, None, wd, pk, dxb, xbits)
    torch.cuda.synchronize()
    for n in range(N):
        assert torch.equal(dx[n], dxb[n]), n
    del dx, dxb, xbits, ybits
    # backward-weight
    ws = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(x, g), device="cuda", dtype=torch.uint8)

    def one(n):
        dW, db = torch.empty((3, 3, 3, C, C), device="cuda"), torch.empty(C, device="cuda")
        k3.conv3d_bwd_weight(x[n:n + 1], g[n:n + 1], None, dW, db, ws)
        return dW, db
    tot_w, tot_b, one_w, one_b = _sum_of_single_sample_runs(one, (3, 3, 3, C, C), (C,))
    ent = wgrad_entries(C, C, 40, 92)
    got = one_w.reshape(27, C, C)[ent[:, 0], ent[:, 1], ent[:, 2]]
    assert rel(got, orc.conv3d_bwd_weight_entries(big.X3(), big.G3(), ent)) < 1e-5
    assert rel(one_b, big.G3().reshape(-1, C).sum(axis=0)) < 1e-5
    dW4, db4 = torch.empty((3, 3, 3, C, C), device="cuda"), torch.empty(C, device="cuda")
    k3.conv3d_bwd_weight(x, g, None, dW4, db4, ws)
    torch.cuda.synchronize()
    assert rel(f64(dW4), tot_w) < TOL_SUM
    assert rel(f64(db4), tot_b) < TOL_SUM


def test_two_source_conv_and_two_destination_dgrad(orc, big):
    """The decoder's first convolution of a level: input [skip | up] from two tensors, its
    backward-data pass writing two tensors, its backward-weight pass reading two."""
    import torch
    from paper_1811_12174_amd import k3
    x1, x2 = big.x, big.g        # two 64-channel sources
    Wt, bh, wd, b, pk = _weights(94, 2 * C, C)
    y = torch.empty_like(x1)
    k3.conv3d_fwd(x1, wd, pk, b, 1, y, x2=x2)
    torch.cuda.synchronize()
    for (n, d0, h0, w0) in CORNERS:
        c1, inner = halo_crop(x1, n, d0, h0, w0)
        c2, _ = halo_crop(x2, n, d0, h0, w0)
        ref = orc.conv3d_fwd(np.concatenate([c1, c2], axis=-1), Wt, bh, relu=True)[0][inner]
        assert rel(block(y, n, d0, h0, w0), ref) < 4e-3, ("fwd2", n, d0, h0, w0)
    # backward-data of dy = y (any tensor of that shape serves) into [dx | dx2], dx masked by x1
    dx, dx2 = torch.empty_like(x1), torch.empty_like(x1)
    k3.conv3d_bwd_data(y, None, wd, pk, dx, dx2=dx2, dx_mask=x1)
    torch.cuda.synchronize()
    for (n, d0, h0, w0) in CORNERS:
        yc, inner = halo_crop(y, n, d0, h0, w0)
        ref = orc.conv3d_bwd_data(yc, Wt)[0][inner]
        ref[..., :C] *= block(x1, n, d0, h0, w0) > 0
        got = np.concatenate([block(dx, n, d0, h0, w0), block(dx2, n, d0, h0, w0)], axis=-1)
        assert rel(got, ref) < 4e-3, ("dgrad2", n, d0, h0, w0)
    del dx, dx2
    # backward-weight with x = [x1 | x2] and dy = y
    ws = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(x1, y, x2=x2), device="cuda", dtype=torch.uint8)

    def one(n):
        dW, db = torch.empty((3, 3, 3, 2 * C, C), device="cuda"), torch.empty(C, device="cuda")
        k3.conv3d_bwd_weight(x1[n:n + 1], y[n:n + 1], None, dW, db, ws, x2=x2[n:n + 1])
        return dW, db
    tot_w, tot_b, one_w, _ = _sum_of_single_sample_runs(one, (3, 3, 3, 2 * C, C), (C,))
    Y3 = f64(y[3])[None]
    ent = wgrad_entries(2 * C, C, 40, 95)
    lo, hi = ent[ent[:, 1] < C], ent[ent[:, 1] >= C].copy()
    got = one_w.reshape(27, 2 * C, C)
    assert rel(got[lo[:, 0], lo[:, 1], lo[:, 2]], orc.conv3d_bwd_weight_entries(big.X3(), Y3, lo)) < 1e-5
    hi_local = hi.copy()
    hi_local[:, 1] -= C      # entries of the second source, in its own channel numbering
    assert rel(got[hi[:, 0], hi[:, 1], hi[:, 2]], orc.conv3d_bwd_weight_entries(big.G3(), Y3, hi_local)) < 1e-5
    del Y3
    dW4, db4 = torch.empty((3, 3, 3, 2 * C, C), device="cuda"), torch.empty(C, device="cuda")
    k3.conv3d_bwd_weight(x1, y, None, dW4, db4, ws, x2=x2)
    torch.cuda.synchronize()
    assert rel(f64(dW4), tot_w) < TOL_SUM
    assert rel(f64(db4), tot_b) < TOL_SUM


def test_first_layer(orc, big):
    """The single-channel first convolution: forward writes, backward-weight reads, 8.4 Gi elements."""
    import torch
    from paper_1811_12174_amd import k3
    x1 = torch.empty((N, S, S, S, 1), device="cuda", dtype=torch.bfloat16)
    for n in range(N):
        x1[n] = torch.rand((S, S, S, 1), device="cuda", generator=big.gen).to(torch.bfloat16)   # volumes are scaled to [0, 1]
    Wt, bh, wd, b, pk = _weights(96, 1, C)
    y = torch.empty_like(big.x)
    k3.conv3d_fwd(x1, wd, pk, b, 1, y)
    torch.cuda.synchronize()
    for (n, d0, h0, w0) in CORNERS:
        xc, inner = halo_crop(x1, n, d0, h0, w0)
        ref = orc.conv3d_fwd(xc, Wt, bh, relu=True)[0][inner]
        assert rel(block(y, n, d0, h0, w0), ref) < 4e-3, ("first fwd", n, d0, h0, w0)
    del y
    g = big.g
    ws = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(x1, g), device="cuda", dtype=torch.uint8)

    def one(n):
        dW, db = torch.empty((3, 3, 3, 1, C), device="cuda"), torch.empty(C, device="cuda")
        k3.conv3d_bwd_weight(x1[n:n + 1], g[n:n + 1], None, dW, db, ws)
        return dW, db
    tot_w, tot_b, one_w, one_b = _sum_of_single_sample_runs(one, (3, 3, 3, 1, C), (C,))
    ent = np.array([(t, 0, co) for t in range(27) for co in (0, 17, 63)], dtype=np.int64)
    got = one_w.reshape(27, 1, C)[ent[:, 0], ent[:, 1], ent[:, 2]]
    assert rel(got, orc.conv3d_bwd_weight_entries(f64(x1[3])[None], big.G3(), ent)) < 1e-5
    assert rel(one_b, big.G3().reshape(-1, C).sum(axis=0)) < 1e-5
    dW4, db4 = torch.empty((3, 3, 3, 1, C), device="cuda"), torch.empty(C, device="cuda")
    k3.conv3d_bwd_weight(x1, g, None, dW4, db4, ws)
    torch.cuda.synchronize()
    assert rel(f64(dW4), tot_w) < TOL_SUM
    assert rel(f64(db4), tot_b) < TOL_SUM


def test_pool(orc, big):
    """2x2x2 max-pool forward and backward (with the skip gradient added and the ReLU mask of x applied; from
    routing bits): exact."""
    import torch
    from paper_1811_12174_amd import k3
    x = torch.relu(big.x)      # a stored ReLU output: ties at zero, positive bf16 ties
    p = torch.empty((N, S // 2, S // 2, S // 2, C), device="cuda", dtype=torch.bfloat16)
    k3.pool3d_fwd(x, p)
    dy = torch.empty_like(p)
    for n in range(N):
        dy[n] = torch.randn((S // 2, S // 2, S // 2, C), device="cuda", generator=big.gen).to(torch.bfloat16)
    dx = torch.empty_like(x)
    k3.pool3d_bwd(x, dy, None, dx)
    dxa = torch.empty_like(x)
    k3.pool3d_bwd(x, dy, big.g, dxa, relu_mask=True)
    torch.cuda.synchronize()
    for (n, d0, h0, w0) in CORNERS:
        d0, h0, w0 = d0 & ~1, h0 & ~1, w0 & ~1     # whole windows
        xc = block(x, n, d0, h0, w0)[None]
        dyc = block(dy, n, d0 // 2, h0 // 2, w0 // 2, E // 2)[None]
        assert np.array_equal(block(p, n, d0 // 2, h0 // 2, w0 // 2, E // 2)[None], orc.pool3d_fwd(xc)), ("pool", n, d0, h0, w0)
        ref = orc.pool3d_bwd(xc, dyc)
        assert np.array_equal(block(dx, n, d0, h0, w0)[None], ref), ("pool bwd", n, d0, h0, w0)
        ref = orc.round_bf16(orc.relu_bwd(ref + block(big.g, n, d0, h0, w0)[None], xc))
        assert np.array_equal(block(dxa, n, d0, h0, w0)[None], ref), ("pool bwd add", n, d0, h0, w0)
    # the form that keeps routing bits in place of x: same pooled tensor; bits and dx against the
    # oracle on the crops; dx against the x-reading pass over the whole tensor
    del dxa
    p2 = torch.empty_like(p)
    bits = torch.empty((N, S, S, S, C // 16), device="cuda", dtype=torch.int16)
    k3.pool3d_fwd_bits(x, p2, bits)
    dxr = torch.empty_like(x)
    k3.pool3d_bwd_bits(bits, dy, dxr)
    k3.pool3d_bwd(x, dy, None, dx, relu_mask=True)
    torch.cuda.synchronize()
    assert torch.equal(p2, p) and torch.equal(dxr, dx)
    for (n, d0, h0, w0) in CORNERS:
        d0, h0, w0 = d0 & ~1, h0 & ~1, w0 & ~1
        xc = block(x, n, d0, h0, w0)[None]
        dyc = block(dy, n, d0 // 2, h0 // 2, w0 // 2, E // 2)[None]
        rb = orc.pool3d_route_bits(xc)
        got = bits[n, d0:d0 + E, h0:h0 + E, w0:w0 + E].cpu().numpy().view(np.uint16)[None]
        assert np.array_equal(got, rb), ("route bits", n, d0, h0, w0)
        assert np.array_equal(block(dxr, n, d0, h0, w0)[None], orc.pool3d_bwd_bits(rb, dyc)), ("pool bwd bits", n, d0, h0, w0)


def test_upconv(orc, big):
    """Transposed convolution 128 -> 64 channels producing / consuming a 4 x 320^3 x 64 tensor."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev
    ci, co, Sh = 2 * C, C, S // 2
    xin = torch.empty((N, Sh, Sh, Sh, ci), device="cuda", dtype=torch.bfloat16)
    for n in range(N):
        xin[n] = torch.randn((Sh, Sh, Sh, ci), device="cuda", generator=big.gen).to(torch.bfloat16)
    wh = synth.upconv_weights(97, ci, co, "bf16")
    bh = (synth.normal(synth.SEED, 98, (co,), np.float64) * 0.5).astype(np.float32)
    wd, b = to_dev(wh, "bf16"), torch.from_numpy(bh).cuda()
    pk = torch.empty(k3.upconv3d_packed_bytes(ci, co, k3.BF16), device="cuda", dtype=torch.uint8)
    k3.upconv3d_pack_weights(wd, pk)
    W64, b64 = wh.astype(np.float64), bh.astype(np.float64)
    y = torch.empty_like(big.x)
    k3.upconv3d_fwd(xin, wd, pk, b, y)
    dy = big.g
    dx = torch.empty_like(xin)
    k3.upconv3d_bwd_data(dy, wd, pk, dx, dx_mask=xin)
    torch.cuda.synchronize()
    e = E // 2
    for (n, d0, h0, w0) in CORNERS:
        d0, h0, w0 = d0 // 2, h0 // 2, w0 // 2      # block of input voxels; it owns output voxels 2 d0 .. 2 d0 + 2 e
        xc = block(xin, n, d0, h0, w0, e)[None]
        ref = orc.upconv3d_fwd(xc, W64, b64)
        assert rel(block(y, n, 2 * d0, 2 * h0, 2 * w0, 2 * e)[None], ref) < 4e-3, ("up fwd", n, d0, h0, w0)
        ref = orc.relu_bwd(orc.upconv3d_bwd_data(block(dy, n, 2 * d0, 2 * h0, 2 * w0, 2 * e)[None], W64), xc)
        assert rel(block(dx, n, d0, h0, w0, e)[None], ref) < 4e-3, ("up dgrad", n, d0, h0, w0)
    del y, dx
    ws = torch.empty(max(1, k3.upconv3d_bwd_weight_workspace_bytes(xin, dy)), device="cuda", dtype=torch.uint8)

    def one(n):
        dW, db = torch.empty((2, 2, 2, ci, co), device="cuda"), torch.empty(co, device="cuda")
        k3.upconv3d_bwd_weight(xin[n:n + 1], dy[n:n + 1], dW, db, ws)
        return dW, db
    tot_w, tot_b, one_w, one_b = _sum_of_single_sample_runs(one, (2, 2, 2, ci, co), (co,))
    # the oracle on a depth slab of sample 3 (the op is local in the input voxel): the GPU on the same slab
    sl = slice(Sh - 24, Sh)
    xs, dys = xin[3:4, sl].contiguous(), dy[3:4, 2 * (Sh - 24):].contiguous()
    dWs, dbs = torch.empty((2, 2, 2, ci, co), device="cuda"), torch.empty(co, device="cuda")
    k3.upconv3d_bwd_weight(xs, dys, dWs, dbs, ws)
    torch.cuda.synchronize()
    rW, rb = orc.upconv3d_bwd_weight(f64(xs), f64(dys))
    assert rel(f64(dWs), rW) < 1e-5 and rel(f64(dbs), rb) < 1e-5
    assert rel(one_b, big.G3().reshape(-1, co).sum(axis=0)) < 1e-5
    dW4, db4 = torch.empty((2, 2, 2, ci, co), device="cuda"), torch.empty(co, device="cuda")
    k3.upconv3d_bwd_weight(xin, dy, dW4, db4, ws)
    torch.cuda.synchronize()
    assert rel(f64(dW4), tot_w) < TOL_SUM
    assert rel(f64(db4), tot_b) < TOL_SUM


def test_head(orc, big):
    """1x1x1 head + softmax cross-entropy over 131 M voxels x 64 channels."""
    import torch
    from paper_1811_12174_amd import k3
    a = big.x
    V = N * S ** 3
    wh = synth.head_weights(99, C)
    bh = (synth.normal(synth.SEED, 100, (3,), np.float64) * 0.3).astype(np.float32)
    whd, bhd = torch.from_numpy(wh).cuda(), torch.from_numpy(bh).cuda()
    lab = torch.randint(0, 3, (N, S, S, S), device="cuda", generator=big.gen, dtype=torch.uint8)
    ws = torch.empty(k3.head_workspace_bytes(a), device="cuda", dtype=torch.uint8)
    loss, dW, db = torch.empty(1, device="cuda"), torch.empty((C, 3), device="cuda"), torch.empty(3, device="cuda")
    da = torch.empty_like(a)
    k3.head_softmax_ce_fwd_bwd(a, whd, bhd, lab, loss, da, dW, db, None, ws, relu_mask=True)
    torch.cuda.synchronize()
    W64, b64 = wh.astype(np.float64), bh.astype(np.float64)
    for (n, d0, h0, w0) in CORNERS:
        ac = block(a, n, d0, h0, w0)
        ref = orc.head_softmax_ce(ac, W64, b64, lab[n, d0:d0 + E, h0:h0 + E, w0:w0 + E].cpu().numpy())
        # the oracle normalises by the crop's voxel count, the kernel by the tensor's
        ref_da = orc.relu_bwd(ref["da"] * (E ** 3 / V), ac)
        assert rel(block(da, n, d0, h0, w0), ref_da) < 4e-3, ("head da", n, d0, h0, w0)
    del da
    # sums: sample 3 alone against the oracle, the whole tensor against the four single-sample runs
    tot_w, tot_b, tot_l = np.zeros((C, 3)), np.zeros(3), 0.0
    for n in range(N):
        l1, dW1, db1 = torch.empty(1, device="cuda"), torch.empty((C, 3), device="cuda"), torch.empty(3, device="cuda")
        da1 = torch.empty_like(a[n:n + 1])
        k3.head_softmax_ce_fwd_bwd(a[n:n + 1], whd, bhd, lab[n:n + 1], l1, da1, dW1, db1, None, ws)
        torch.cuda.synchronize()
        tot_w += f64(dW1) / N
        tot_b += f64(db1) / N
        tot_l += l1.item() / N
        if n == 3:
            ref = orc.head_softmax_ce(big.X3()[0], W64, b64, lab[3].cpu().numpy())
            assert abs(l1.item() - ref["loss"]) < 1e-5 * abs(ref["loss"])
            assert rel(f64(dW1), ref["dW"]) < 1e-5
            assert np.abs(f64(db1) - ref["db"]).max() < 1e-5 * max(1e-3, np.abs(ref["db"]).max()) + 1e-7
        del da1
    assert abs(loss.item() - tot_l) < 1e-5 * abs(tot_l)
    assert rel(f64(dW), tot_w) < 1e-5
    assert np.abs(f64(db) - tot_b).max() < 1e-5 * max(1e-3, np.abs(tot_b).max()) + 1e-7
