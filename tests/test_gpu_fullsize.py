"""GPU parity at the sizes and in the launch configuration the benchmark times.

The small cases of test_gpu_conv.py run the small-volume kernels; volumes with at least one
tile per compute unit take the persistent pipelined kernels, which these tests cover: the
whole encoder block of workload config 2 (1 x 64^3, 32 -> 32) exactly as bench.py issues it,
and U-Net-sized layers (64 and 128 channels, two sources / two destinations, ragged tiles).
The oracle evaluates sampled output voxels (all channels) and sampled weight-gradient entries
(full voxel sum) one by one; the samples include every corner, points on faces and edges, and
points on both sides of tile borders.
"""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def sample_points(N, D, H, W, count, seed):
    """Voxel coordinates: the 8 corners of each sample, border and tile-border points, random fill."""
    rng = np.random.default_rng(seed)
    pts = []
    for n in range(N):
        for d in (0, D - 1):
            for h in (0, H - 1):
                for w in (0, W - 1):
                    pts.append((n, d, h, w))
    special = {  # coordinates next to tile borders of every kernel (tiles of 4, 8 and 16 voxels)
        "d": [v for v in (0, 1, 3, 4, 5, 6, 7, 8, 9, 15, 16, D // 2, D - 2, D - 1) if 0 <= v < D],
        "h": [v for v in (0, 1, 7, 8, 9, 15, 16, 17, H // 2, H - 2, H - 1) if 0 <= v < H],
        "w": [v for v in (0, 1, 7, 8, 15, 16, 17, 31, 32, W // 2, W - 2, W - 1) if 0 <= v < W],
    }
    for _ in range(count // 2):
        pts.append((int(rng.integers(N)), int(rng.choice(special["d"])), int(rng.choice(special["h"])),
                    int(rng.choice(special["w"]))))
    while len(pts) < count:
        pts.append((int(rng.integers(N)), int(rng.integers(D)), int(rng.integers(H)), int(rng.integers(W))))
    return np.array(pts, dtype=np.int64)


def gather(t, pts):
    """device tensor [N,D,H,W,C] -> float64 numpy [npts, C] at the sampled voxels."""
    import torch
    idx = torch.from_numpy(pts).cuda()
    return t[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].to(torch.float32).cpu().numpy().astype(np.float64)


def host64(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rel(got, ref):
    from gpu_util import rel_l2
    return rel_l2(got, ref, depth=2)


def wgrad_entries(cin, cout, count, seed):
    rng = np.random.default_rng(seed)
    ent = [(t, int(rng.integers(cin)), int(rng.integers(cout))) for t in range(27)]   # every tap once
    while len(ent) < count:
        ent.append((int(rng.integers(27)), int(rng.integers(cin)), int(rng.integers(cout))))
    return np.array(ent, dtype=np.int64)


def test_cfg2_block_as_benchmarked(orc):
    """The encoder block of workload config 2, call for call as bench.py runs it."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev
    N, S, C = 1, 64, 32
    bf = torch.bfloat16
    xh = synth.activations(1, (N, S, S, S, C), "bf16")
    w1h, w2h = synth.conv_weights(2, C, C, "bf16"), synth.conv_weights(3, C, C, "bf16")
    b1h = (synth.normal(synth.SEED, 5, (C,), np.float64) * 0.1).astype(np.float32)
    b2h = (synth.normal(synth.SEED, 6, (C,), np.float64) * 0.1).astype(np.float32)
    dyph = synth.activations(4, (N, S // 2, S // 2, S // 2, C), "bf16")
    x, w1, w2, dyp = to_dev(xh, "bf16"), to_dev(w1h, "bf16"), to_dev(w2h, "bf16"), to_dev(dyph, "bf16")
    b1, b2 = torch.from_numpy(b1h).cuda(), torch.from_numpy(b2h).cuda()
    pk1 = torch.empty(k3.conv3d_packed_bytes(C, C, k3.BF16), device="cuda", dtype=torch.uint8)
    pk2 = torch.empty_like(pk1)
    k3.conv3d_pack_weights(w1, pk1)
    k3.conv3d_pack_weights(w2, pk2)
    a1, a2, da2, da1, dx = (torch.full_like(x, float("nan")) for _ in range(5))
    p = torch.empty_like(dyp)
    dW1, dW2 = torch.empty((3, 3, 3, C, C), device="cuda"), torch.empty((3, 3, 3, C, C), device="cuda")
    db1, db2 = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    ws = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(x, a1), device="cuda", dtype=torch.uint8)
    a1bits = torch.empty(k3.relu_bits_bytes(a1) // 2, device="cuda", dtype=torch.int16)
    k3.conv3d_fwd_bits(x, w1, pk1, b1, 1, a1, a1bits)
    k3.conv3d_fwd(a1, w2, pk2, b2, 1, a2)
    k3.pool3d_fwd(a2, p)
    k3.pool3d_bwd(a2, dyp, None, da2, relu_mask=True)
    k3.conv3d_bwd_weight(a1, da2, None, dW2, db2, ws)
    k3.conv3d_bwd_data_bits(da2, None, w2, pk2, da1, a1bits)
    k3.conv3d_bwd_weight(x, da1, None, dW1, db1, ws)
    k3.conv3d_bwd_data(da1, None, w1, pk1, dx)
    torch.cuda.synchronize()
    for t in (a1, a2, da2, da1, dx):
        assert torch.isfinite(t.float()).all()

    pts = sample_points(N, S, S, S, 3000, 11)
    X, W1, W2 = xh.astype(np.float64), w1h.astype(np.float64), w2h.astype(np.float64)
    A1, A2, DA2, DA1 = host64(a1), host64(a2), host64(da2), host64(da1)
    # forward convs on the GPU's own inputs: one bf16 rounding of an fp32 sum
    e = rel(gather(a1, pts), orc.conv3d_fwd_points(X, W1, b1h.astype(np.float64), True, pts))
    assert e < 4e-3, e
    e = rel(gather(a2, pts), orc.conv3d_fwd_points(A1, W2, b2h.astype(np.float64), True, pts))
    assert e < 4e-3, e
    # pool forward and pool backward with the ReLU mask of a2: compare-only, exact
    assert np.array_equal(host64(p), orc.pool3d_fwd(A2))
    assert np.array_equal(DA2, orc.relu_bwd(orc.pool3d_bwd(A2, dyph.astype(np.float64)), A2))
    # backward-data of conv2, masked by a1 at the producer
    ref = orc.conv3d_bwd_data_points(DA2, W2, pts) * (gather(a1, pts) > 0)
    e = rel(gather(da1, pts), ref)
    assert e < 4e-3, e
    ref = orc.conv3d_bwd_data_points(DA1, W1, pts)
    e = rel(gather(dx, pts), ref)
    assert e < 4e-3, e
    # weight gradients: sampled entries with the full voxel sum, bias gradients in full
    ent = wgrad_entries(C, C, 160, 12)
    got2 = host64(dW2).reshape(27, C, C)[ent[:, 0], ent[:, 1], ent[:, 2]]
    assert rel(got2, orc.conv3d_bwd_weight_entries(A1, DA2, ent)) < 1e-5
    got1 = host64(dW1).reshape(27, C, C)[ent[:, 0], ent[:, 1], ent[:, 2]]
    assert rel(got1, orc.conv3d_bwd_weight_entries(X, DA1, ent)) < 1e-5
    assert rel(host64(db2), DA2.reshape(-1, C).sum(axis=0)) < 1e-5
    assert rel(host64(db1), DA1.reshape(-1, C).sum(axis=0)) < 1e-5


# (N, D, H, W, c1, c2, cout): U-Net layer shapes, several tiles per compute unit, ragged edges
BIG_CASES = [
    (1, 64, 72, 140, 64, 0, 64),     # encoder conv2 (two output blocks per workgroup), ragged in w
    (2, 44, 64, 64, 64, 64, 64),     # decoder conv1: two sources / two destinations, ragged depth
    (1, 64, 64, 64, 128, 0, 128),    # deeper level: four channel blocks, two channel groups
    (1, 66, 70, 72, 64, 0, 32),      # one output block per workgroup, ragged everywhere
    (1, 128, 128, 128, 32, 0, 32),   # level 0 of the base-32 net: plane-streaming kernel, 8 tiles per workgroup; 32 planes per weight-gradient workgroup
    (1, 32, 32, 32, 128, 0, 128),    # deep level: 4x8x8 tiles, two output blocks per workgroup
    (1, 16, 16, 16, 256, 0, 256),    # bottleneck: 4x8x8 tiles, one output block per workgroup
    (1, 14, 20, 28, 64, 64, 128),    # 4x8x8 tiles, two sources / destinations, ragged
    (1, 40, 36, 50, 1, 0, 64),       # single-channel first layer (MFMA im2col kernels), ragged tiles
    (2, 20, 24, 48, 1, 0, 32),       # first layer, two samples, one output block
    (2, 36, 40, 44, 1, 0, 128),      # first layer with 128 channels, ragged tiles
]


@pytest.mark.parametrize("case", BIG_CASES, ids=lambda c: "x".join(map(str, c)))
def test_unet_sized_layers_sampled(orc, case):
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, packed_for
    N, D, H, W, c1, c2, co = case
    cin = c1 + c2
    xh = synth.activations(50, (N, D, H, W, c1), "bf16")
    x2h = synth.activations(51, (N, D, H, W, c2), "bf16") if c2 else None
    wh = synth.conv_weights(52, cin, co, "bf16")
    bh = (synth.normal(synth.SEED, 53, (co,), np.float64) * 0.3).astype(np.float32)
    gh = synth.activations(54, (N, D, H, W, co), "bf16")
    mh = synth.activations(55, (N, D, H, W, c1), "bf16")
    mh[mh < 0.2] = 0.0
    x, wd, g, m = to_dev(xh, "bf16"), to_dev(wh, "bf16"), to_dev(gh, "bf16"), to_dev(mh, "bf16")
    x2 = to_dev(x2h, "bf16") if c2 else None
    b = torch.from_numpy(bh).cuda()
    pk = packed_for(wd)
    pts = sample_points(N, D, H, W, 1500, 21)
    X = xh.astype(np.float64) if not c2 else np.concatenate([xh, x2h], axis=-1).astype(np.float64)
    Wt, G = wh.astype(np.float64), gh.astype(np.float64)

    y = torch.full((N, D, H, W, co), float("nan"), device="cuda", dtype=torch.bfloat16)
    k3.conv3d_fwd(x, wd, pk, b, 1, y, x2=x2)
    torch.cuda.synchronize()
    assert torch.isfinite(y.float()).all()
    e = rel(gather(y, pts), orc.conv3d_fwd_points(X, Wt, bh.astype(np.float64), True, pts))
    assert e < 4e-3, e

    dx = torch.full((N, D, H, W, c1), float("nan"), device="cuda", dtype=torch.bfloat16)
    dx2 = torch.full((N, D, H, W, c2), float("nan"), device="cuda", dtype=torch.bfloat16) if c2 else None
    k3.conv3d_bwd_data(g, None, wd, pk, dx, dx2=dx2, dx_mask=m)
    torch.cuda.synchronize()
    ref = orc.conv3d_bwd_data_points(G, Wt, pts)
    ref[:, :c1] *= gather(m, pts) > 0
    got = gather(dx, pts) if not c2 else np.concatenate([gather(dx, pts), gather(dx2, pts)], axis=1)
    assert np.isfinite(got).all()
    e = rel(got, ref)
    assert e < 4e-3, e

    dW = torch.full((3, 3, 3, cin, co), float("nan"), device="cuda")
    db = torch.full((co,), float("nan"), device="cuda")
    ws = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(x, g, x2=x2), device="cuda", dtype=torch.uint8)
    k3.conv3d_bwd_weight(x, g, None, dW, db, ws, x2=x2)
    torch.cuda.synchronize()
    assert torch.isfinite(dW).all()
    ent = wgrad_entries(cin, co, 60, 22)
    got = host64(dW).reshape(27, cin, co)[ent[:, 0], ent[:, 1], ent[:, 2]]
    assert rel(got, orc.conv3d_bwd_weight_entries(X, G, ent)) < 1e-5
    assert rel(host64(db), G.reshape(-1, co).sum(axis=0)) < 1e-5


@pytest.mark.parametrize("sp,ci,co", [((1, 32, 32, 32), 128, 64),     # four channel blocks per wave, 4 steps per tap
                                      ((1, 32, 32, 32), 64, 32),      # two blocks per wave
                                      ((1, 32, 32, 32), 128, 128),    # four blocks, 8 steps in two halves
                                      ((1, 16, 32, 32), 256, 256),    # 16 steps in chunks of 4
                                      ((1, 20, 24, 44), 128, 64),     # ragged last voxel block
                                      ((1, 8, 8, 16), 256, 128)])     # small volume: one block per wave
def test_upconv_bwd_data_at_unet_sizes(orc, sp, ci, co):
    """The transposed-conv backward-data instantiations that only large volumes select.  The pass is
    local (dx at an input voxel reads the 2x2x2 output voxels it covers), so the oracle runs on
    crops of whole blocks, cut at the corners and inside."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty
    N, D, H, W = sp
    x = np.maximum(synth.activations(64, (N, D, H, W, ci), "bf16"), 0)       # the stored ReLU output used as mask
    w = synth.upconv_weights(65, ci, co, "bf16")
    dy = synth.activations(66, (N, 2 * D, 2 * H, 2 * W, co), "bf16")
    xd, wd, dyd = to_dev(x, "bf16"), to_dev(w, "bf16"), to_dev(dy, "bf16")
    pk = torch.empty(k3.upconv3d_packed_bytes(ci, co, k3.BF16), device="cuda", dtype=torch.uint8)
    k3.upconv3d_pack_weights(wd, pk)
    dx, dxm = empty(x.shape, "bf16"), empty(x.shape, "bf16")
    k3.upconv3d_bwd_data(dyd, wd, pk, dx)
    k3.upconv3d_bwd_data(dyd, wd, pk, dxm, dx_mask=xd)
    torch.cuda.synchronize()
    got, gotm = to_f64(dx), to_f64(dxm)
    cd, ch, cw = min(4, D), min(4, H), min(8, W)
    for (d0, h0, w0) in [(0, 0, 0), (D - cd, H - ch, W - cw), (D // 2 - 1, H // 3, W // 2 - 3), (0, H - ch, W // 2)]:
        crop = dy[:, 2 * d0:2 * (d0 + cd), 2 * h0:2 * (h0 + ch), 2 * w0:2 * (w0 + cw), :].astype(np.float64)
        ref = orc.upconv3d_bwd_data(crop, w.astype(np.float64))
        sl = (slice(None), slice(d0, d0 + cd), slice(h0, h0 + ch), slice(w0, w0 + cw))
        assert rel(got[sl], ref) < 4e-3, (d0, h0, w0)
        assert rel(gotm[sl], orc.relu_bwd(ref, x[sl].astype(np.float64))) < 4e-3, (d0, h0, w0)


@pytest.mark.parametrize("sp,ci,co", [((2, 40, 42, 41), 128, 64),      # all four blocks of dx in one workgroup, dy read once; ragged last block
                                      ((1, 52, 51, 50), 256, 128),    # two blocks per workgroup, two voxel groups per wave
                                      ((1, 51, 52, 50), 512, 256),    # one block per workgroup, 16 groups
                                      ((1, 64, 64, 40), 256, 64)])    # two groups of four blocks
def test_upconv_bwd_data_with_weights_in_lds(orc, sp, ci, co):
    """The transposed-conv backward-data kernel that large volumes select (weights resident in LDS, persistent
    workgroups, the next tap's loads in flight), without and with the ReLU mask of dx.  Tensors are made on
    the device; the pass is local, so the oracle runs on crops of input voxels (corners, the ragged end,
    inside), and every element of dx is checked to have been written."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev
    N, D, H, W = sp
    assert N * D * H * W >= 4 * 256 * 128            # what the dispatch asks for before it picks this kernel
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1811 + ci + co)
    dyd = torch.randn((N, 2 * D, 2 * H, 2 * W, co), device="cuda", generator=gen).to(torch.bfloat16)
    xd = torch.relu(torch.randn((N, D, H, W, ci), device="cuda", generator=gen)).to(torch.bfloat16)   # the stored ReLU output used as mask
    w = synth.upconv_weights(65, ci, co, "bf16")
    wd = to_dev(w, "bf16")
    pk = torch.empty(k3.upconv3d_packed_bytes(ci, co, k3.BF16), device="cuda", dtype=torch.uint8)
    k3.upconv3d_pack_weights(wd, pk)
    dx = torch.full_like(xd, float("nan"))
    dxm = torch.full_like(xd, float("nan"))
    k3.upconv3d_bwd_data(dyd, wd, pk, dx)
    k3.upconv3d_bwd_data(dyd, wd, pk, dxm, dx_mask=xd)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(dx).any()) and not bool(torch.isnan(dxm).any())
    f64 = lambda t: t.to(torch.float32).cpu().numpy().astype(np.float64)
    cd, ch, cw = 3, 3, 4
    for n in sorted({0, N - 1}):
        for (d0, h0, w0) in [(0, 0, 0), (D - cd, H - ch, W - cw), (D // 2, H // 3, W // 2 - 1), (D - cd, 0, W // 2), (1, H - ch, 3)]:
            crop = f64(dyd[n:n + 1, 2 * d0:2 * (d0 + cd), 2 * h0:2 * (h0 + ch), 2 * w0:2 * (w0 + cw), :])
            ref = orc.upconv3d_bwd_data(crop, w.astype(np.float64))
            sl = (slice(n, n + 1), slice(d0, d0 + cd), slice(h0, h0 + ch), slice(w0, w0 + cw))
            assert rel(f64(dx[sl]), ref) < 4e-3, (n, d0, h0, w0)
            assert rel(f64(dxm[sl]), orc.relu_bwd(ref, f64(xd[sl]))) < 4e-3, (n, d0, h0, w0)


@pytest.mark.parametrize("sp,ci,co", [((2, 32, 32, 32), 256, 128),    # level 2 -> 1 of a base-64 net: 4 blocks of 256 voxels per workgroup
                                      ((1, 17, 16, 19), 512, 256),    # level 3 -> 2: 3 blocks per workgroup, ragged last block, two tap groups
                                      ((1, 9, 7, 5), 256, 64),        # fewer blocks than workgroups, ragged
                                      ((1, 40, 36, 28), 512, 512)])   # 16 output blocks x 2 tap groups: 8 workgroups per pair, 40 blocks each
def test_upconv_fwd_at_deep_levels(orc, sp, ci, co):
    """The transposed-conv forward kernel of the 256- and 512-channel levels (voxel blocks walked by
    persistent workgroups with the next block's loads in flight).  The pass is local (an output voxel
    reads one input voxel), so the oracle runs on crops of input voxels, cut at the corners, at the
    ragged end and inside; every output voxel is also checked to have been written."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty
    N, D, H, W = sp
    x = synth.activations(67, (N, D, H, W, ci), "bf16")
    w = synth.upconv_weights(68, ci, co, "bf16")
    b = (synth.normal(synth.SEED, 69, (co,), np.float64) * 0.5).astype(np.float32)
    xd, wd, bd = to_dev(x, "bf16"), to_dev(w, "bf16"), torch.from_numpy(b).cuda()
    pk = torch.empty(k3.upconv3d_packed_bytes(ci, co, k3.BF16), device="cuda", dtype=torch.uint8)
    k3.upconv3d_pack_weights(wd, pk)
    y = empty((N, 2 * D, 2 * H, 2 * W, co), "bf16")
    y.fill_(float("nan"))
    k3.upconv3d_fwd(xd, wd, pk, bd, y)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(y).any())
    got = to_f64(y)
    cd, ch, cw = min(3, D), min(3, H), min(4, W)
    for n in sorted({0, N - 1}):
        for (d0, h0, w0) in [(0, 0, 0), (D - cd, H - ch, W - cw), (D // 2, H // 3, W // 2 - 1), (D - cd, 0, W // 2)]:
            crop = x[n:n + 1, d0:d0 + cd, h0:h0 + ch, w0:w0 + cw, :].astype(np.float64)
            ref = orc.upconv3d_fwd(crop, w.astype(np.float64), b.astype(np.float64))
            sl = (slice(n, n + 1), slice(2 * d0, 2 * (d0 + cd)), slice(2 * h0, 2 * (h0 + ch)), slice(2 * w0, 2 * (w0 + cw)))
            assert rel(got[sl], ref) < 4e-3, (n, d0, h0, w0)


@pytest.mark.parametrize("N,S,c1,c2,co", [(1, 64, 32, 0, 32),      # 8x8x16 tiles, one output block per workgroup (the benchmark's layer)
                                           (1, 64, 64, 0, 64),      # two blocks per workgroup: ring of mask words vs bits
                                           (1, 32, 128, 0, 128),    # 4x8x8 tiles, two blocks
                                           (1, 48, 64, 64, 64),     # two sources / two destinations, mask on the first
                                           (1, 40, 32, 0, 64)])     # ragged 8x8x16 tiles
def test_relu_bit_masks_in_the_pipelined_kernels(orc, N, S, c1, c2, co):
    """Bit masks written by the pipelined forward kernel against the oracle's mask of the stored
    output, and backward-data with the mask as bits against backward-data with the mask as tensor
    (bit-identical), at sizes that select every tile variant."""
    import torch
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, packed_for
    cin = c1 + c2
    D = H = S
    W = S + (4 if S == 40 else 0)
    x = synth.activations(24, (N, D, H, W, cin), "bf16")
    wd = to_dev(synth.conv_weights(25, cin, co, "bf16"), "bf16")
    bd = torch.from_numpy((synth.normal(synth.SEED, 26, (co,), np.float64) * 0.3).astype(np.float32)).cuda()
    xd = to_dev(x, "bf16")
    x1 = xd[..., :c1].contiguous()
    x2 = xd[..., c1:].contiguous() if c2 else None
    pk = packed_for(wd)
    y0 = torch.empty((N, D, H, W, co), device="cuda", dtype=torch.bfloat16)
    y1 = torch.empty_like(y0)
    bits = torch.full((N, D, H, W, co // 16), -1, device="cuda", dtype=torch.int16)
    k3.conv3d_fwd(x1, wd, pk, bd, 1, y0, x2=x2)
    k3.conv3d_fwd_bits(x1, wd, pk, bd, 1, y1, bits, x2=x2)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1)
    assert np.array_equal(bits.cpu().numpy().view(np.uint16), orc.relu_bits(host64(y1)))
    m = torch.relu(x1)
    mbits = torch.from_numpy(orc.relu_bits(host64(m)).view(np.int16)).cuda()
    g = to_dev(synth.activations(27, (N, D, H, W, co), "bf16"), "bf16")
    dxa, dxb = torch.empty_like(x1), torch.empty_like(x1)
    dx2a = torch.empty_like(x2) if c2 else None
    dx2b = torch.empty_like(x2) if c2 else None
    k3.conv3d_bwd_data(g, None, wd, pk, dxa, dx2=dx2a, dx_mask=m)
    k3.conv3d_bwd_data_bits(g, None, wd, pk, dxb, mbits, dx2=dx2b)
    torch.cuda.synchronize()
    assert torch.equal(dxa, dxb)
    assert c2 == 0 or torch.equal(dx2a, dx2b)
