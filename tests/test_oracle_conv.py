"""Pins for the oracle's 3x3x3 convolution, its two gradients and the ReLU mask.

None of these go through the oracle's own loop nest: they are closed forms, exact
shift identities, an independently structured numpy evaluation (explicit padding +
einsum over shifted views), bilinear identities, finite differences and PyTorch's CPU
operators used as a library special case.
"""
import numpy as np
import pytest

import synth

RNG = np.random.default_rng(1234)


def _einsum_conv(x, w, b=None):
    """Padded-array evaluation: sum over 27 shifted views, contraction by einsum."""
    N, D, H, W, Ci = x.shape
    xp = np.zeros((N, D + 2, H + 2, W + 2, Ci))
    xp[:, 1:-1, 1:-1, 1:-1] = x
    y = np.zeros((N, D, H, W, w.shape[4]))
    for kd in range(3):
        for kh in range(3):
            for kw in range(3):
                y += np.einsum("ndhwi,io->ndhwo", xp[:, kd:kd + D, kh:kh + H, kw:kw + W], w[kd, kh, kw])
    if b is not None:
        y += b
    return y


@pytest.mark.parametrize("shape,ci,co", [((2, 3, 4, 5), 3, 2), ((1, 1, 1, 1), 2, 3), ((1, 2, 1, 3), 1, 1), ((1, 6, 5, 4), 4, 8)])
def test_fwd_matches_padded_einsum(orc, shape, ci, co):
    x = RNG.standard_normal(shape + (ci,))
    w = RNG.standard_normal((3, 3, 3, ci, co))
    b = RNG.standard_normal(co)
    np.testing.assert_allclose(orc.conv3d_fwd(x, w, b), _einsum_conv(x, w, b), rtol=0, atol=1e-12)
    np.testing.assert_allclose(orc.conv3d_fwd(x, w, b, relu=True), np.maximum(_einsum_conv(x, w, b), 0), rtol=0, atol=1e-12)


def test_identity_and_shift_kernels_are_exact(orc):
    """A one-hot kernel at tap (kd,kh,kw) shifts x by (kd-1,kh-1,kw-1) with zero fill."""
    C = 3
    x = RNG.standard_normal((2, 4, 5, 6, C))
    for kd in range(3):
        for kh in range(3):
            for kw in range(3):
                w = np.zeros((3, 3, 3, C, C))
                w[kd, kh, kw] = np.eye(C)
                y = orc.conv3d_fwd(x, w)
                exp = np.zeros_like(x)
                sd, sh, sw = kd - 1, kh - 1, kw - 1

                def rng_(s, n):
                    return (slice(max(0, -s), n - max(0, s)), slice(max(0, s), n - max(0, -s)))
                (od, id_), (oh, ih), (ow, iw) = rng_(sd, 4), rng_(sh, 5), rng_(sw, 6)
                exp[:, od, oh, ow] = x[:, id_, ih, iw]
                assert np.array_equal(y, exp), (kd, kh, kw)


def test_channel_mixing_orientation(orc):
    """W[1,1,1] = M (C_in x C_out) must give y = x @ M, not x @ M.T."""
    x = RNG.standard_normal((1, 2, 2, 2, 3))
    M = RNG.standard_normal((3, 4))
    w = np.zeros((3, 3, 3, 3, 4))
    w[1, 1, 1] = M
    np.testing.assert_allclose(orc.conv3d_fwd(x, w), x @ M, atol=1e-13)


def test_all_ones_closed_form(orc):
    """x = 1, W = 1: y = C_in * m_d m_h m_w, m = 2 on a boundary index, 3 inside."""
    N, D, H, W, Ci, Co = 1, 5, 4, 6, 3, 2
    y = orc.conv3d_fwd(np.ones((N, D, H, W, Ci)), np.ones((3, 3, 3, Ci, Co)))

    def m(n):
        v = np.full(n, 3.0)
        v[0] = v[-1] = 2.0
        return v
    exp = Ci * m(D)[:, None, None] * m(H)[None, :, None] * m(W)[None, None, :]
    assert np.array_equal(y[0, ..., 0], exp) and np.array_equal(y[0, ..., 1], exp)
    # weight gradient of all ones: N (D-|kd-1|)(H-|kh-1|)(W-|kw-1|); bias gradient: V
    dW, db = orc.conv3d_bwd_weight(np.ones((N, D, H, W, Ci)), np.ones((N, D, H, W, Co)))
    for kd in range(3):
        for kh in range(3):
            for kw in range(3):
                e = N * (D - abs(kd - 1)) * (H - abs(kh - 1)) * (W - abs(kw - 1))
                assert np.all(dW[kd, kh, kw] == e)
    assert np.all(db == N * D * H * W)


def test_size_one_dims(orc):
    """A 1x1x1 volume only sees the centre tap."""
    x = RNG.standard_normal((1, 1, 1, 1, 4))
    w = RNG.standard_normal((3, 3, 3, 4, 5))
    np.testing.assert_allclose(orc.conv3d_fwd(x, w)[0, 0, 0, 0], x[0, 0, 0, 0] @ w[1, 1, 1], atol=1e-13)


def test_linearity(orc):
    x1, x2 = RNG.standard_normal((2, 1, 3, 4, 5, 2))
    w = RNG.standard_normal((3, 3, 3, 2, 3))
    lhs = orc.conv3d_fwd(2.5 * x1 - 0.75 * x2, w)
    rhs = 2.5 * orc.conv3d_fwd(x1, w) - 0.75 * orc.conv3d_fwd(x2, w)
    np.testing.assert_allclose(lhs, rhs, atol=1e-12)


@pytest.mark.parametrize("shape,ci,co", [((2, 3, 4, 5), 3, 2), ((1, 2, 2, 2), 1, 4), ((1, 1, 5, 1), 2, 2)])
def test_adjoint_and_bilinear_identities(orc, shape, ci, co):
    """<conv(x;W), g> = <x, dgrad(g;W)> = <W, wgrad(x,g)>."""
    x = RNG.standard_normal(shape + (ci,))
    w = RNG.standard_normal((3, 3, 3, ci, co))
    g = RNG.standard_normal(shape + (co,))
    ref = np.sum(orc.conv3d_fwd(x, w) * g)
    assert abs(np.sum(x * orc.conv3d_bwd_data(g, w)) - ref) < 1e-10 * max(1, abs(ref))
    dW, db = orc.conv3d_bwd_weight(x, g)
    assert abs(np.sum(w * dW) - ref) < 1e-10 * max(1, abs(ref))
    np.testing.assert_allclose(db, g.reshape(-1, co).sum(0), atol=1e-12)


def test_dgrad_one_hot_is_kernel_stamp(orc):
    """A single 1 in g at voxel p, channel co stamps W[:, :, :, :, co] flipped around p."""
    D = H = W = 5
    ci, co = 2, 3
    w = RNG.standard_normal((3, 3, 3, ci, co))
    g = np.zeros((1, D, H, W, co))
    g[0, 2, 2, 2, 1] = 1.0
    dx = orc.conv3d_bwd_data(g, w)
    for kd in range(3):
        for kh in range(3):
            for kw in range(3):
                # output voxel p sees x at p + k - 1, so dx[p + k - 1] = W[k]
                np.testing.assert_array_equal(dx[0, 1 + kd, 1 + kh, 1 + kw], w[kd, kh, kw, :, 1])
    assert np.count_nonzero(dx) <= 27 * ci


def test_wgrad_finite_differences(orc):
    """Central differences of L(W) = <relu(conv(x;W,b)), r> against wgrad through the ReLU mask."""
    x = RNG.standard_normal((1, 3, 4, 3, 2))
    w = RNG.standard_normal((3, 3, 3, 2, 3)) * 0.3
    b = RNG.standard_normal(3) * 0.1
    r = RNG.standard_normal((1, 3, 4, 3, 3))

    def L(w_, b_):
        return np.sum(orc.conv3d_fwd(x, w_, b_, relu=True) * r)
    y = orc.conv3d_fwd(x, w, b, relu=True)
    g = orc.relu_bwd(r, y)
    dW, db = orc.conv3d_bwd_weight(x, g)
    dx = orc.conv3d_bwd_data(g, w)
    eps = 1e-6
    for _ in range(12):
        v = RNG.standard_normal(w.shape)
        fd = (L(w + eps * v, b) - L(w - eps * v, b)) / (2 * eps)
        assert abs(fd - np.sum(dW * v)) < 1e-6 * max(1.0, abs(fd))
    vb = RNG.standard_normal(3)
    fd = (L(w, b + eps * vb) - L(w, b - eps * vb)) / (2 * eps)
    assert abs(fd - db @ vb) < 1e-6 * max(1.0, abs(fd))
    vx = RNG.standard_normal(x.shape)
    fd = (np.sum(orc.conv3d_fwd(x + eps * vx, w, b, relu=True) * r) - np.sum(orc.conv3d_fwd(x - eps * vx, w, b, relu=True) * r)) / (2 * eps)
    assert abs(fd - np.sum(dx * vx)) < 1e-6 * max(1.0, abs(fd))


def test_relu_mask_is_strict(orc):
    dy = np.array([1.0, 2.0, 3.0, 4.0])
    y = np.array([0.0, -0.0, 1e-300, -1.0])
    assert np.array_equal(orc.relu_bwd(dy, y), [0.0, 0.0, 3.0, 0.0])


def test_points_and_entries_match_full(orc):
    x = RNG.standard_normal((2, 4, 5, 3, 3))
    w = RNG.standard_normal((3, 3, 3, 3, 4))
    b = RNG.standard_normal(4)
    g = RNG.standard_normal((2, 4, 5, 3, 4))
    y = orc.conv3d_fwd(x, w, b, relu=True)
    pts = np.array([[0, 0, 0, 0], [1, 3, 4, 2], [0, 2, 2, 1], [1, 0, 4, 0]])
    yp = orc.conv3d_fwd_points(x, w, b, True, pts)
    for i, (n, d, h, ww) in enumerate(pts):
        np.testing.assert_array_equal(yp[i], y[n, d, h, ww])
    # the backward-data sampler on every voxel of the tensor, corners, edges and faces included
    dx = orc.conv3d_bwd_data(g, w)
    allp = np.array([(n, d, h, ww) for n in range(2) for d in range(4) for h in range(5) for ww in range(3)])
    dxp = orc.conv3d_bwd_data_points(g, w, allp)
    np.testing.assert_array_equal(dxp.reshape(dx.shape), dx)
    dW, _ = orc.conv3d_bwd_weight(x, g)
    ent = np.array([[0, 0, 0], [13, 2, 3], [26, 1, 1], [5, 2, 0]])
    out = orc.conv3d_bwd_weight_entries(x, g, ent)
    for i, (t, ci, co) in enumerate(ent):
        np.testing.assert_allclose(out[i], dW.reshape(27, 3, 4)[t, ci, co], rtol=1e-13)


def test_bwd_data_points_is_the_adjoint_at_single_voxels(orc):
    """<conv(x), g> = <x, dgrad(g)> with x a one-hot tensor reads off one entry of dgrad(g): the sampler
    must return exactly that entry, computed through the forward pass only."""
    w = RNG.standard_normal((3, 3, 3, 3, 2))
    g = RNG.standard_normal((1, 3, 4, 3, 2))
    pts = np.array([[0, 0, 0, 0], [0, 2, 3, 2], [0, 1, 2, 1], [0, 0, 3, 1]])
    got = orc.conv3d_bwd_data_points(g, w, pts)
    for i, (n, d, h, ww) in enumerate(pts):
        for ci in range(3):
            e = np.zeros((1, 3, 4, 3, 3))
            e[n, d, h, ww, ci] = 1.0
            assert abs(np.sum(orc.conv3d_fwd(e, w) * g) - got[i, ci]) < 1e-12


def test_against_torch_cpu_fp64(orc):
    """Library special case: torch.nn.functional.conv3d on CPU in fp64 with autograd."""
    torch = pytest.importorskip("torch")
    x = synth.activations(1, (2, 6, 5, 7, 4), "f32").astype(np.float64)
    w = synth.conv_weights(2, 4, 8, "f32").astype(np.float64)
    b = RNG.standard_normal(8)
    r = synth.activations(3, (2, 6, 5, 7, 8), "f32").astype(np.float64)
    xt = torch.tensor(x).permute(0, 4, 1, 2, 3).clone().requires_grad_(True)
    wt = torch.tensor(w).permute(4, 3, 0, 1, 2).clone().requires_grad_(True)
    bt = torch.tensor(b, requires_grad=True)
    yt = torch.relu(torch.nn.functional.conv3d(xt, wt, bt, padding=1))
    (yt * torch.tensor(r).permute(0, 4, 1, 2, 3)).sum().backward()
    y = orc.conv3d_fwd(x, w, b, relu=True)
    np.testing.assert_allclose(y, yt.detach().permute(0, 2, 3, 4, 1).numpy(), atol=1e-12)
    g = orc.relu_bwd(r, y)
    np.testing.assert_allclose(orc.conv3d_bwd_data(g, w), xt.grad.permute(0, 2, 3, 4, 1).numpy(), atol=1e-11)
    dW, db = orc.conv3d_bwd_weight(x, g)
    np.testing.assert_allclose(dW, wt.grad.permute(2, 3, 4, 1, 0).numpy(), atol=1e-10)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-10)


def test_relu_bits_by_hand_and_against_relu_bwd(orc):
    y = np.zeros((1, 1, 1, 2, 32))
    y[0, 0, 0, 0, [0, 3, 15, 16, 31]] = [1.0, 0.5, 2.0, 1e-30, 7.0]
    y[0, 0, 0, 1, [1, 17]] = [-1.0, 3.0]                       # a negative value sets no bit
    b = orc.relu_bits(y)
    assert b.shape == (1, 1, 1, 2, 2) and b.dtype == np.uint16
    assert b[0, 0, 0, 0].tolist() == [(1 << 0) | (1 << 3) | (1 << 15), (1 << 0) | (1 << 15)]
    assert b[0, 0, 0, 1].tolist() == [0, 1 << 1]
    rng = np.random.default_rng(12)
    y = np.maximum(rng.normal(size=(2, 3, 2, 5, 48)), 0)
    dy = rng.normal(size=y.shape)
    assert np.array_equal(orc.apply_relu_bits(dy, orc.relu_bits(y)), orc.relu_bwd(dy, y))
    assert orc.relu_bits(np.ones((1, 1, 1, 1, 16)))[0, 0, 0, 0, 0] == 0xFFFF
