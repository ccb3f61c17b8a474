"""Pins for the oracle's max-pool, transposed conv and softmax-CE head."""
import math

import numpy as np
import pytest

import synth

RNG = np.random.default_rng(4321)


# ----------------------------------------------------------------- pool
def test_pool_matches_reshape_max(orc):
    x = RNG.standard_normal((2, 4, 6, 8, 3))
    exp = x.reshape(2, 2, 2, 3, 2, 4, 2, 3).max(axis=(2, 4, 6))
    assert np.array_equal(orc.pool3d_fwd(x), exp)


def test_pool_ramp_and_constant_tie_rule(orc):
    """A strictly increasing ramp selects corner (1,1,1); a constant selects (0,0,0)."""
    D = 4
    ramp = np.arange(D * D * D, dtype=np.float64).reshape(1, D, D, D, 1)
    dy = np.ones((1, 2, 2, 2, 1))
    dx = orc.pool3d_bwd(ramp, dy)
    exp = np.zeros_like(ramp)
    exp[0, 1::2, 1::2, 1::2, 0] = 1
    assert np.array_equal(dx, exp)
    dx = orc.pool3d_bwd(np.full_like(ramp, 7.0), dy)
    exp = np.zeros_like(ramp)
    exp[0, 0::2, 0::2, 0::2, 0] = 1
    assert np.array_equal(dx, exp)


def test_pool_first_max_in_lexicographic_order(orc):
    x = np.zeros((1, 2, 2, 2, 1))
    x[0, 0, 1, 1, 0] = 5.0   # (i,j,k) = (0,1,1)
    x[0, 1, 0, 0, 0] = 5.0   # (1,0,0) comes later
    dx = orc.pool3d_bwd(x, np.full((1, 1, 1, 1, 1), 3.0))
    assert dx[0, 0, 1, 1, 0] == 3.0 and np.count_nonzero(dx) == 1


def test_pool_bwd_conserves_mass_and_is_gradient(orc):
    x = RNG.standard_normal((2, 4, 4, 6, 3))
    dy = RNG.standard_normal((2, 2, 2, 3, 3))
    dx = orc.pool3d_bwd(x, dy)
    assert abs(dx.sum() - dy.sum()) < 1e-12
    assert np.count_nonzero(dx) == dy.size
    v = RNG.standard_normal(x.shape)
    eps = 1e-7
    fd = (np.sum(orc.pool3d_fwd(x + eps * v) * dy) - np.sum(orc.pool3d_fwd(x - eps * v) * dy)) / (2 * eps)
    assert abs(fd - np.sum(dx * v)) < 1e-6


def test_pool_route_bits_by_hand(orc):
    """One window, 16 channels: channel 0 has its maximum at (0,1,1) twice-tied with (1,0,0), channel 1
    is all negative (nothing routed), channel 2 all zero (nothing routed: ReLU off), channel 3 peaks
    at (1,1,1); the other channels are constant 2 -> the first element (0,0,0)."""
    x = np.full((1, 2, 2, 2, 16), 2.0)
    x[..., 0] = 0.0; x[0, 0, 1, 1, 0] = 5.0; x[0, 1, 0, 0, 0] = 5.0
    x[..., 1] = -1.0; x[0, 1, 1, 0, 1] = -0.5
    x[..., 2] = 0.0
    x[..., 3] = 1.0; x[0, 1, 1, 1, 3] = 9.0
    bits = orc.pool3d_route_bits(x)
    assert bits.shape == (1, 2, 2, 2, 1) and bits.dtype == np.uint16
    exp = np.zeros((1, 2, 2, 2, 1), dtype=np.uint16)
    exp[0, 0, 0, 0, 0] = 0xFFF0            # channels 4..15 at the first element
    exp[0, 0, 1, 1, 0] = 0x0001            # channel 0
    exp[0, 1, 1, 1, 0] = 0x0008            # channel 3
    assert np.array_equal(bits, exp)
    dy = np.arange(1, 17, dtype=np.float64).reshape(1, 1, 1, 1, 16)
    dx = orc.pool3d_bwd_bits(bits, dy)
    assert dx[0, 0, 1, 1, 0] == 1.0 and dx[0, 1, 1, 1, 3] == 4.0 and dx[0, 0, 0, 0, 15] == 16.0
    assert np.count_nonzero(dx) == 14


@pytest.mark.parametrize("ties", [False, True])
def test_pool_route_bits_equal_pool_bwd_then_relu_bwd(orc, ties):
    """The bit form is the loop form: routing by the C loops (strict >, first maximum) followed by
    the ReLU mask of x, on data with and without many equal values and zeros."""
    shape = (2, 4, 6, 8, 32)
    x = RNG.integers(-2, 3, shape).astype(np.float64) if ties else RNG.standard_normal(shape)
    dy = RNG.standard_normal((2, 2, 3, 4, 32))
    bits = orc.pool3d_route_bits(x)
    assert bits.shape == (2, 4, 6, 8, 2)
    ref = orc.relu_bwd(orc.pool3d_bwd(x, dy), x)
    assert np.array_equal(orc.pool3d_bwd_bits(bits, dy), ref)
    # at most one bit per window and channel; exactly one where the pooled value is positive
    per_window = orc.pool3d_bwd_bits(bits, np.ones_like(dy)).reshape(2, 2, 2, 3, 2, 4, 2, 32).sum(axis=(2, 4, 6))
    assert np.array_equal(per_window, (orc.pool3d_fwd(x) > 0).astype(np.float64))


def test_pool_against_torch(orc):
    torch = pytest.importorskip("torch")
    x = RNG.standard_normal((1, 4, 6, 4, 5))
    dy = RNG.standard_normal((1, 2, 3, 2, 5))
    xt = torch.tensor(x).permute(0, 4, 1, 2, 3).clone().requires_grad_(True)
    yt = torch.nn.functional.max_pool3d(xt, 2)
    (yt * torch.tensor(dy).permute(0, 4, 1, 2, 3)).sum().backward()
    assert np.array_equal(orc.pool3d_fwd(x), yt.detach().permute(0, 2, 3, 4, 1).numpy())
    assert np.array_equal(orc.pool3d_bwd(x, dy), xt.grad.permute(0, 2, 3, 4, 1).numpy())


# ----------------------------------------------------------------- upconv
def test_upconv_blockwise_definition(orc):
    x = RNG.standard_normal((2, 2, 3, 2, 3))
    w = RNG.standard_normal((2, 2, 2, 3, 4))
    b = RNG.standard_normal(4)
    y = orc.upconv3d_fwd(x, w, b)
    assert y.shape == (2, 4, 6, 4, 4)
    for i in range(2):
        for j in range(2):
            for k in range(2):
                np.testing.assert_allclose(y[:, i::2, j::2, k::2], x @ w[i, j, k] + b, atol=1e-13)


def test_upconv_ones(orc):
    y = orc.upconv3d_fwd(np.ones((1, 2, 2, 2, 5)), np.ones((2, 2, 2, 5, 2)))
    assert np.all(y == 5.0)


def test_upconv_adjoint_and_bilinear(orc):
    x = RNG.standard_normal((2, 2, 3, 2, 3))
    w = RNG.standard_normal((2, 2, 2, 3, 4))
    g = RNG.standard_normal((2, 4, 6, 4, 4))
    ref = np.sum(orc.upconv3d_fwd(x, w) * g)
    assert abs(np.sum(x * orc.upconv3d_bwd_data(g, w)) - ref) < 1e-11 * max(1, abs(ref))
    dW, db = orc.upconv3d_bwd_weight(x, g)
    assert abs(np.sum(w * dW) - ref) < 1e-11 * max(1, abs(ref))
    np.testing.assert_allclose(db, g.reshape(-1, 4).sum(0), atol=1e-12)


def test_upconv_against_torch(orc):
    torch = pytest.importorskip("torch")
    x = RNG.standard_normal((1, 3, 2, 4, 3))
    w = RNG.standard_normal((2, 2, 2, 3, 5))
    b = RNG.standard_normal(5)
    r = RNG.standard_normal((1, 6, 4, 8, 5))
    xt = torch.tensor(x).permute(0, 4, 1, 2, 3).clone().requires_grad_(True)
    wt = torch.tensor(w).permute(3, 4, 0, 1, 2).clone().requires_grad_(True)   # [C_in, C_out, kd, kh, kw]
    bt = torch.tensor(b, requires_grad=True)
    yt = torch.nn.functional.conv_transpose3d(xt, wt, bt, stride=2)
    (yt * torch.tensor(r).permute(0, 4, 1, 2, 3)).sum().backward()
    np.testing.assert_allclose(orc.upconv3d_fwd(x, w, b), yt.detach().permute(0, 2, 3, 4, 1).numpy(), atol=1e-12)
    np.testing.assert_allclose(orc.upconv3d_bwd_data(r, w), xt.grad.permute(0, 2, 3, 4, 1).numpy(), atol=1e-12)
    dW, db = orc.upconv3d_bwd_weight(x, r)
    np.testing.assert_allclose(dW, wt.grad.permute(2, 3, 4, 0, 1).numpy(), atol=1e-11)
    np.testing.assert_allclose(db, bt.grad.numpy(), atol=1e-11)


# ----------------------------------------------------------------- head
def test_head_zero_logits_closed_form(orc):
    """z = 0: loss = ln 3 and dz = (1/3 - onehot)/V."""
    V, C = 10, 4
    a = RNG.standard_normal((V, C))
    lab = (np.arange(V) % 3).astype(np.uint8)
    out = orc.head_softmax_ce(a, np.zeros((C, 3)), np.zeros(3), lab)
    assert abs(out["loss"] - 1.0986122886681098) < 1e-15
    dz = (np.full((V, 3), 1 / 3) - np.eye(3)[lab]) / V
    np.testing.assert_allclose(out["db"], dz.sum(0), atol=1e-15)
    np.testing.assert_allclose(out["dW"], a.T @ dz, atol=1e-15)
    assert np.all(out["da"] == 0)


def test_head_known_logits(orc):
    """One voxel, identity weights: loss = log(sum exp z) - z_label by hand."""
    z = np.array([[1.0, 2.0, 0.5]])
    out = orc.head_softmax_ce(z, np.eye(3), np.zeros(3), np.array([1], dtype=np.uint8))
    lse = math.log(math.exp(1.0) + math.exp(2.0) + math.exp(0.5))
    assert abs(out["loss"] - (lse - 2.0)) < 1e-14
    p = np.exp(z[0] - lse)
    np.testing.assert_allclose(out["da"][0], p - np.array([0, 1, 0]), atol=1e-14)
    np.testing.assert_allclose(out["logits"], z, atol=0)


def test_head_large_logits_are_stable(orc):
    z = np.array([[1000.0, 999.0, -1000.0]])
    out = orc.head_softmax_ce(z, np.eye(3), np.zeros(3), np.array([0], dtype=np.uint8))
    assert abs(out["loss"] - math.log1p(math.exp(-1.0))) < 1e-12


def test_head_finite_differences_and_torch(orc):
    torch = pytest.importorskip("torch")
    V, C = 24, 5
    a = RNG.standard_normal((V, C))
    w = RNG.standard_normal((C, 3))
    b = RNG.standard_normal(3)
    lab = RNG.integers(0, 3, V).astype(np.uint8)
    out = orc.head_softmax_ce(a, w, b, lab)
    at = torch.tensor(a, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    bt = torch.tensor(b, requires_grad=True)
    loss = torch.nn.functional.cross_entropy(at @ wt + bt, torch.tensor(lab.astype(np.int64)))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-13
    np.testing.assert_allclose(out["da"], at.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(out["dW"], wt.grad.numpy(), atol=1e-14)
    np.testing.assert_allclose(out["db"], bt.grad.numpy(), atol=1e-14)
    assert abs(out["db"].sum()) < 1e-15   # rows of dz sum to zero
    eps = 1e-6
    v = RNG.standard_normal(a.shape)
    fd = (orc.head_softmax_ce(a + eps * v, w, b, lab)["loss"] - orc.head_softmax_ce(a - eps * v, w, b, lab)["loss"]) / (2 * eps)
    assert abs(fd - np.sum(out["da"] * v)) < 1e-8


# ----------------------------------------------------------------- bf16 helpers
def test_bf16_helpers(orc):
    bits = np.array([0x3F80, 0xBF80, 0x0000, 0x4049, 0x7F7F], dtype=np.uint16)
    f = orc.bf16_to_f64(bits)
    assert f[0] == 1.0 and f[1] == -1.0 and f[2] == 0.0 and f[3] == 3.140625
    assert f[4] == float(np.float32(3.3895313892515355e38))
    # round-to-nearest-even at the bf16 grid (8 significant bits)
    assert orc.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0            # tie -> even
    assert orc.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6   # tie -> even (up)
    assert orc.round_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0] == 1.0 + 2.0 ** -7
    x = synth.activations(9, (1000,), "bf16").astype(np.float64)
    assert np.array_equal(orc.round_bf16(x), x)
    assert np.array_equal(orc.bf16_to_f64(synth.f32_to_bf16_bits(x.astype(np.float32))), x)
