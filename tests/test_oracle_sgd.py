"""Pins for the oracle's weight update and its short training loop (CPU only)."""
import numpy as np

import synth


def test_two_steps_by_hand(orc):
    # w0 = 1, g = 0.5 both steps, lr = 0.1, momentum 0.9, decay 0.01
    # v1 = 0.5 + 0.01*1 = 0.51          w1 = 1 - 0.051 = 0.949
    # v2 = 0.9*0.51 + 0.5 + 0.00949     w2 = 0.949 - 0.1*v2
    w, v = orc.sgd_momentum_step([1.0], [0.0], [0.5], 0.1, 0.9, 0.01)
    assert abs(v[0] - 0.51) < 1e-15 and abs(w[0] - 0.949) < 1e-15
    w, v = orc.sgd_momentum_step(w, v, [0.5], 0.1, 0.9, 0.01)
    assert abs(v[0] - 0.96849) < 1e-14 and abs(w[0] - 0.852151) < 1e-14


def test_constant_gradient_closed_form(orc):
    # v_t = g (1 - mu^t) / (1 - mu);  w_t = w_0 - lr * sum_{k<=t} v_k
    rng = np.random.default_rng(3)
    w0, g = rng.normal(size=7), rng.normal(size=7)
    lr, mu, T = 0.03, 0.8, 25
    w, v = w0.copy(), np.zeros(7)
    for _ in range(T):
        w, v = orc.sgd_momentum_step(w, v, g, lr, mu)
    vt = g * (1 - mu ** T) / (1 - mu)
    sumv = g * (T - mu * (1 - mu ** T) / (1 - mu)) / (1 - mu)
    assert np.allclose(v, vt, rtol=1e-13) and np.allclose(w, w0 - lr * sumv, rtol=1e-12)


def test_plain_sgd_on_a_quadratic_and_pure_decay(orc):
    # f(w) = a/2 w^2, gradient a w: every step multiplies w by (1 - lr a)
    a, lr = np.array([0.5, 2.0, 7.0]), 0.1
    w, v = np.ones(3), np.zeros(3)
    for _ in range(10):
        w, v = orc.sgd_momentum_step(w, v, a * w, lr)
    assert np.allclose(w, (1 - lr * a) ** 10, rtol=1e-13)
    # zero gradient, decay only: the same contraction with a = weight_decay
    w, v = np.ones(3), np.zeros(3)
    for _ in range(10):
        w, v = orc.sgd_momentum_step(w, v, np.zeros(3), lr, 0.0, 0.25)
    assert np.allclose(w, (1 - lr * 0.25) ** 10, rtol=1e-13)


def test_inputs_are_not_modified(orc):
    w0, v0, g = np.ones(4), np.full(4, 2.0), np.full(4, 3.0)
    orc.sgd_momentum_step(w0, v0, g, 0.1, 0.5, 0.1)
    assert (w0 == 1).all() and (v0 == 2).all()


def test_training_run_descends(orc):
    """First step against the first-order prediction L(w - lr g) = L(w) - lr |g|^2 + O(lr^2), which
    fails for a wrong sign or a gradient paired with the wrong parameter; then a short run with
    momentum must lower the loss."""
    from oracle.unet import unet_step, train
    base, levels, size = 2, 2, 8
    params = synth.unet_params(base=base, levels=levels, dtype="f32")
    x = synth.volume_field(7, 1, size, sigma=2.0, dtype="f32").astype(np.float64)
    lab = synth.ellipsoid_labels(8, 1, size)
    l0, g, _ = unet_step(x, lab, params, base=base, levels=levels)
    g2 = sum(float((g[k] ** 2).sum()) for k in params)
    lr = 1e-3 / max(g2, 1e-12) ** 0.5
    losses, P = train(x, lab, params, base, levels, steps=2, lr=lr)
    assert abs(losses[0] - l0) < 1e-15
    pred = -lr * g2
    assert abs((losses[1] - l0) - pred) < 0.05 * abs(pred), (losses, pred)
    losses, _ = train(x, lab, params, base, levels, steps=8, lr=0.05, momentum=0.9)
    assert losses[-1] < 0.9 * losses[0], losses
    assert all(np.isfinite(losses))
