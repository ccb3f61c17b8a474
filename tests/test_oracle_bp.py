"""Pins for the oracle pieces of the section-4.1 encoder / decoder workload (CPU only)."""
import numpy as np

import synth


def _bp():
    from oracle import bp
    return bp


def test_upsample_matches_kronecker_product_and_hand_example(orc):
    bp = _bp()
    x = np.arange(2 * 2 * 1 * 3 * 2, dtype=np.float64).reshape(2, 2, 1, 3, 2)
    y = bp.upsample3d_fwd(x)
    assert y.shape == (2, 4, 2, 6, 2)
    for n in range(2):
        for c in range(2):
            assert np.array_equal(y[n, ..., c], np.kron(x[n, ..., c], np.ones((2, 2, 2))))
    # by hand: output voxel (3, 1, 4) lies in the block of input voxel (1, 0, 2)
    assert y[1, 3, 1, 4, 1] == x[1, 1, 0, 2, 1]
    assert y[0, 0, 0, 1, 0] == x[0, 0, 0, 0, 0] and y[0, 0, 0, 2, 0] == x[0, 0, 0, 1, 0]


def test_upsample_backward_is_the_adjoint(orc):
    bp = _bp()
    rng = np.random.default_rng(5)
    x = rng.normal(size=(1, 2, 3, 2, 3))
    dy = rng.normal(size=(1, 4, 6, 4, 3))
    assert abs((bp.upsample3d_fwd(x) * dy).sum() - (x * bp.upsample3d_bwd(dy)).sum()) < 1e-12
    assert np.array_equal(bp.upsample3d_bwd(np.ones((1, 2, 2, 2, 1))), np.full((1, 1, 1, 1, 1), 8.0))
    # a single one at output voxel (1, 2, 3) lands on input voxel (0, 1, 1) only
    e = np.zeros((1, 2, 4, 4, 1)); e[0, 1, 2, 3, 0] = 1.0
    dx = bp.upsample3d_bwd(e)
    assert dx[0, 0, 1, 1, 0] == 1.0 and dx.sum() == 1.0


def test_weighted_loss_reduces_to_the_unweighted_head(orc):
    """With unit weights the numpy head must agree with the independently written C head."""
    bp = _bp()
    rng = np.random.default_rng(6)
    a = rng.normal(size=(2, 3, 2, 2, 5)); wh = rng.normal(size=(5, 3)); bh = rng.normal(size=3)
    lab = rng.integers(0, 3, size=(2, 3, 2, 2)).astype(np.uint8)
    r0 = orc.head_softmax_ce(a, wh, bh, lab)
    r1 = bp.head_softmax_wce(a, wh, bh, lab, [1.0, 1.0, 1.0])
    assert abs(r0["loss"] - r1["loss"]) < 1e-13
    for k in ("logits", "da", "dW", "db"):
        assert np.allclose(r0[k], r1[k], rtol=1e-12, atol=1e-14), k


def test_weighted_loss_closed_form_and_scaling(orc):
    bp = _bp()
    lab = np.array([0, 1, 1, 2, 2, 2], dtype=np.uint8).reshape(1, 1, 1, 6)
    a = np.zeros((1, 1, 1, 6, 4))
    w = np.array([2.0, 0.5, 3.0])
    r = bp.head_softmax_wce(a, np.zeros((4, 3)), np.zeros(3), lab, w)
    # uniform likelihoods: every voxel costs w[label] * ln 3
    assert abs(r["loss"] - (2.0 + 2 * 0.5 + 3 * 3.0) * np.log(3.0) / 6) < 1e-14
    # dL/db_k = sum_v w_v (1/3 - [label_v = k]) / V
    assert np.allclose(r["db"], [(-2.0 + 12.0 / 3) / 6, (-1.0 + 12.0 / 3) / 6, (-9.0 + 12.0 / 3) / 6])
    # a class with weight zero contributes nothing: same as deleting its voxels (up to the 1/V)
    rng = np.random.default_rng(7)
    a = rng.normal(size=(1, 1, 1, 6, 4)); wh = rng.normal(size=(4, 3)); bh = rng.normal(size=3)
    full = bp.head_softmax_wce(a, wh, bh, lab, [1.0, 1.0, 0.0])
    part = bp.head_softmax_wce(a[..., :3, :], wh, bh, lab[..., :3], [1.0, 1.0, 1.0])
    assert abs(full["loss"] * 6 - part["loss"] * 3) < 1e-13
    assert np.allclose(full["dW"] * 6, part["dW"] * 3) and np.all(full["da"][..., 3:, :] == 0)


def test_weighted_loss_gradients_by_finite_differences(orc):
    bp = _bp()
    rng = np.random.default_rng(8)
    a = rng.normal(size=(1, 2, 2, 1, 3)); wh = rng.normal(size=(3, 3)); bh = rng.normal(size=3)
    lab = rng.integers(0, 3, size=(1, 2, 2, 1)).astype(np.uint8)
    w = np.array([1.3, 4.6, 0.5])
    r = bp.head_softmax_wce(a, wh, bh, lab, w)
    eps = 1e-6
    for name, arr, grad in (("a", a, r["da"]), ("wh", wh, r["dW"]), ("bh", bh, r["db"])):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + eps; lp = bp.head_softmax_wce(a, wh, bh, lab, w)["loss"]
            arr[i] = old - eps; lm = bp.head_softmax_wce(a, wh, bh, lab, w)["loss"]
            arr[i] = old
            assert abs((lp - lm) / (2 * eps) - grad[i]) < 1e-8, (name, i)


def test_classify(orc):
    bp = _bp()
    z = np.array([[0.1, 0.7, 0.2], [3.0, 3.0, -1.0], [-5.0, -4.0, -4.0], [1.0, 1.0, 1.0]]).reshape(1, 1, 2, 2, 3)
    assert bp.classify(z).reshape(-1).tolist() == [1, 0, 1, 0]      # ties: lowest index
    rng = np.random.default_rng(9)
    z = rng.normal(size=(2, 3, 3, 3, 3))
    brute = [max(range(3), key=lambda k: (row[k], -k)) for row in z.reshape(-1, 3)]
    assert bp.classify(z).reshape(-1).tolist() == brute


def test_class_weights_of_the_label_generator():
    lab = synth.ellipsoid_labels(8, 2, 32)
    w = synth.inverse_frequency_class_weights(lab)
    frac = np.bincount(lab.reshape(-1), minlength=3) / lab.size
    assert np.allclose(w * frac * 3, 1.0, rtol=1e-6)     # every class carries a third of the total weight
    assert np.allclose(synth.inverse_frequency_class_weights(np.array([0, 0, 2, 2], dtype=np.uint8)), [2 / 3, 1.0, 2 / 3])


def test_step_gradients_by_finite_differences(orc):
    """The composed step: directional derivative of the loss along a random direction in every
    parameter against the analytic gradients (catches a wrong tensor paired with a gradient,
    a missing ReLU mask or a missing up-sampling adjoint)."""
    bp = _bp()
    params = {k: v.astype(np.float64) for k, v in synth.bp_params(cin=1, channels=4, dtype="f32", bias_scale=0.1).items()}
    x = synth.volume_field(7, 1, 8, sigma=1.5, dtype="f32").astype(np.float64)
    lab = synth.ellipsoid_labels(8, 1, 8)
    cw = synth.inverse_frequency_class_weights(lab).astype(np.float64)
    loss, g, acts = bp.bp_step(x, lab, params, cw)
    assert acts["u2"].shape == (1, 8, 8, 8, 4) and acts["a3"].shape == (1, 2, 2, 2, 4)
    rng = np.random.default_rng(10)
    direction = {k: rng.normal(size=v.shape) for k, v in params.items()}
    analytic = sum(float((g[k] * direction[k]).sum()) for k in params)
    eps = 1e-6
    lp = bp.bp_step(x, lab, {k: params[k] + eps * direction[k] for k in params}, cw)[0]
    lm = bp.bp_step(x, lab, {k: params[k] - eps * direction[k] for k in params}, cw)[0]
    assert abs((lp - lm) / (2 * eps) - analytic) < 1e-6 * max(1.0, abs(analytic)), ((lp - lm) / (2 * eps), analytic)


def test_dice_by_hand_and_special_cases(orc):
    bp = _bp()
    pred = np.array([0, 0, 1, 2, 2, 2, 1, 0], dtype=np.uint8)
    true = np.array([0, 1, 1, 2, 2, 0, 1, 0], dtype=np.uint8)
    # class 0: P = {0,1,7}, T = {0,5,7}, both = {0,7}: 2*2/6.  class 1: P = {2,6}, T = {1,2,6}: 2*2/5.
    # class 2: P = {3,4,5}, T = {3,4}: 2*2/5
    assert np.allclose(bp.dice_coefficients(pred, true), [4 / 6, 4 / 5, 4 / 5])
    c = bp.confusion_counts(pred, true)
    assert c.tolist() == [[2, 0, 1], [1, 2, 0], [0, 0, 2]] and c.sum() == 8
    # the coefficients follow from the confusion matrix: 2 c_kk / (row_k + column_k)
    assert np.allclose(bp.dice_coefficients(pred, true), 2 * np.diag(c) / (c.sum(0) + c.sum(1)))
    assert bp.dice_coefficients(true, true).tolist() == [1.0, 1.0, 1.0]
    assert bp.dice_coefficients(np.zeros(4, np.uint8), np.full(4, 2, np.uint8)).tolist() == [0.0, 1.0, 0.0]
    # symmetric in its arguments
    rng = np.random.default_rng(11)
    a, b = rng.integers(0, 3, 200), rng.integers(0, 3, 200)
    assert np.array_equal(bp.dice_coefficients(a, b), bp.dice_coefficients(b, a))
    assert np.array_equal(bp.confusion_counts(a, b), bp.confusion_counts(b, a).T)
