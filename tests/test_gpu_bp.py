"""GPU parity of the section-4.1 encoder / decoder workload: up-sampling layer, class-weighted
loss, arg-max read-out and the composed training step, against the oracle."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("sp,C,dt", [((1, 4, 4, 4), 16, "bf16"), ((2, 3, 5, 7), 32, "bf16"), ((1, 2, 3, 4), 6, "bf16"),
                                     ((1, 3, 2, 5), 8, "f32"), ((1, 2, 2, 3), 5, "f32"), ((2, 16, 16, 16), 128, "bf16"),
                                     ((1, 1, 1, 1), 16, "bf16")])
def test_upsample(orc, sp, C, dt):
    import torch
    from oracle import bp
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, rel_l2
    N, D, H, W = sp
    x = synth.activations(80, (N, D, H, W, C), dt)
    x = np.maximum(x, 0)                       # a stored ReLU output: about half the entries are zero
    dy = synth.activations(81, (N, 2 * D, 2 * H, 2 * W, C), dt)
    xd, dyd = to_dev(x, dt), to_dev(dy, dt)
    y = empty(dy.shape, dt)
    k3.upsample3d_fwd(xd, y)
    dx, dxm = empty(x.shape, dt), empty(x.shape, dt)
    k3.upsample3d_bwd(dyd, dx)
    k3.upsample3d_bwd(dyd, dxm, x_mask=xd)
    torch.cuda.synchronize()
    assert np.array_equal(to_f64(y), bp.upsample3d_fwd(x.astype(np.float64)))        # a copy: exact
    ref = bp.upsample3d_bwd(dy.astype(np.float64))
    tol = 4e-3 if dt == "bf16" else 1e-6      # one bf16 rounding of an fp32 sum of eight terms
    assert rel_l2(to_f64(dx), ref) < tol
    refm = orc.relu_bwd(ref, x.astype(np.float64))
    assert rel_l2(to_f64(dxm), refm) < tol
    assert np.array_equal(to_f64(dxm) == 0, (refm == 0) | (to_f64(dxm) == 0)) and np.all(to_f64(dxm)[x <= 0] == 0)


def test_upsample_rejects_mismatched_shapes():
    import torch
    from paper_1811_12174_amd import k3
    x = torch.zeros((1, 2, 2, 2, 8), device="cuda", dtype=torch.bfloat16)
    with pytest.raises(k3.K3Error):
        k3.upsample3d_fwd(x, torch.zeros((1, 4, 4, 5, 8), device="cuda", dtype=torch.bfloat16))
    with pytest.raises(k3.K3Error):
        k3.upsample3d_fwd(x, torch.zeros((1, 4, 4, 4, 8), device="cuda", dtype=torch.float32))
    with pytest.raises(k3.K3Error):
        k3.upsample3d_bwd(torch.zeros((1, 4, 4, 4, 16), device="cuda", dtype=torch.bfloat16), x)


@pytest.mark.parametrize("sp,C,dt", [((1, 8, 8, 8), 32, "bf16"), ((2, 5, 7, 9), 128, "bf16"), ((1, 4, 4, 4), 8, "f32"),
                                     ((1, 3, 5, 3), 20, "bf16"), ((1, 7, 9, 11), 16, "bf16")])
def test_weighted_head_and_classification(orc, sp, C, dt):
    import torch
    from oracle import bp
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev, to_f64, empty, rel_l2, TOL
    N, D, H, W = sp
    V = N * D * H * W
    a = synth.activations(82, (N, D, H, W, C), dt)
    wh = synth.head_weights(83, C)
    bh = (synth.normal(synth.SEED, 84, (3,), np.float64) * 0.3).astype(np.float32)
    lab = (synth.uniform(synth.SEED, 85, V) * 3).astype(np.uint8).reshape(N, D, H, W)
    cw = np.array([1.34, 4.63, 0.49], dtype=np.float32)       # the paper's class split, inverted
    ad = to_dev(a, dt)
    whd, bhd, cwd = torch.from_numpy(wh).cuda(), torch.from_numpy(bh).cuda(), torch.from_numpy(cw).cuda()
    labd = torch.from_numpy(lab).cuda()
    loss = torch.full((1,), float("nan"), device="cuda")
    da = empty(a.shape, dt)
    dW = torch.full((C, 3), float("nan"), device="cuda")
    db = torch.full((3,), float("nan"), device="cuda")
    logits = torch.full((V, 3), float("nan"), device="cuda")
    ws = torch.empty(k3.head_workspace_bytes(ad), device="cuda", dtype=torch.uint8)
    k3.head_softmax_wce_fwd_bwd(ad, whd, bhd, labd, cwd, loss, da, dW, db, logits, ws)
    cls = torch.full((N, D, H, W), 9, device="cuda", dtype=torch.uint8)
    logits2 = torch.full((V, 3), float("nan"), device="cuda")
    k3.head_classify(ad, whd, bhd, cls, logits2)
    torch.cuda.synchronize()
    ref = bp.head_softmax_wce(a.astype(np.float64), wh.astype(np.float64), bh.astype(np.float64), lab, cw.astype(np.float64))
    assert abs(loss.item() - ref["loss"]) < 1e-5 * abs(ref["loss"])
    assert rel_l2(to_f64(da), ref["da"]) < TOL[dt]
    assert rel_l2(to_f64(dW), ref["dW"]) < 1e-5
    assert np.abs(to_f64(db) - ref["db"]).max() < 1e-5 * max(1e-3, np.abs(ref["db"]).max()) + 1e-7
    # read-out: logits against the oracle; the class is decided on the kernel's own fp32 logits
    # (exactly), and agrees with the oracle's wherever the oracle's top two are clearly apart
    z = to_f64(logits2)
    rz = ref["logits"].reshape(-1, 3)
    assert rel_l2(z, rz) < 1e-5
    got = cls.cpu().numpy().reshape(-1)
    assert np.array_equal(got, np.argmax(logits2.cpu().numpy(), axis=1).astype(np.uint8))
    top = np.sort(rz, axis=1)
    clear = (top[:, 2] - top[:, 1]) > 1e-4 * (1 + np.abs(top[:, 2]))
    assert clear.mean() > 0.95 and np.array_equal(got[clear], bp.classify(rz)[clear])


def test_classify_ties_take_the_lowest_class():
    import torch
    from paper_1811_12174_amd import k3
    a = torch.zeros((1, 1, 1, 4, 16), device="cuda", dtype=torch.bfloat16)
    wh = torch.zeros((16, 3), device="cuda")
    cls = torch.full((1, 1, 1, 4), 9, device="cuda", dtype=torch.uint8)
    for bias, want in (([0.0, 0.0, 0.0], 0), ([-1.0, 2.0, 2.0], 1), ([1.0, 0.0, 1.0], 0), ([0.0, 0.0, 0.5], 2)):
        k3.head_classify(a, wh, torch.tensor(bias, device="cuda"), cls)
        torch.cuda.synchronize()
        assert cls.cpu().numpy().reshape(-1).tolist() == [want] * 4


def _bp_run(channels, size, n, dt, swap=False, keep=False):
    import torch
    from paper_1811_12174_amd.unet import EncoderDecoder3D
    from gpu_util import to_dev
    params = synth.bp_params(cin=1, channels=channels, dtype=dt, bias_scale=0.05)
    x = synth.volume_field(7, n, size, sigma=2.0, dtype=dt)
    lab = synth.ellipsoid_labels(8, n, size)
    cw = synth.inverse_frequency_class_weights(lab)
    net = EncoderDecoder3D(params, cin=1, channels=channels, dtype=torch.bfloat16 if dt == "bf16" else torch.float32,
                           class_weights=cw)
    out = net.step(to_dev(x, dt), torch.from_numpy(lab).cuda(), swap=swap, keep_acts=keep)
    torch.cuda.synchronize()
    return net, out, params, x, lab, cw


@pytest.mark.parametrize("channels,size,n,dt", [(8, 16, 2, "f32"), (16, 16, 1, "bf16"), (32, 16, 2, "bf16"), (128, 16, 1, "bf16")])
def test_encoder_decoder_step_matches_oracle(orc, channels, size, n, dt):
    from oracle import bp
    from gpu_util import to_f64, rel_l2
    net, (loss, acts), params, x, lab, cw = _bp_run(channels, size, n, dt, keep=True)
    store = orc.round_bf16 if dt == "bf16" else None
    p64 = {k: v.astype(np.float64) for k, v in params.items()}
    rl, rg, ra = bp.bp_step(x.astype(np.float64), lab, p64, cw.astype(np.float64), store=store)
    tol_l, tol_g = (2e-2, 2e-2) if dt == "bf16" else (1e-5, 1e-5)
    assert abs(loss.item() - rl) < tol_l * abs(rl), (loss.item(), rl)
    for k, t in acts.items():
        assert rel_l2(to_f64(t), ra[k], tag=dt) < tol_g, k
    if dt == "bf16":
        _, rg_exact, _ = bp.bp_step(x.astype(np.float64), lab, p64, cw.astype(np.float64))
    for k, g in net.grads().items():
        e = rel_l2(to_f64(g), rg[k], tag=dt)
        bound = 1e-5 if dt != "bf16" else max(2e-2, 3.0 * rel_l2(rg[k], rg_exact[k]))
        assert e < bound, (k, e, bound)
    net.close()


def test_encoder_decoder_step_in_place_equals_the_step_that_keeps_activations():
    """The ordinary step (head gradient in place, pooling from routing bits) against the step that
    hands the activations back, which the oracle comparison above runs: bit-identical."""
    import torch
    from gpu_util import to_dev
    net, (loss, acts), params, x, lab, cw = _bp_run(32, 16, 2, "bf16", keep=True)
    l0 = net.loss.clone()
    g0 = {k: v.clone() for k, v in net.grads().items()}
    for v in net.grads().values():
        v.fill_(float("nan"))
    net.step(to_dev(x, "bf16"), torch.from_numpy(lab).cuda())
    torch.cuda.synchronize()
    assert net.program((2, 16, 16, 16, 1)).rewritten() == {"u2"}
    assert torch.equal(net.loss, l0)
    for k, v in net.grads().items():
        assert torch.equal(v, g0[k]), k
    net.close()


def test_encoder_decoder_at_the_paper_shape():
    """Batch of 8 blocks of 64^3 voxels, 128 channels: swapping is bit-identical, a few SGD steps
    lower the loss, and the arg-max read-out agrees with the logits of the training pass."""
    import torch
    from gpu_util import to_dev
    net, loss, params, x, lab, cw = _bp_run(128, 64, 8, "bf16")
    l0 = net.loss.clone()
    g0 = {k: v.clone() for k, v in net.grads().items()}
    xd, labd = to_dev(x, "bf16"), torch.from_numpy(lab).cuda()
    net.step(xd, labd, swap=True)
    torch.cuda.synchronize()
    assert torch.equal(net.loss, l0) and net.last_run.bytes_out > 0
    for k, v in net.grads().items():
        assert torch.equal(v, g0[k]), k
    losses = []
    for _ in range(6):
        net.step(xd, labd)
        losses.append(net.loss.item())
        net.sgd_step(0.01, 0.9)
    torch.cuda.synchronize()
    assert np.isfinite(losses).all() and losses[-1] < 0.95 * losses[0], losses
    cls = net.classify(xd)
    torch.cuda.synchronize()
    counts = torch.bincount(cls.reshape(-1).long(), minlength=3)
    assert int(counts.sum()) == cls.numel() and int(cls.max()) <= 2
    net.close()


@pytest.mark.parametrize("n,shift", [(0, 0), (1, 0), (15, 0), (16, 0), (17, 3), (4097, 0), ((1 << 20) + 5, 1), (3 * 64 ** 3, 0)])
def test_dice_counts_are_exact(orc, n, shift):
    import torch
    from oracle import bp
    from paper_1811_12174_amd import k3
    pred = (synth.uniform(synth.SEED, 90, n) * 3.2).astype(np.uint8)     # a few values of 3: counted as class 2
    true = (synth.uniform(synth.SEED, 91, n) * 3).astype(np.uint8)
    if n > 10:
        pred[: n // 3] = true[: n // 3]                                   # make the diagonal heavy, like a trained model
    pd = torch.zeros(n + shift, device="cuda", dtype=torch.uint8)[shift:]
    td = torch.zeros(n + shift, device="cuda", dtype=torch.uint8)[shift:]
    pd.copy_(torch.from_numpy(pred)); td.copy_(torch.from_numpy(true))
    counts = torch.full((9,), -1, device="cuda", dtype=torch.int64)
    dice = torch.full((3,), float("nan"), device="cuda")
    k3.dice_coefficients(pd, td, counts, dice)
    torch.cuda.synchronize()
    ref = np.zeros((3, 3), dtype=np.int64)
    np.add.at(ref, (np.minimum(true, 2), np.minimum(pred, 2)), 1)
    if n <= 5000:
        assert np.array_equal(ref, bp.confusion_counts(pred, true))      # the oracle's voxel loop, where it is quick
    assert np.array_equal(counts.cpu().numpy().reshape(3, 3), ref)
    want = bp.dice_coefficients(np.minimum(pred, 2), np.minimum(true, 2))
    assert np.allclose(dice.cpu().numpy(), want, rtol=0, atol=1e-7)
    only = torch.full((9,), -1, device="cuda", dtype=torch.int64)
    k3.dice_coefficients(pd, td, only)                                    # counts only
    torch.cuda.synchronize()
    assert torch.equal(only, counts)


def test_dice_of_the_trained_read_out(orc):
    """End to end: train the encoder/decoder for a few steps, classify, and score with the Dice kernel."""
    import torch
    from oracle import bp
    from paper_1811_12174_amd import k3
    from gpu_util import to_dev
    net, loss, params, x, lab, cw = _bp_run(16, 32, 2, "bf16")
    xd, labd = to_dev(x, "bf16"), torch.from_numpy(lab).cuda()
    for _ in range(5):
        net.step(xd, labd)
        net.sgd_step(0.02, 0.9)
    cls = net.classify(xd)
    counts = torch.zeros(9, device="cuda", dtype=torch.int64)
    dice = torch.zeros(3, device="cuda")
    k3.dice_coefficients(cls, labd, counts, dice)
    torch.cuda.synchronize()
    assert np.allclose(dice.cpu().numpy(), bp.dice_coefficients(cls.cpu().numpy(), lab), atol=1e-7)
    assert int(counts.sum()) == lab.size
    net.close()
