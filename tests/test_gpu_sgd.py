"""GPU parity of the weight-update kernel and of short training runs (step + update) against the oracle."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n,shift", [(1, 0), (3, 0), (63, 0), (64, 0), (4097, 0), ((1 << 20) + 3, 0), (4099, 1), (70001, 3)])
@pytest.mark.parametrize("lr,mu,wd,lowp", [(0.1, 0.0, 0.0, False), (0.05, 0.9, 0.0, True), (0.02, 0.8, 0.01, True)])
def test_sgd_kernel_matches_oracle(orc, n, shift, lr, mu, wd, lowp):
    """Three consecutive updates; ragged sizes, and views that start `shift` elements into an
    allocation (misaligned for the 16-byte path)."""
    import torch
    from paper_1811_12174_amd import k3
    w0 = synth.normal(synth.SEED, 300 + n % 97, (n,), np.float64).astype(np.float32)
    w = torch.zeros(n + shift, device="cuda")[shift:]
    v = torch.zeros(n + shift, device="cuda")[shift:]
    g = torch.zeros(n + shift, device="cuda")[shift:]
    lp = torch.zeros(n + shift, device="cuda", dtype=torch.bfloat16)[shift:] if lowp else None
    w.copy_(torch.from_numpy(w0))
    rw, rv = w0.astype(np.float64), np.zeros(n)
    for t in range(3):
        gh = synth.normal(synth.SEED, 400 + t, (n,), np.float64).astype(np.float32)
        g.copy_(torch.from_numpy(gh))
        k3.sgd_momentum_step(w, v, g, lr, mu, wd, w_bf16=lp)
        rw, rv = orc.sgd_momentum_step(rw, rv, gh.astype(np.float64), lr, mu, wd)
    torch.cuda.synchronize()
    gw, gv = w.cpu().numpy().astype(np.float64), v.cpu().numpy().astype(np.float64)
    # fp32 fused multiply-adds against fp64: a few ulp of the operand magnitudes per step
    assert np.max(np.abs(gw - rw)) <= 2e-6 * (1 + np.max(np.abs(rw)))
    assert np.max(np.abs(gv - rv)) <= 2e-6 * (1 + np.max(np.abs(rv)))
    if lowp:
        # the working copy is the rounding of the kernel's own fp32 result: exact
        assert np.array_equal(lp.float().cpu().numpy().astype(np.float64), orc.round_bf16(gw))


def test_sgd_kernel_edge_cases():
    import torch
    from paper_1811_12174_amd import k3
    w = torch.ones(8, device="cuda")
    v = torch.zeros(8, device="cuda")
    g = torch.ones(8, device="cuda")
    k3.sgd_momentum_step(w[:0], v[:0], g[:0], 0.1)     # empty: no-op
    torch.cuda.synchronize()
    assert (w == 1).all()
    with pytest.raises(k3.K3Error):
        k3.sgd_momentum_step(w, v, g, float("nan"))
    k3.sgd_momentum_step(w, v, g, 0.0, 0.5, 0.0)       # lr = 0 leaves w, still updates v
    torch.cuda.synchronize()
    assert (w == 1).all() and (v == 1).all()


def _train_gpu(params, x, lab, base, levels, dt, steps, lr, mu, wd, swap=False):
    import torch
    from paper_1811_12174_amd.unet import UNet3D
    from gpu_util import to_dev
    net = UNet3D(params, base=base, levels=levels, dtype=torch.bfloat16 if dt == "bf16" else torch.float32)
    xd, ld = to_dev(x, dt), torch.from_numpy(lab).cuda()
    losses = []
    for _ in range(steps):
        net.step(xd, ld, swap=swap)
        losses.append(net.loss.clone())
        net.sgd_step(lr, mu, wd)
    torch.cuda.synchronize()
    final = {k: t.clone() for k, t in net.parameters().items()}
    net.close()
    return [float(l.item()) for l in losses], final


@pytest.mark.parametrize("base,levels,size,dt,steps", [(4, 3, 16, "f32", 4), (16, 2, 16, "bf16", 4)])
def test_training_run_matches_oracle(orc, base, levels, size, dt, steps):
    from oracle.unet import train
    from gpu_util import to_f64, rel_l2
    params = synth.unet_params(base=base, levels=levels, dtype=dt)
    x = synth.volume_field(7, 1, size, sigma=2.0, dtype=dt)
    lab = synth.ellipsoid_labels(8, 1, size)
    lr, mu, wd = 0.02, 0.9, 1e-4
    losses, final = _train_gpu(params, x, lab, base, levels, dt, steps, lr, mu, wd)
    st = orc.round_bf16 if dt == "bf16" else None
    rl, rp = train(x.astype(np.float64), lab, params, base, levels, steps, lr, mu, wd, store=st, store_w=st)
    tol = 2e-2 if dt == "bf16" else 1e-4
    for a, b in zip(losses, rl):
        assert abs(a - b) < tol * abs(b), (losses, rl)
    for k in rp:
        # parameters move by lr * (accumulated gradient): compare the movement, not the value
        moved = rel_l2(to_f64(final[k]) - params[k].astype(np.float64), rp[k] - params[k].astype(np.float64), tag=dt)
        assert moved < (8e-2 if dt == "bf16" else 1e-3), (k, moved)


def test_training_run_descends_and_swapping_is_bit_identical():
    """The paper's check that training with and without LMS gives equivalent loss (section 3),
    here in its strongest form: identical bits, for every loss of the run and every final weight."""
    import torch
    base, levels, size, steps = 32, 3, 32, 10
    params = synth.unet_params(base=base, levels=levels, dtype="bf16")
    x = synth.volume_field(7, 2, size, sigma=2.0, dtype="bf16")
    lab = synth.ellipsoid_labels(8, 2, size)
    la, fa = _train_gpu(params, x, lab, base, levels, "bf16", steps, 0.02, 0.9, 0.0, swap=False)
    lb, fb = _train_gpu(params, x, lab, base, levels, "bf16", steps, 0.02, 0.9, 0.0, swap=True)
    print("losses", la)
    assert la == lb
    for k in fa:
        assert torch.equal(fa[k], fb[k]), k
    assert all(np.isfinite(la)) and la[-1] < 0.9 * la[0], la
