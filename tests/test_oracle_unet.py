"""Pins for the oracle's U-Net step composition: finite differences of the whole loss
and PyTorch CPU autograd on the same architecture (library special case)."""
import numpy as np
import pytest

import synth
from oracle.unet import unet_step


def _setup(size=8, base=2, levels=3, n=1):
    params = {k: v.astype(np.float64) for k, v in synth.unet_params(base=base, levels=levels, dtype="f32", bias_scale=0.1).items()}
    x = synth.volume_field(7, n, size, sigma=1.5, dtype="f32").astype(np.float64)
    lab = synth.ellipsoid_labels(8, n, size)
    return x, lab, params


def test_unet_finite_differences(orc):
    x, lab, params = _setup()
    loss, grads, _ = unet_step(x, lab, params, base=2, levels=3)
    assert np.isfinite(loss) and loss > 0
    rng = np.random.default_rng(5)
    eps = 1e-6
    for name in ["enc0.conv1.w", "enc1.conv2.w", "enc2.conv1.b", "dec1.up.w", "dec1.up.b", "dec0.conv1.w", "dec0.conv2.b", "head.w", "head.b"]:
        v = rng.standard_normal(params[name].shape)
        pp = dict(params); pm = dict(params)
        pp[name] = params[name] + eps * v
        pm[name] = params[name] - eps * v
        fd = (unet_step(x, lab, pp, 2, 3)[0] - unet_step(x, lab, pm, 2, 3)[0]) / (2 * eps)
        an = np.sum(grads[name] * v)
        assert abs(fd - an) < 2e-6 * max(1e-3, abs(fd)) + 1e-9, (name, fd, an)
    v = rng.standard_normal(x.shape)
    fd = (unet_step(x + eps * v, lab, params, 2, 3)[0] - unet_step(x - eps * v, lab, params, 2, 3)[0]) / (2 * eps)
    assert abs(fd - np.sum(grads["x"] * v)) < 2e-6 * max(1e-3, abs(fd)) + 1e-9


def test_unet_against_torch_autograd(orc):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    x, lab, params = _setup(size=8, base=2, levels=3, n=2)
    loss, grads, acts = unet_step(x, lab, params, base=2, levels=3)
    T = {}
    for k, v in params.items():
        t = torch.tensor(v)
        if k.endswith(".w") and t.dim() == 5:
            t = t.permute(3, 4, 0, 1, 2) if ".up." in k else t.permute(4, 3, 0, 1, 2)
        T[k] = t.clone().requires_grad_(True)
    cur = torch.tensor(x).permute(0, 4, 1, 2, 3)
    skips = []
    for l in range(3):
        cur = torch.relu(F.conv3d(cur, T[f"enc{l}.conv1.w"], T[f"enc{l}.conv1.b"], padding=1))
        cur = torch.relu(F.conv3d(cur, T[f"enc{l}.conv2.w"], T[f"enc{l}.conv2.b"], padding=1))
        if l < 2:
            skips.append(cur)
            cur = F.max_pool3d(cur, 2)
    for l in (1, 0):
        up = F.conv_transpose3d(cur, T[f"dec{l}.up.w"], T[f"dec{l}.up.b"], stride=2)
        cur = torch.cat([skips[l], up], dim=1)
        cur = torch.relu(F.conv3d(cur, T[f"dec{l}.conv1.w"], T[f"dec{l}.conv1.b"], padding=1))
        cur = torch.relu(F.conv3d(cur, T[f"dec{l}.conv2.w"], T[f"dec{l}.conv2.b"], padding=1))
    logits = torch.einsum("ncdhw,ck->nkdhw", cur, T["head.w"]) + T["head.b"].view(1, 3, 1, 1, 1)
    lt = F.cross_entropy(logits, torch.tensor(lab.astype(np.int64)))
    lt.backward()
    assert abs(loss - lt.item()) < 1e-12
    for k in params:
        g = T[k].grad
        if k.endswith(".w") and g.dim() == 5:
            g = g.permute(2, 3, 4, 0, 1) if ".up." in k else g.permute(2, 3, 4, 1, 0)
        np.testing.assert_allclose(grads[k], g.numpy(), atol=1e-11, err_msg=k)


def test_storage_emulation_changes_little(orc):
    import oracle
    x, lab, params = _setup()
    l0, g0, _ = unet_step(x, lab, params, 2, 3)
    l1, g1, _ = unet_step(x, lab, params, 2, 3, store=oracle.round_bf16)
    assert abs(l0 - l1) < 2e-2 * abs(l0)


def test_label_fractions_near_paper_split():
    lab = synth.ellipsoid_labels(8, 8, 48)
    frac = np.bincount(lab.reshape(-1), minlength=3) / lab.size
    # paper section 4.1: 24.9 / 7.2 / 67.9 %; the synthetic masks only need to be in that regime
    assert 0.10 < frac[0] < 0.45 and 0.02 < frac[1] < 0.20 and 0.45 < frac[2] < 0.85, frac
