"""Synthetic tensors with the shapes and statistics of the paper's workloads.

The paper trains on brain-MRI volumes (section 3) and on seismic-like voxel blocks
with a 24.9 / 7.2 / 67.9 % class split (section 4.1).  Neither data set is available
or needed: a smooth random field stands in for a volume and three random ellipsoids
stand in for the label masks.  Weights use He-normal initialisation.  Each tensor is
identified by a small integer stream id so that every consumer regenerates exactly
the same bytes.
"""
import numpy as np

from .rng import SEED, normal, uniform, round_to_bf16


def _finish(a, dtype):
    a = a.astype(np.float32)
    if dtype == "bf16":
        return round_to_bf16(a)
    if dtype == "f32":
        return a
    raise ValueError("dtype must be 'bf16' or 'f32'")


def activations(stream, shape, dtype="bf16", seed=SEED, scale=1.0):
    """i.i.d. N(0, scale^2) tensor (NDHWC), as float32 values representable in `dtype`."""
    return _finish(normal(seed, stream, shape, np.float64) * scale, dtype)


def conv_weights(stream, cin, cout, dtype="bf16", seed=SEED):
    """3x3x3 weights [3][3][3][cin][cout], N(0, 2/(27*cin))."""
    std = np.sqrt(2.0 / (27.0 * cin))
    return _finish(normal(seed, stream, (3, 3, 3, cin, cout), np.float64) * std, dtype)


def upconv_weights(stream, cin, cout, dtype="bf16", seed=SEED):
    """2x2x2 stride-2 transposed-conv weights [2][2][2][cin][cout], N(0, 1/cin)."""
    std = np.sqrt(1.0 / cin)
    return _finish(normal(seed, stream, (2, 2, 2, cin, cout), np.float64) * std, dtype)


def head_weights(stream, cin, classes=3, seed=SEED):
    """1x1x1 head weights [cin][classes], N(0, 1/cin), float32."""
    std = np.sqrt(1.0 / cin)
    return (normal(seed, stream, (cin, classes), np.float64) * std).astype(np.float32)


def volume_field(stream, n, size, sigma=4.0, dtype="bf16", seed=SEED):
    """Smooth single-channel volumes (n, size, size, size, 1) scaled to [0, 1].

    White noise blurred by a separable Gaussian (periodic boundary), then min-max
    scaled per sample."""
    from scipy.ndimage import gaussian_filter1d
    out = np.empty((n, size, size, size, 1), dtype=np.float32)
    for i in range(n):
        f = normal(seed, stream * 1000 + i, (size, size, size), np.float32)
        for ax in range(3):
            f = gaussian_filter1d(f, sigma, axis=ax, mode="wrap")
        lo, hi = float(f.min()), float(f.max())
        out[i, ..., 0] = (f - lo) / (hi - lo)
    return _finish(out, dtype)


def ellipsoid_labels(stream, n, size, seed=SEED):
    """uint8 labels (n, size, size, size) in {0,1,2}: background 2, two ellipsoids of
    class 0, then one of class 1 painted last.  Semi-axes are drawn so the class
    fractions land near the paper's 24.9 / 7.2 / 67.9 % split."""
    lab = np.full((n, size, size, size), 2, dtype=np.uint8)
    g = np.arange(size, dtype=np.float32)
    zz, yy, xx = np.meshgrid(g, g, g, indexing="ij", sparse=True)
    for i in range(n):
        u = uniform(seed, stream * 1000 + i, 18)
        for e in range(3):
            c = (0.25 + 0.5 * u[6 * e:6 * e + 3]) * size
            lo, hi = (0.27, 0.40) if e < 2 else (0.20, 0.30)
            r = (lo + (hi - lo) * u[6 * e + 3:6 * e + 6]) * size
            inside = ((zz - c[0]) / r[0]) ** 2 + ((yy - c[1]) / r[1]) ** 2 + ((xx - c[2]) / r[2]) ** 2 <= 1.0
            lab[i][inside] = 0 if e < 2 else 1
    return lab


def unet_plan(base=32, cin=1, levels=4, classes=3):
    """Layer list of the U-Net: encoder level l has conv1 (C_prev -> F_l) and conv2
    (F_l -> F_l) with F_l = base * 2**l, a 2x2x2 max-pool after every level but the
    last; decoder level l = levels-2 .. 0 has a 2x2x2 stride-2 transposed conv
    (F_{l+1} -> F_l), then conv1 (2 F_l -> F_l) on [skip, up] and conv2 (F_l -> F_l);
    a 1x1x1 head maps F_0 to `classes`.  Returns [(name, kind, cin, cout)]."""
    plan = []
    prev = cin
    for l in range(levels):
        f = base * 2 ** l
        plan.append((f"enc{l}.conv1", "conv", prev, f))
        plan.append((f"enc{l}.conv2", "conv", f, f))
        prev = f
    for l in range(levels - 2, -1, -1):
        f = base * 2 ** l
        plan.append((f"dec{l}.up", "upconv", 2 * f, f))
        plan.append((f"dec{l}.conv1", "conv", 2 * f, f))
        plan.append((f"dec{l}.conv2", "conv", f, f))
    plan.append(("head", "head", base, classes))
    return plan


def unet_params(base=32, cin=1, levels=4, classes=3, dtype="bf16", bias_scale=0.0, seed=SEED, stream0=100):
    """All parameters of the U-Net as float32 arrays: name+'.w', name+'.b'.

    Biases are zero by default (the workload's initialisation); tests pass a nonzero
    bias_scale so the bias paths are exercised."""
    p = {}
    for i, (name, kind, ci, co) in enumerate(unet_plan(base, cin, levels, classes)):
        s = stream0 + 2 * i
        if kind == "conv":
            p[name + ".w"] = conv_weights(s, ci, co, dtype, seed)
        elif kind == "upconv":
            p[name + ".w"] = upconv_weights(s, ci, co, dtype, seed)
        else:
            p[name + ".w"] = head_weights(s, ci, co, seed)
        p[name + ".b"] = (normal(seed, s + 1, (co,), np.float64) * bias_scale).astype(np.float32)
    return p


def bp_plan(cin=1, channels=128, classes=3):
    """Layer list of the section-4.1 encoder / decoder: two encoder layers (3x3x3 conv, 2x2x2
    max-pool) and two decoder layers (3x3x3 conv, up-sampling), `channels` channels per voxel,
    then the per-voxel class likelihoods."""
    return [("enc0.conv", "conv", cin, channels), ("enc1.conv", "conv", channels, channels),
            ("dec1.conv", "conv", channels, channels), ("dec0.conv", "conv", channels, channels),
            ("head", "head", channels, classes)]


def bp_params(cin=1, channels=128, classes=3, dtype="bf16", bias_scale=0.0, seed=SEED, stream0=300):
    p = {}
    for i, (name, kind, ci, co) in enumerate(bp_plan(cin, channels, classes)):
        s = stream0 + 2 * i
        p[name + ".w"] = conv_weights(s, ci, co, dtype, seed) if kind == "conv" else head_weights(s, ci, co, seed)
        p[name + ".b"] = (normal(seed, s + 1, (co,), np.float64) * bias_scale).astype(np.float32)
    return p


def inverse_frequency_class_weights(labels, classes=3):
    """Per-class voxel weights that balance the classes of a label volume: w_k = V / (classes * V_k)
    (1 for a class that does not occur).  With the paper's 24.9 / 7.2 / 67.9 % split this gives
    about 1.34 / 4.63 / 0.49."""
    counts = np.bincount(np.asarray(labels).reshape(-1), minlength=classes).astype(np.float64)
    w = np.where(counts > 0, labels.size / (classes * np.maximum(counts, 1)), 1.0)
    return w.astype(np.float32)
