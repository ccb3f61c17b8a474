"""Oracle pieces of the paper's second workload (section 4.1): the 3-D encoder / decoder
segmentation model whose decoder layers are a 3x3x3 convolution followed by an up-sampling
layer, trained with class-weighted voxels and read out by taking the most likely class.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  Plain numpy, fp64, written from the
definitions:
  * nearest-neighbour up-sampling by 2 per axis: every input voxel is repeated into the
    2x2x2 block of output voxels it covers; its backward is the sum over that block (the
    adjoint).  The paper says "upsampling layer" without naming the interpolation; nearest
    neighbour is the reading taken.
  * class-weighted softmax cross-entropy over three classes: voxel v contributes
    w[label_v] * (-log p[v, label_v]); the sum is divided by the number of voxels.  The paper
    says the weight of voxels is adjusted for the class imbalance without giving the
    normalisation; dividing by the voxel count (not by the sum of weights) is the reading taken.
  * classification = arg-max of the per-voxel likelihoods, lowest class index on ties.
Pinned in tests/test_oracle_bp.py.
"""
import numpy as np

from . import conv3d_fwd, conv3d_bwd_data, conv3d_bwd_weight, relu_bwd, pool3d_fwd, pool3d_bwd


def upsample3d_fwd(x):
    """x: [N, D, H, W, C] -> [N, 2D, 2H, 2W, C]."""
    x = np.asarray(x, dtype=np.float64)
    N, D, H, W, C = x.shape
    y = np.empty((N, 2 * D, 2 * H, 2 * W, C), dtype=np.float64)
    for i in range(2):
        for j in range(2):
            for k in range(2):
                y[:, i::2, j::2, k::2, :] = x
    return y


def upsample3d_bwd(dy):
    """dy: [N, 2D, 2H, 2W, C] -> dx [N, D, H, W, C], dx = sum of dy over each 2x2x2 block."""
    dy = np.asarray(dy, dtype=np.float64)
    dx = np.zeros((dy.shape[0], dy.shape[1] // 2, dy.shape[2] // 2, dy.shape[3] // 2, dy.shape[4]), dtype=np.float64)
    for i in range(2):
        for j in range(2):
            for k in range(2):
                dx += dy[:, i::2, j::2, k::2, :]
    return dx


def head_softmax_wce(a, wh, bh, labels, class_w):
    """1x1x1 head, softmax, class-weighted cross-entropy.  Returns dict(loss, logits, da, dW, db)."""
    a = np.asarray(a, dtype=np.float64)
    C = a.shape[-1]
    A = a.reshape(-1, C)
    V = A.shape[0]
    lab = np.asarray(labels).reshape(-1).astype(np.int64)
    cw = np.asarray(class_w, dtype=np.float64)
    z = A @ np.asarray(wh, dtype=np.float64) + np.asarray(bh, dtype=np.float64)
    zs = z - z.max(axis=1, keepdims=True)
    logp = zs - np.log(np.exp(zs).sum(axis=1, keepdims=True))
    wv = cw[lab]
    loss = float(-(wv * logp[np.arange(V), lab]).sum() / V)
    dz = np.exp(logp)
    dz[np.arange(V), lab] -= 1.0
    dz *= (wv / V)[:, None]
    return {"loss": loss, "logits": z.reshape(a.shape[:-1] + (z.shape[1],)), "da": (dz @ np.asarray(wh, dtype=np.float64).T).reshape(a.shape),
            "dW": A.T @ dz, "db": dz.sum(axis=0)}


def classify(logits):
    """Most likely class per voxel (softmax is monotone, so the arg-max of the logits)."""
    return np.argmax(np.asarray(logits, dtype=np.float64), axis=-1).astype(np.uint8)


def bp_step(x, labels, params, class_w, store=None):
    """One training step of the section-4.1 model: conv+ReLU, pool, conv+ReLU, pool, conv+ReLU,
    up-sample, conv+ReLU, up-sample, head.  Returns (loss, grads, acts)."""
    st = (lambda t: t) if store is None else store
    P = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
    x = np.asarray(x, dtype=np.float64)
    a1 = st(conv3d_fwd(x, P["enc0.conv.w"], P["enc0.conv.b"], relu=True))
    p1 = pool3d_fwd(a1)
    a2 = st(conv3d_fwd(p1, P["enc1.conv.w"], P["enc1.conv.b"], relu=True))
    p2 = pool3d_fwd(a2)
    a3 = st(conv3d_fwd(p2, P["dec1.conv.w"], P["dec1.conv.b"], relu=True))
    u1 = upsample3d_fwd(a3)
    a4 = st(conv3d_fwd(u1, P["dec0.conv.w"], P["dec0.conv.b"], relu=True))
    u2 = upsample3d_fwd(a4)
    hd = head_softmax_wce(u2, P["head.w"], P["head.b"], labels, class_w)
    acts = {"a1": a1, "p1": p1, "a2": a2, "p2": p2, "a3": a3, "u1": u1, "a4": a4, "u2": u2, "logits": hd["logits"]}
    g = {"head.w": hd["dW"], "head.b": hd["db"]}
    gu2 = st(hd["da"])
    ga4 = st(relu_bwd(upsample3d_bwd(gu2), a4))
    g["dec0.conv.w"], g["dec0.conv.b"] = conv3d_bwd_weight(u1, ga4)
    gu1 = st(conv3d_bwd_data(ga4, P["dec0.conv.w"]))
    ga3 = st(relu_bwd(upsample3d_bwd(gu1), a3))
    g["dec1.conv.w"], g["dec1.conv.b"] = conv3d_bwd_weight(p2, ga3)
    gp2 = st(conv3d_bwd_data(ga3, P["dec1.conv.w"]))
    ga2 = st(relu_bwd(pool3d_bwd(a2, gp2), a2))
    g["enc1.conv.w"], g["enc1.conv.b"] = conv3d_bwd_weight(p1, ga2)
    gp1 = st(conv3d_bwd_data(ga2, P["enc1.conv.w"]))
    ga1 = st(relu_bwd(pool3d_bwd(a1, gp1), a1))
    g["enc0.conv.w"], g["enc0.conv.b"] = conv3d_bwd_weight(x, ga1)
    return hd["loss"], g, acts


def confusion_counts(classes, labels, k=3):
    """counts[t, p] = number of voxels with label t that were classified p (plain loop over voxels)."""
    c = np.zeros((k, k), dtype=np.int64)
    for p, t in zip(np.asarray(classes).reshape(-1).tolist(), np.asarray(labels).reshape(-1).tolist()):
        c[min(t, k - 1), min(p, k - 1)] += 1
    return c


def dice_coefficients(classes, labels, k=3):
    """Dice coefficient per class between the predicted and the labelled voxel sets (section 3.1
    lists it among the figures compared between runs):  D_c = 2 |P_c and T_c| / (|P_c| + |T_c|),
    taken as 1 for a class that neither set contains."""
    classes = np.asarray(classes).reshape(-1)
    labels = np.asarray(labels).reshape(-1)
    out = np.empty(k, dtype=np.float64)
    for c in range(k):
        P, T = classes == c, labels == c
        den = int(P.sum()) + int(T.sum())
        out[c] = 1.0 if den == 0 else 2.0 * int((P & T).sum()) / den
    return out
