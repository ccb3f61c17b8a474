"""Oracle composition of one 3-D U-Net training step (forward + backward), fp64.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).  The network is the encoder /
decoder family the paper trains (sections 3 and 4.1) in the exact shape the workload
fixes: per encoder level two 3x3x3 conv + ReLU layers then a 2x2x2 max-pool; per
decoder level a 2x2x2 stride-2 transposed conv, channel concatenation [skip, up],
two 3x3x3 conv + ReLU layers; a 1x1x1 head with softmax cross-entropy averaged over
all voxels.  Each step calls the plain operator definitions of this package in the
order the data flows; nothing is fused.

`store` is applied to every tensor a bf16 GPU implementation would write to memory
(activations and activation gradients).  Identity gives the exact fp64 step; passing
`oracle.round_bf16` emulates bf16 storage so a chained GPU run can be compared without
ReLU-sign / arg-max flips dominating the error.
"""
import numpy as np

from . import (conv3d_fwd, conv3d_bwd_data, conv3d_bwd_weight, relu_bwd, pool3d_fwd,
               pool3d_bwd, upconv3d_fwd, upconv3d_bwd_data, upconv3d_bwd_weight,
               head_softmax_ce)


def unet_step(x, labels, params, base, levels=4, store=None):
    """Returns (loss, grads, acts): grads maps every parameter name to its gradient,
    plus 'x' -> dL/dx; acts maps tensor names to forward activations."""
    st = (lambda t: t) if store is None else store
    P = {k: np.asarray(v, dtype=np.float64) for k, v in params.items()}
    acts = {"x": np.asarray(x, dtype=np.float64)}
    cur = acts["x"]
    # ---- forward, encoder
    for l in range(levels):
        a1 = st(conv3d_fwd(cur, P[f"enc{l}.conv1.w"], P[f"enc{l}.conv1.b"], relu=True))
        a2 = st(conv3d_fwd(a1, P[f"enc{l}.conv2.w"], P[f"enc{l}.conv2.b"], relu=True))
        acts[f"enc{l}.a1"], acts[f"enc{l}.a2"] = a1, a2
        if l < levels - 1:
            cur = pool3d_fwd(a2)
            acts[f"enc{l}.pool"] = cur
        else:
            cur = a2
    # ---- forward, decoder
    for l in range(levels - 2, -1, -1):
        up = st(upconv3d_fwd(cur, P[f"dec{l}.up.w"], P[f"dec{l}.up.b"]))
        cat = np.concatenate([acts[f"enc{l}.a2"], up], axis=-1)
        a1 = st(conv3d_fwd(cat, P[f"dec{l}.conv1.w"], P[f"dec{l}.conv1.b"], relu=True))
        a2 = st(conv3d_fwd(a1, P[f"dec{l}.conv2.w"], P[f"dec{l}.conv2.b"], relu=True))
        acts[f"dec{l}.up"], acts[f"dec{l}.a1"], acts[f"dec{l}.a2"] = up, a1, a2
        cur = a2
    hd = head_softmax_ce(cur, P["head.w"], P["head.b"], labels)
    loss = hd["loss"]
    acts["logits"] = hd["logits"]
    grads = {"head.w": hd["dW"], "head.b": hd["db"]}
    d = st(hd["da"])
    skip_grad = {}
    # ---- backward, decoder (level 0 first)
    for l in range(0, levels - 1):
        F = base * 2 ** l
        below = acts[f"dec{l + 1}.a2"] if l + 1 <= levels - 2 else acts[f"enc{levels - 1}.a2"]
        g2 = relu_bwd(d, acts[f"dec{l}.a2"])
        grads[f"dec{l}.conv2.w"], grads[f"dec{l}.conv2.b"] = conv3d_bwd_weight(acts[f"dec{l}.a1"], g2)
        d1 = st(conv3d_bwd_data(g2, P[f"dec{l}.conv2.w"]))
        g1 = relu_bwd(d1, acts[f"dec{l}.a1"])
        cat = np.concatenate([acts[f"enc{l}.a2"], acts[f"dec{l}.up"]], axis=-1)
        grads[f"dec{l}.conv1.w"], grads[f"dec{l}.conv1.b"] = conv3d_bwd_weight(cat, g1)
        dcat = st(conv3d_bwd_data(g1, P[f"dec{l}.conv1.w"]))
        skip_grad[l] = dcat[..., :F]
        dup = dcat[..., F:]
        grads[f"dec{l}.up.w"], grads[f"dec{l}.up.b"] = upconv3d_bwd_weight(below, dup)
        d = st(upconv3d_bwd_data(dup, P[f"dec{l}.up.w"]))
    # ---- backward, encoder (deepest level first)
    for l in range(levels - 1, -1, -1):
        if l < levels - 1:
            d = st(pool3d_bwd(acts[f"enc{l}.a2"], d) + skip_grad[l])
        inp = acts[f"enc{l - 1}.pool"] if l > 0 else acts["x"]
        g2 = relu_bwd(d, acts[f"enc{l}.a2"])
        grads[f"enc{l}.conv2.w"], grads[f"enc{l}.conv2.b"] = conv3d_bwd_weight(acts[f"enc{l}.a1"], g2)
        d1 = st(conv3d_bwd_data(g2, P[f"enc{l}.conv2.w"]))
        g1 = relu_bwd(d1, acts[f"enc{l}.a1"])
        grads[f"enc{l}.conv1.w"], grads[f"enc{l}.conv1.b"] = conv3d_bwd_weight(inp, g1)
        d = st(conv3d_bwd_data(g1, P[f"enc{l}.conv1.w"]))
    grads["x"] = d
    return loss, grads, acts


def train(x, labels, params, base, levels, steps, lr, momentum=0.0, weight_decay=0.0, store=None, store_w=None):
    """A short training run on one fixed batch: `steps` times (step gradient, SGD update of every
    parameter).  Master weights and momentum buffers are fp64; `store_w` (identity, or
    `oracle.round_bf16`) is applied to the convolution weights each step uses, which models a
    bf16 working copy of fp32 master weights; biases and the head stay unrounded.  Returns
    (list of the losses before each update, final master parameters)."""
    from . import sgd_momentum_step
    sw = (lambda t: t) if store_w is None else store_w
    P = {k: np.asarray(v, dtype=np.float64).copy() for k, v in params.items()}
    V = {k: np.zeros_like(v) for k, v in P.items()}
    losses = []
    for _ in range(steps):
        used = {k: (sw(v) if (k.endswith(".w") and not k.startswith("head")) else v) for k, v in P.items()}
        loss, grads, _ = unet_step(x, labels, used, base=base, levels=levels, store=store)
        losses.append(loss)
        for k in P:
            P[k], V[k] = sgd_momentum_step(P[k], V[k], grads[k], lr, momentum, weight_decay)
    return losses, P
