"""One 3-D U-Net training step (forward + backward) driven through the k3 C-ABI.

This is the harness that strings the library calls together in data-flow order; all
arithmetic runs in the HIP kernels.  PyTorch supplies device memory and the compute
stream only.  The network is the encoder / decoder family of the paper (sections 3 and
4.1) in the shape the workload fixes: per encoder level two 3x3x3 conv + ReLU layers and
a 2x2x2 max-pool; per decoder level a 2x2x2 stride-2 transposed conv, a virtual channel
concatenation [skip, up] (never materialised: the conv kernels take two sources / two
destinations), two 3x3x3 conv + ReLU layers; a 1x1x1 head with softmax cross-entropy.

With `swap=True` the step follows the paper's LMS scheme (section 2.2): the encoder-side
tensors of every level but the deepest -- the level input, a1, a2 -- leave the GPU on the
device-to-host copy stream as soon as their last forward reader is enqueued, and come
back on the host-to-device stream ahead of their backward (or skip-connection) consumer.
Device copies of swapped tensors are dropped lazily, when the copy is seen to be complete,
so the compute stream never waits for an outgoing copy.

Under a device-memory limit (the situation the paper's LMS exists for: the stored
activations do not fit) an allocation that fails makes the harness wait for the oldest
outgoing copy, drop that tensor's device copy and try again -- the step then runs at the
pace of the host link instead of failing.  Without swapping the same limit ends the step
with an out-of-memory error.
"""
import time

import torch

from . import k3


class _Slot:
    """A stored activation: on the device, on its way out, or on the host."""
    __slots__ = ("name", "t", "shape", "nbytes", "host", "host_bytes", "handle", "out_pending")

    def __init__(self, name):
        self.name = name
        self.t = None
        self.shape = None
        self.nbytes = 0
        self.host = None
        self.host_bytes = 0
        self.handle = None
        self.out_pending = False


class UNet3D:
    def __init__(self, params, base=32, cin=1, levels=4, classes=3, dtype=torch.bfloat16, device="cuda"):
        """params: dict name -> float32 numpy array (see synth.unet_params)."""
        if classes != 3:
            raise ValueError("the head kernel is written for the paper's three classes")
        self.base, self.cin, self.levels, self.dtype, self.dev = base, cin, levels, dtype, device
        self.code = k3.BF16 if dtype == torch.bfloat16 else k3.F32
        self.w, self.b, self.pk, self.gw, self.gb = {}, {}, {}, {}, {}
        self.kind = {}
        # All parameters live in flat arenas so that the weight update is one kernel launch:
        # fp32 master values, their momentum buffers and their gradients at the same element
        # offsets; bf16 networks add a bf16 working copy (what the conv kernels read), also at
        # the same offsets.  Every tensor starts on a 64-element boundary; the gaps stay zero.
        names = sorted({k[:-2] for k in params})
        off, self._span = 0, {}
        for name in names:
            for suf in (".w", ".b"):
                n = int(params[name + suf].size)
                self._span[name + suf] = (off, n)
                off += (n + 63) // 64 * 64
        self.n_params = off
        self.master = torch.zeros(off, device=device, dtype=torch.float32)
        self.mom = torch.zeros(off, device=device, dtype=torch.float32)
        self.gflat = torch.zeros(off, device=device, dtype=torch.float32)
        self.work = torch.zeros(off, device=device, dtype=torch.bfloat16) if dtype == torch.bfloat16 else None
        for name in names:
            o, n = self._span[name + ".w"]
            shape = tuple(params[name + ".w"].shape)
            self.master[o:o + n].copy_(torch.from_numpy(params[name + ".w"]).reshape(-1).to(device).float())
            ob, nb = self._span[name + ".b"]
            self.master[ob:ob + nb].copy_(torch.from_numpy(params[name + ".b"]).reshape(-1).to(device).float())
            self.b[name] = self.master[ob:ob + nb]
            if name == "head":
                self.kind[name] = "head"
                self.w[name] = self.master[o:o + n].view(shape)
            else:
                self.kind[name] = "upconv" if name.endswith(".up") else "conv"
                if self.work is not None:
                    self.work[o:o + n].copy_(self.master[o:o + n])
                    self.w[name] = self.work[o:o + n].view(shape)
                else:
                    self.w[name] = self.master[o:o + n].view(shape)
            self.gw[name] = self.gflat[o:o + n].view(shape)
            self.gb[name] = self.gflat[ob:ob + nb]
        self.repack()
        self._ws = None
        self._slots = {}
        self.lms = None
        self.loss = torch.zeros(1, device=device, dtype=torch.float32)
        self.last_stats = {}
        self.stall_count, self.stall_seconds = 0, 0.0   # allocations that had to wait for an outgoing copy

    # ------------------------------------------------------------------ parameters
    def repack(self):
        """(Re)build the packed weight forms; call after the weights change."""
        for name, kind in self.kind.items():
            if kind == "head":
                continue
            w = self.w[name]
            fn_bytes = k3.conv3d_packed_bytes if kind == "conv" else k3.upconv3d_packed_bytes
            nb = fn_bytes(w.shape[3], w.shape[4], self.code)
            if nb == 0:
                self.pk[name] = None
                continue
            if self.pk.get(name) is None:
                self.pk[name] = torch.empty(nb, device=self.dev, dtype=torch.uint8)
            (k3.conv3d_pack_weights if kind == "conv" else k3.upconv3d_pack_weights)(w, self.pk[name])

    def grads(self):
        out = {}
        for name in self.w:
            out[name + ".w"] = self.gw[name]
            out[name + ".b"] = self.gb[name]
        return out

    def sgd_step(self, lr, momentum=0.0, weight_decay=0.0):
        """SGD(-momentum) update of every parameter from the gradients of the last step(): one
        launch over the parameter arena, then the packed weight forms are rebuilt."""
        k3.sgd_momentum_step(self.master, self.mom, self.gflat, lr, momentum, weight_decay, w_bf16=self.work)
        self.repack()

    def parameters(self):
        """name -> fp32 master tensor (views into the arena)."""
        out = {}
        for key, (o, n) in self._span.items():
            name = key[:-2]
            shape = self.w[name].shape if key.endswith(".w") else self.b[name].shape
            out[key] = self.master[o:o + n].view(shape)
        return out

    # ------------------------------------------------------------------ helpers
    def _workspace(self, nbytes):
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = None
            self._ws = torch.empty(max(nbytes, 1 << 20), device=self.dev, dtype=torch.uint8)
        return self._ws

    def _empty(self, shape):
        """Device tensor; when the allocator is out of memory, reclaim swapped-out tensors and retry."""
        while True:
            try:
                return torch.empty(tuple(shape), device=self.dev, dtype=self.dtype)
            except torch.cuda.OutOfMemoryError:
                if not self._reclaim():
                    raise

    def _new(self, like_shape, c):
        n, d, h, w, _ = like_shape
        return self._empty((n, d, h, w, c))

    def _conv(self, name, x, x2=None, relu=True):
        y = self._new(x.shape, self.w[name].shape[4])
        k3.conv3d_fwd(x, self.w[name], self.pk[name], self.b[name], relu, y, x2=x2)
        return y

    def _conv_bwd(self, name, x, x2, g, need_dx=True, dx_mask=None):
        """Weight / bias gradients of layer `name`, and dx (split like the inputs).

        g is the gradient of the layer's pre-activation: every producer of an activation
        gradient (head, pool backward, transposed-conv backward, conv backward-data) applies
        the ReLU mask of the tensor it differentiates, so no mask is read here.  dx_mask is
        the stored ReLU output that the first input x is (None when x is not a ReLU output)."""
        ws = self._workspace(k3.conv3d_bwd_weight_workspace_bytes(x, g, x2=x2))
        k3.conv3d_bwd_weight(x, g, None, self.gw[name], self.gb[name], ws, x2=x2)
        if not need_dx:
            return None, None
        dx = self._empty(x.shape)
        dx2 = self._empty(x2.shape) if x2 is not None else None
        k3.conv3d_bwd_data(g, None, self.w[name], self.pk[name], dx, dx2=dx2, dx_mask=dx_mask)
        return dx, dx2

    # ------------------------------------------------------------------ swapping
    def _slot(self, name):
        s = self._slots.get(name)
        if s is None:
            s = self._slots[name] = _Slot(name)
        return s

    def _swap_out(self, name, t):
        s = self._slot(name)
        s.t, s.shape, s.nbytes = t, tuple(t.shape), t.numel() * t.element_size()
        if self.lms is None:
            return
        if s.host is None or s.host_bytes < s.nbytes:
            if s.host is not None:
                k3.lms_host_free(s.host)
            s.host, s.host_bytes = k3.lms_host_alloc(s.nbytes), s.nbytes
        s.handle = k3.lms_swap_out(self.lms, t.data_ptr(), s.nbytes, s.host)
        s.out_pending = True

    def _poll(self):
        """Drop device copies whose outgoing copy has completed (never blocks)."""
        if self.lms is None:
            return
        for s in self._slots.values():
            if s.out_pending and k3.lms_swap_out_done(self.lms, s.handle):
                s.out_pending = False
                s.t = None

    def _reclaim(self):
        """Free device memory held by tensors that are on their way to the host: drop every copy
        that has completed, else block on the oldest outgoing copy.  False when nothing can be freed."""
        if self.lms is None:
            return False
        pending = [s for s in self._slots.values() if s.out_pending]
        if not pending:
            return False
        self.stall_count += 1
        t0 = time.perf_counter()
        while True:
            done = [s for s in pending if k3.lms_swap_out_done(self.lms, s.handle)]
            if done:
                break
            time.sleep(0.0002)
        for s in done:
            s.out_pending = False
            s.t = None
        self.stall_seconds += time.perf_counter() - t0
        return True

    def _prefetch(self, name):
        """Start bringing a swapped tensor back (no-op while it is still on the device)."""
        s = self._slots[name]
        if s.t is not None or self.lms is None:
            s.out_pending = False
            return
        s.t = self._empty(s.shape)
        k3.lms_prefetch_in(self.lms, s.handle, s.t.data_ptr())

    def _get(self, name):
        s = self._slots[name]
        if s.t is None:
            self._prefetch(name)
        return s.t

    def _drop(self, name):
        s = self._slots[name]
        if s.handle is not None and self.lms is not None:
            k3.lms_release(self.lms, s.handle)
        s.handle, s.t, s.out_pending = None, None, False

    def reset(self):
        """Drop every stored activation and swap handle (after a step that ended in an error)."""
        if self.lms is not None:
            k3.lms_sync(self.lms)
        for s in self._slots.values():
            if s.handle is not None and self.lms is not None:
                k3.lms_release(self.lms, s.handle)
            s.handle, s.t, s.out_pending = None, None, False
        self._ws = None

    def close(self):
        for s in self._slots.values():
            if s.handle is not None and self.lms is not None:
                k3.lms_release(self.lms, s.handle)
                s.handle = None
            if s.host is not None:
                k3.lms_host_free(s.host)
                s.host = None
        if self.lms is not None:
            k3.lms_destroy(self.lms)
            self.lms = None

    # ------------------------------------------------------------------ the step
    def step(self, x, labels, swap=False, prefetch_distance=2, keep_acts=False):
        """Forward + backward on x (N,D,H,W,cin) and uint8 labels (N,D,H,W).

        Fills the gradient buffers and self.loss (device scalar); returns self.loss.
        With keep_acts=True (swap must be off) the forward activations are returned too."""
        L = self.levels
        if swap and self.lms is None:
            self.lms = k3.lms_create(0)
        if not swap and self.lms is not None:
            k3.lms_sync(self.lms)
        lms_saved = self.lms
        if not swap:
            self.lms = None
        acts = {}
        try:
            # ---------------- forward, encoder
            cur = x
            for l in range(L):
                a1 = self._conv(f"enc{l}.conv1", cur)
                a2 = self._conv(f"enc{l}.conv2", a1)
                swap_level = l < L - 1
                self._slot(f"in{l}").t = cur
                if swap_level:
                    self._swap_out(f"in{l}", cur)
                    self._swap_out(f"a1_{l}", a1)
                else:
                    self._slot(f"a1_{l}").t = a1
                if l < L - 1:
                    pooled = self._empty((a2.shape[0], a2.shape[1] // 2, a2.shape[2] // 2, a2.shape[3] // 2, a2.shape[4]))
                    k3.pool3d_fwd(a2, pooled)
                    self._swap_out(f"a2_{l}", a2)
                    nxt = pooled
                else:
                    self._slot(f"a2_{l}").t = a2
                    nxt = a2
                if keep_acts:
                    acts[f"enc{l}.a1"], acts[f"enc{l}.a2"] = a1, a2
                    if l < L - 1:
                        acts[f"enc{l}.pool"] = nxt
                del a1, a2, cur
                cur = nxt
                self._poll()
            del nxt
            # ---------------- forward, decoder
            if L >= 2:
                self._prefetch(f"a2_{L - 2}")
            for l in range(L - 2, -1, -1):
                if l >= 1:
                    self._prefetch(f"a2_{l - 1}")   # one level ahead of its skip-connection reader
                name = f"dec{l}.up"
                up = self._empty((cur.shape[0], cur.shape[1] * 2, cur.shape[2] * 2, cur.shape[3] * 2, self.w[name].shape[4]))
                k3.upconv3d_fwd(cur, self.w[name], self.pk[name], self.b[name], up)
                skip = self._get(f"a2_{l}")
                a1 = self._conv(f"dec{l}.conv1", skip, x2=up)
                a2 = self._conv(f"dec{l}.conv2", a1)
                self._slot(f"dbelow{l}").t = cur
                self._slot(f"dup{l}").t = up
                self._slot(f"da1_{l}").t = a1
                # a2 is kept only as the input of the next transposed conv (slot dbelow) or of the
                # head: its own backward needs the gradient mask only, which the producer of that
                # gradient applies
                if keep_acts:
                    acts[f"dec{l}.up"], acts[f"dec{l}.a1"], acts[f"dec{l}.a2"] = up, a1, a2
                del up, a1, skip, cur
                cur = a2
                del a2
                self._poll()
            # ---------------- head: loss and the gradient of the last activation
            d = self._empty(cur.shape)
            ws = self._workspace(k3.head_workspace_bytes(cur))
            k3.head_softmax_ce_fwd_bwd(cur, self.w["head"], self.b["head"], labels, self.loss, d,
                                       self.gw["head"], self.gb["head"], None, ws, relu_mask=True)
            del cur
            # ---------------- backward: stage list, with prefetches issued `prefetch_distance` stages ahead
            stages = [("dec", l) for l in range(0, L - 1)] + [("enc", l) for l in range(L - 1, -1, -1)]

            def needs(stage):
                kind, l = stage
                if kind == "enc" and l < L - 1:
                    return [f"a1_{l}", f"in{l}"]
                return []
            issued = set()
            skip_grad = {}
            for si, stage in enumerate(stages):
                for sj in range(si, min(si + prefetch_distance + 1, len(stages))):
                    for nm in needs(stages[sj]):
                        if nm not in issued:
                            self._prefetch(nm)
                            issued.add(nm)
                kind, l = stage
                if kind == "dec":
                    a1 = self._slots[f"da1_{l}"].t
                    up, below = self._slots[f"dup{l}"].t, self._slots[f"dbelow{l}"].t
                    skip = self._get(f"a2_{l}")
                    # d already carries the ReLU mask of a2 (applied by its producer)
                    d1, _ = self._conv_bwd(f"dec{l}.conv2", a1, None, d, dx_mask=a1)
                    del d, a1
                    self._slots[f"da1_{l}"].t = None   # not read again: free it before the next allocations
                    dskip, dup = self._conv_bwd(f"dec{l}.conv1", skip, up, d1)
                    del d1
                    skip_grad[l] = dskip
                    name = f"dec{l}.up"
                    ws = self._workspace(k3.upconv3d_bwd_weight_workspace_bytes(below, dup))
                    k3.upconv3d_bwd_weight(below, dup, self.gw[name], self.gb[name], ws)
                    d = self._empty(below.shape)
                    k3.upconv3d_bwd_data(dup, self.w[name], self.pk[name], d, dx_mask=below)
                    del dup, dskip, up, below, skip
                    for nm in (f"da1_{l}", f"dup{l}", f"dbelow{l}"):
                        self._slots[nm].t = None
                else:
                    a2 = self._get(f"a2_{l}")
                    if l < L - 1:
                        dd = self._empty(a2.shape)
                        k3.pool3d_bwd(a2, d, skip_grad.pop(l), dd, relu_mask=True)
                        d = dd
                        del dd
                    a1 = self._get(f"a1_{l}")
                    d1, _ = self._conv_bwd(f"enc{l}.conv2", a1, None, d, dx_mask=a1)
                    del d
                    inp = self._get(f"in{l}")
                    d, _ = self._conv_bwd(f"enc{l}.conv1", inp, None, d1, need_dx=(l > 0))
                    del d1, a1, a2, inp
                    for nm in (f"a2_{l}", f"a1_{l}", f"in{l}"):
                        self._drop(nm)
                self._poll()
            if self.lms is not None:
                st = k3.lms_get_stats(self.lms)
                self.last_stats = st
        finally:
            self.lms = lms_saved
        return (self.loss, acts) if keep_acts else self.loss
