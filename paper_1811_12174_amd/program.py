"""Static program of one 3-D U-Net training step, and its rewrite for tensor swapping.

The step (forward + backward of the encoder / decoder network of sections 3 and 4.1) is
written down once as a linear list of kernel calls over named tensors with known shapes.
Everything else is derived from that list by static analysis, which is the role the graph
analysis plays in the paper's LMS module (section 2.2): when each tensor is allocated and
freed (liveness), in which idle gaps between two uses it could live in host memory, and --
for a chosen set of gaps -- where the swap-out, the drop of the device copy, the prefetch
and the wait for the prefetch go.  The same instruction stream is executed on the GPU by the
U-Net harness and in virtual time by the planner's simulator, so the memory the planner
predicts is the memory the run uses.

No arithmetic of the network lives here, only shapes, byte counts and operation counts.
"""
from collections import namedtuple


class TensorInfo:
    """kind: "act" (an activation or gradient in the network's dtype), "bits" (one bit per element of an
    activation, a ReLU mask or a pooling layer's routing: uint16 words, one per 16 channels) or "labels"."""
    __slots__ = ("name", "shape", "ebytes", "external", "kind")

    def __init__(self, name, shape, ebytes, external=False, kind="act"):
        self.name, self.shape, self.ebytes, self.external = name, tuple(int(s) for s in shape), ebytes, external
        self.kind = kind

    @property
    def nbytes(self):
        n = self.ebytes
        for s in self.shape:
            n *= s
        return n


class Call:
    """One kernel-level library call.  `args` maps argument names to tensor names (or None) and
    plain values; reads / writes list the activation tensors touched; flops and nbytes are the
    algorithmic operation and HBM byte counts the simulator's cost model uses."""
    __slots__ = ("fn", "layer", "args", "reads", "writes", "flops", "nbytes", "vox", "ci", "co", "allocs", "frees")

    def __init__(self, fn, layer, args, reads, writes, flops, nbytes, vox, ci, co):
        self.fn, self.layer, self.args = fn, layer, args
        self.reads = [r for r in reads if r is not None]
        self.writes = [w for w in writes if w is not None]
        self.flops, self.nbytes, self.vox, self.ci, self.co = flops, nbytes, vox, ci, co
        self.allocs, self.frees = [], []

    def touches(self):
        return self.reads + self.writes


Gap = namedtuple("Gap", "tensor index first last")   # idle between call `first` and call `last`


class Program:
    def __init__(self, ebytes=2):
        self.ebytes = ebytes
        self.tensors = {}
        self.calls = []
        self._pending_allocs = []
        self.keep = set()

    # ---- construction
    def external(self, name, shape, ebytes=None):
        self.tensors[name] = TensorInfo(name, shape, self.ebytes if ebytes is None else ebytes, external=True)
        return name

    def new(self, name, shape):
        assert name not in self.tensors, name
        self.tensors[name] = TensorInfo(name, shape, self.ebytes)
        self._pending_allocs.append(name)
        return name

    def new_bits(self, name, like):
        """The bit mask of the ReLU output `like` (allocated with the same call)."""
        n, d, h, w, c = self.tensors[like].shape
        assert c % 16 == 0 and name not in self.tensors
        self.tensors[name] = TensorInfo(name, (n, d, h, w, c // 16), 2, kind="bits")
        self._pending_allocs.append(name)
        return name

    def _vox(self, name):
        n, d, h, w, _ = self.tensors[name].shape
        return n * d * h * w

    def _nb(self, *names):
        return sum(self.tensors[n].nbytes for n in names if n is not None)

    def _add(self, call):
        call.allocs, self._pending_allocs = self._pending_allocs, []
        self.calls.append(call)

    def conv_fwd(self, layer, x, x2, y, ci, co, relu=True, bits=None):
        v = self._vox(y)
        self._add(Call("conv_fwd", layer, dict(x=x, x2=x2, y=y, relu=relu, bits=bits), [x, x2], [y, bits],
                       2 * 27 * v * ci * co, self._nb(x, x2, y, bits), v, ci, co))

    def conv_wgrad(self, layer, x, x2, g, ci, co):
        v = self._vox(g)
        self._add(Call("conv_wgrad", layer, dict(x=x, x2=x2, g=g), [x, x2, g], [],
                       2 * 27 * v * ci * co, self._nb(x, x2, g), v, ci, co))

    def conv_dgrad(self, layer, g, dx, dx2, mask, ci, co, mask_bits=None):
        """mask: the stored ReLU output dx is masked with; mask_bits: the same as a bit tensor."""
        assert mask is None or mask_bits is None
        v = self._vox(g)
        self._add(Call("conv_dgrad", layer, dict(g=g, dx=dx, dx2=dx2, mask=mask, mask_bits=mask_bits), [g, mask, mask_bits],
                       [dx, dx2], 2 * 27 * v * ci * co, self._nb(g, mask, mask_bits, dx, dx2), v, ci, co))

    def pool_fwd(self, x, y, route=None):
        """route: a bit tensor (new_bits of x) that receives the backward pass's routing."""
        self._add(Call("pool_fwd", None, dict(x=x, y=y, route=route), [x], [y, route], 0, self._nb(x, y, route),
                       self._vox(x), 0, 0))

    def pool_bwd(self, x, dy, add, dx, relu_mask, route=None):
        """With route (the bits pool_fwd wrote) the pass reads those in place of x: x is None, and
        the result is the one of relu_mask=True without add."""
        assert route is None or (x is None and add is None and relu_mask)
        self._add(Call("pool_bwd", None, dict(x=x, dy=dy, add=add, dx=dx, relu_mask=relu_mask, route=route),
                       [x, dy, add, route], [dx], 0, self._nb(x, dy, add, route, dx), self._vox(dx), 0, 0))

    def up_fwd(self, layer, x, y, ci, co):
        v = self._vox(x)
        self._add(Call("up_fwd", layer, dict(x=x, y=y), [x], [y], 2 * 8 * v * ci * co, self._nb(x, y), v, ci, co))

    def up_wgrad(self, layer, x, dy, ci, co):
        v = self._vox(x)
        self._add(Call("up_wgrad", layer, dict(x=x, dy=dy), [x, dy], [], 2 * 8 * v * ci * co, self._nb(x, dy), v, ci, co))

    def up_dgrad(self, layer, dy, dx, mask, ci, co):
        v = self._vox(dx)
        self._add(Call("up_dgrad", layer, dict(dy=dy, dx=dx, mask=mask), [dy, mask], [dx],
                       2 * 8 * v * ci * co, self._nb(dy, dx, mask), v, ci, co))

    def head(self, a, da, c, relu_mask=True):
        """da may be a: the gradient then replaces the activations (see gaps for what that excludes)."""
        v = self._vox(a)
        self._add(Call("head", "head", dict(a=a, da=da, relu_mask=relu_mask), [a, "labels"], [da], 2 * 2 * 3 * v * c,
                       self._nb(a, da) + v, v, c, 3))

    def upsample_fwd(self, x, y):
        self._add(Call("upsample_fwd", None, dict(x=x, y=y), [x], [y], 0, self._nb(x, y), self._vox(y), 0, 0))

    def upsample_bwd(self, dy, dx, mask):
        self._add(Call("upsample_bwd", None, dict(dy=dy, dx=dx, mask=mask), [dy, mask], [dx], 0, self._nb(dy, dx, mask),
                       self._vox(dy), 0, 0))

    # ---- analysis
    def finish(self, keep=()):
        """Liveness: every tensor the step allocates is freed after the last call that touches it
        (tensors named in `keep` are left to the caller)."""
        self.keep = set(keep)
        last = {}
        for k, c in enumerate(self.calls):
            c.frees = []
            for t in c.touches():
                last[t] = k
        for t, k in last.items():
            info = self.tensors[t]
            if not info.external and t not in self.keep:
                self.calls[k].frees.append(t)
        return self

    def uses(self):
        u = {}
        for k, c in enumerate(self.calls):
            for t in c.touches():
                if not u.get(t) or u[t][-1] != k:
                    u.setdefault(t, []).append(k)
        return u

    def rewritten(self):
        """Tensors more than one call writes (a call that works in place)."""
        n = {}
        for c in self.calls:
            for t in set(c.writes):
                n[t] = n.get(t, 0) + 1
        return {t for t, k in n.items() if k > 1}

    def gaps(self, min_calls=3):
        """Idle intervals: consecutive uses of a step-owned tensor at least `min_calls` calls apart.
        A tensor that is rewritten in place has none: the swap scheme copies a tensor out once,
        behind its producer, and relies on that host copy for every later gap."""
        out = []
        rewritten = self.rewritten()
        for t, ks in self.uses().items():
            info = self.tensors[t]
            if info.external or t in self.keep or t in rewritten:
                continue
            for i in range(len(ks) - 1):
                if ks[i + 1] - ks[i] >= min_calls:
                    out.append(Gap(t, i, ks[i], ks[i + 1]))
        return out

    def instructions(self, gaps=(), lead=2, at=None):
        """The linear instruction stream: ("alloc", t), ("call", Call), ("free", t) and, for the
        chosen gaps, ("swap_out", t) after the call that produces t (once per tensor: the host copy
        stays valid because stored activations are never rewritten), ("evict", t) after the last use
        before the gap,
        ("prefetch", t) ahead of the next use -- before the call `at[(tensor, index)]` when given,
        else `lead` calls ahead -- and ("wait", t) right before that use."""
        at = at or {}
        before, after = {}, {}
        by_tensor = {}
        produced = {t: ks[0] for t, ks in self.uses().items()} if gaps else {}
        for g in gaps:
            by_tensor.setdefault(g.tensor, []).append(g)
        for t, gs in by_tensor.items():
            gs.sort(key=lambda g: g.index)
            for j, g in enumerate(gs):
                if j == 0:
                    # the copy only reads the tensor, so it starts right behind the producer and
                    # runs alongside the forward readers
                    after.setdefault(produced[t], []).append(("swap_out", t))
                after.setdefault(g.first, []).append(("evict", t))
                pos = at.get((t, g.index), g.last - max(1, lead))
                pos = min(max(g.first + 1, pos), g.last)
                before.setdefault(pos, []).append((g.last, ("prefetch", t)))
                before.setdefault(g.last, []).append((-1, ("wait", t)))
        out = []
        for k, c in enumerate(self.calls):
            # a prefetch placed at its own reader call (lead 0) first, so that the wait below fences
            # it; then the waits; then the prefetches for later readers in the order these run
            for _, ins in sorted(before.get(k, []), key=lambda e: -2 if e[0] == k else e[0]):
                out.append(ins)
            for t in c.allocs:
                out.append(("alloc", t))
            out.append(("call", c))
            for ins in after.get(k, []):
                out.append(ins)
            for t in c.frees:
                out.append(("free", t))
        return out


def unet_program(base, cin, levels, n, d, h, w, ebytes=2, keep_acts=False):
    """The U-Net step in data-flow order: per encoder level two 3x3x3 conv + ReLU layers and a
    2x2x2 max-pool; per decoder level a 2x2x2 stride-2 transposed conv, the two-source conv over
    [skip, up] and a second conv; the 1x1x1 head with softmax cross-entropy; then the backward
    pass, decoder (level 0 first) and encoder (deepest level first).  Every producer of an
    activation gradient applies the ReLU mask of the tensor it differentiates (mask / relu_mask
    arguments), so no separate ReLU-backward pass exists."""
    L = levels
    if (d | h | w) % (1 << (L - 1)):
        raise ValueError("volume edges must be divisible by 2^(levels-1)")
    p = Program(ebytes)
    F = [base * 2 ** l for l in range(L)]

    def sh(l, c):
        return (n, d >> l, h >> l, w >> l, c)
    p.external("x", sh(0, cin))
    p.external("labels", (n, d, h, w), 1)
    # The first convolution of every level is differentiated through its ReLU by the second one's
    # backward-data pass; with bf16 tensors and channel counts in whole 16s that mask travels as
    # one bit per element, written by the forward pass (1/16 of the bytes in the backward pass).
    use_bits = ebytes == 2 and base % 16 == 0

    def bits_of(t):
        return p.new_bits("b:" + t, t) if use_bits else None
    cur = "x"
    for l in range(L):
        ci = cin if l == 0 else F[l - 1]
        p.conv_fwd(f"enc{l}.conv1", cur, None, p.new(f"a1_{l}", sh(l, F[l])), ci, F[l], bits=bits_of(f"a1_{l}"))
        p.conv_fwd(f"enc{l}.conv2", f"a1_{l}", None, p.new(f"a2_{l}", sh(l, F[l])), F[l], F[l])
        if l < L - 1:
            p.pool_fwd(f"a2_{l}", p.new(f"p_{l}", sh(l + 1, F[l])))
            cur = f"p_{l}"
        else:
            cur = f"a2_{l}"
    below = {}
    for l in range(L - 2, -1, -1):
        below[l] = cur
        p.up_fwd(f"dec{l}.up", cur, p.new(f"up_{l}", sh(l, F[l])), F[l + 1], F[l])
        p.conv_fwd(f"dec{l}.conv1", f"a2_{l}", f"up_{l}", p.new(f"da1_{l}", sh(l, F[l])), 2 * F[l], F[l],
                   bits=bits_of(f"da1_{l}"))
        p.conv_fwd(f"dec{l}.conv2", f"da1_{l}", None, p.new(f"da2_{l}", sh(l, F[l])), F[l], F[l])
        cur = f"da2_{l}"
    # The head's gradient replaces its input, which nothing else reads: one full-resolution tensor
    # less at the step's memory peak (not when the caller wants the activations back).
    if keep_acts:
        p.head(cur, p.new("g:" + cur, p.tensors[cur].shape), F[0])
        g = "g:" + cur
    else:
        p.head(cur, cur, F[0])
        g = cur
    for l in range(0, L - 1):
        Fl = F[l]
        p.conv_wgrad(f"dec{l}.conv2", f"da1_{l}", None, g, Fl, Fl)
        p.conv_dgrad(f"dec{l}.conv2", g, p.new(f"g:da1_{l}", sh(l, Fl)), None, None if use_bits else f"da1_{l}", Fl, Fl,
                     mask_bits=f"b:da1_{l}" if use_bits else None)
        p.conv_wgrad(f"dec{l}.conv1", f"a2_{l}", f"up_{l}", f"g:da1_{l}", 2 * Fl, Fl)
        p.conv_dgrad(f"dec{l}.conv1", f"g:da1_{l}", p.new(f"gs_{l}", sh(l, Fl)), p.new(f"g:up_{l}", sh(l, Fl)), None, 2 * Fl, Fl)
        p.up_wgrad(f"dec{l}.up", below[l], f"g:up_{l}", F[l + 1], Fl)
        p.up_dgrad(f"dec{l}.up", f"g:up_{l}", p.new("g:" + below[l], p.tensors[below[l]].shape), below[l], F[l + 1], Fl)
        g = "g:" + below[l]
    for l in range(L - 1, -1, -1):
        Fl = F[l]
        if l < L - 1:
            p.pool_bwd(f"a2_{l}", g, f"gs_{l}", p.new(f"g:a2_{l}", sh(l, Fl)), True)
            g = f"g:a2_{l}"
        p.conv_wgrad(f"enc{l}.conv2", f"a1_{l}", None, g, Fl, Fl)
        p.conv_dgrad(f"enc{l}.conv2", g, p.new(f"g:a1_{l}", sh(l, Fl)), None, None if use_bits else f"a1_{l}", Fl, Fl,
                     mask_bits=f"b:a1_{l}" if use_bits else None)
        inp = "x" if l == 0 else f"p_{l - 1}"
        ci = cin if l == 0 else F[l - 1]
        p.conv_wgrad(f"enc{l}.conv1", inp, None, f"g:a1_{l}", ci, Fl)
        if l > 0:
            p.conv_dgrad(f"enc{l}.conv1", f"g:a1_{l}", p.new(f"g:p_{l - 1}", sh(l, F[l - 1])), None, None, ci, Fl)
            g = f"g:p_{l - 1}"
    keep = [t for t, i in p.tensors.items() if not i.external and i.kind == "act" and not t.startswith("g")] if keep_acts else []
    return p.finish(keep)


def bp_program(cin, channels, n, d, h, w, ebytes=2, keep_acts=False):
    """The section-4.1 encoder / decoder step: two encoder layers (3x3x3 conv + ReLU, 2x2x2
    max-pool), two decoder layers (3x3x3 conv + ReLU, up-sampling by 2), the per-voxel class
    likelihoods with the class-weighted loss; then the backward pass.  The up-sampling backward
    applies the ReLU mask of the convolution output it differentiates; the head does not (its
    input is an up-sampled tensor, whose gradient goes through that adjoint first)."""
    if (d | h | w) % 4:
        raise ValueError("volume edges must be divisible by 4")
    p = Program(ebytes)
    C = channels

    def sh(l, c):
        return (n, d >> l, h >> l, w >> l, c)
    p.external("x", sh(0, cin))
    p.external("labels", (n, d, h, w), 1)
    # Nothing but its pooling layer reads an encoder activation here, so (bf16, whole 16-channel
    # words) the pooling keeps one routing bit per element and the activation ends with it.
    route = ebytes == 2 and C % 16 == 0
    p.conv_fwd("enc0.conv", "x", None, p.new("a1", sh(0, C)), cin, C)
    p.pool_fwd("a1", p.new("p1", sh(1, C)), route=p.new_bits("r:a1", "a1") if route else None)
    p.conv_fwd("enc1.conv", "p1", None, p.new("a2", sh(1, C)), C, C)
    p.pool_fwd("a2", p.new("p2", sh(2, C)), route=p.new_bits("r:a2", "a2") if route else None)
    p.conv_fwd("dec1.conv", "p2", None, p.new("a3", sh(2, C)), C, C)
    p.upsample_fwd("a3", p.new("u1", sh(1, C)))
    p.conv_fwd("dec0.conv", "u1", None, p.new("a4", sh(1, C)), C, C)
    p.upsample_fwd("a4", p.new("u2", sh(0, C)))
    gu2 = p.new("g:u2", sh(0, C)) if keep_acts else "u2"     # in place unless the activations are wanted back
    p.head("u2", gu2, C, relu_mask=False)
    p.upsample_bwd(gu2, p.new("g:a4", sh(1, C)), "a4")
    p.conv_wgrad("dec0.conv", "u1", None, "g:a4", C, C)
    p.conv_dgrad("dec0.conv", "g:a4", p.new("g:u1", sh(1, C)), None, None, C, C)
    p.upsample_bwd("g:u1", p.new("g:a3", sh(2, C)), "a3")
    p.conv_wgrad("dec1.conv", "p2", None, "g:a3", C, C)
    p.conv_dgrad("dec1.conv", "g:a3", p.new("g:p2", sh(2, C)), None, None, C, C)
    p.pool_bwd(None if route else "a2", "g:p2", None, p.new("g:a2", sh(1, C)), True, route="r:a2" if route else None)
    p.conv_wgrad("enc1.conv", "p1", None, "g:a2", C, C)
    p.conv_dgrad("enc1.conv", "g:a2", p.new("g:p1", sh(1, C)), None, None, C, C)
    p.pool_bwd(None if route else "a1", "g:p1", None, p.new("g:a1", sh(0, C)), True, route="r:a1" if route else None)
    p.conv_wgrad("enc0.conv", "x", None, "g:a1", cin, C)
    keep = [t for t, i in p.tensors.items() if not i.external and i.kind == "act" and not t.startswith("g")] if keep_acts else []
    return p.finish(keep)
