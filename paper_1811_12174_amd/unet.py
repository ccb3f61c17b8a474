"""One 3-D U-Net training step (forward + backward) driven through the k3 C-ABI.

This is the harness that strings the library calls together in data-flow order; all
arithmetic runs in the HIP kernels.  PyTorch supplies device memory and the compute
stream only.  The network is the encoder / decoder family of the paper (sections 3 and
4.1) in the shape the workload fixes: per encoder level two 3x3x3 conv + ReLU layers and
a 2x2x2 max-pool; per decoder level a 2x2x2 stride-2 transposed conv, a virtual channel
concatenation [skip, up] (never materialised: the conv kernels take two sources / two
destinations), two 3x3x3 conv + ReLU layers; a 1x1x1 head with softmax cross-entropy.

The step is a static program (program.py) run by an interpreter (executor.py) for which this
class is the GPU backend.  With swapping on, the step follows the paper's LMS scheme (section
2.2): chosen tensors are copied to pinned host memory on the device-to-host stream after the
last reader before an idle gap, their device copies are dropped when an allocation needs the
room (only then does the compute stream wait for the outgoing copy), and they come back on
the host-to-device stream a few calls ahead of the next reader, overlapping the kernels in
between.  Which gaps are used, and the prefetch lead, come from a plan (planner.py): all idle
gaps of the stored encoder activations, or a selection made for a device-memory budget.
Without swapping, a step that needs more than the budget fails with OutOfBudget (or the
allocator's out-of-memory error); with a plan for that budget it runs.
"""
import torch

from . import k3, planner
from .executor import Executor
from .program import bp_program, unet_program


class StepNet:
    """Parameters, GPU backend of the interpreter and the training step of a network whose step
    program a subclass supplies (`_build_program`)."""

    def __init__(self, params, dtype=torch.bfloat16, device="cuda", class_weights=None):
        """params: dict name -> float32 numpy array, name + '.w' / '.b' per layer; a layer named
        'head' is the 1x1x1 classifier, names ending in '.up' are transposed convolutions, all
        others 3x3x3 convolutions.  class_weights: three per-class voxel weights for the loss
        (None: unweighted)."""
        self.dtype, self.dev = dtype, device
        self.class_w = None if class_weights is None else torch.tensor([float(v) for v in class_weights], device=device,
                                                                       dtype=torch.float32)
        if self.class_w is not None and self.class_w.numel() != 3:
            raise ValueError("the head kernel is written for the paper's three classes")
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
                    self.w[name] = self.work[o:o + n].view(shape)
                else:
                    self.w[name] = self.master[o:o + n].view(shape)
            self.gw[name] = self.gflat[o:o + n].view(shape)
            self.gb[name] = self.gflat[ob:ob + nb]
        if self.work is not None:
            # the bf16 working copy comes from the library's own rounding: an update with a zero
            # step (momentum and gradient buffers are still zero) leaves the master weights as they
            # are and writes their round-to-nearest-even bf16 values
            k3.sgd_momentum_step(self.master, self.mom, self.gflat, 0.0, 0.0, 0.0, w_bf16=self.work)
        self.repack()
        self._ws = None
        self._host = {}        # tensor name -> (pinned host pointer, bytes), kept across steps
        self._deferred = []    # swap handles whose last copy may still be in flight
        self._programs = {}
        self.lms = None
        self.loss = torch.zeros(1, device=device, dtype=torch.float32)
        self.last_stats = {}
        self.last_run = None   # the Executor of the last step (peak bytes, bytes moved, drops)
        self._timing = None
        self._slab = None
        self.copies_only = False   # when set, step() issues the plan's copies but launches no kernel

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

    # ------------------------------------------------------------------ program and plans
    def program(self, x_shape, keep_acts=False):
        """The static step program for an input of this shape (cached)."""
        key = (tuple(x_shape), keep_acts)
        if key not in self._programs:
            self._programs[key] = self._build_program(tuple(x_shape), 2 if self.dtype == torch.bfloat16 else 4, keep_acts)
        return self._programs[key]

    def workspace_bytes(self, prog):
        """Largest scratch buffer any call of the program needs (shapes only; nothing is launched)."""
        def meta(name):
            return None if name is None else torch.empty(prog.tensors[name].shape, device="meta", dtype=self.dtype)
        need = 1 << 20
        for c in prog.calls:
            if c.fn == "conv_wgrad":
                need = max(need, k3.conv3d_bwd_weight_workspace_bytes(meta(c.args["x"]), meta(c.args["g"]), x2=meta(c.args["x2"])))
            elif c.fn == "up_wgrad":
                need = max(need, k3.upconv3d_bwd_weight_workspace_bytes(meta(c.args["x"]), meta(c.args["dy"])))
            elif c.fn == "head":
                need = max(need, k3.head_workspace_bytes(meta(c.args["a"])))
        return need

    def fixed_bytes(self, prog):
        """Device bytes a step holds besides its activations: the parameter arenas (master, momentum,
        gradient, working copy), the packed weights, the scratch buffer and the caller's batch."""
        n = sum(t.numel() * t.element_size() for t in (self.master, self.mom, self.gflat) if t is not None)
        if self.work is not None:
            n += self.work.numel() * 2
        n += sum(t.numel() for t in self.pk.values() if t is not None)
        n += self.workspace_bytes(prog)
        n += sum(i.nbytes for i in prog.tensors.values() if i.external)
        return n

    # ------------------------------------------------------------------ backend of the interpreter
    def slab(self, nbytes):
        """One device buffer for every tensor of a budgeted step (kept across steps)."""
        if self._slab is None or self._slab.numel() != nbytes:
            self._slab = None
            self._slab = torch.empty(nbytes, device=self.dev, dtype=torch.uint8)

    def alloc(self, info, offset):
        dt = torch.int16 if info.kind == "bits" else self.dtype
        if offset is None:
            return torch.empty(info.shape, device=self.dev, dtype=dt)
        return self._slab[offset:offset + info.nbytes].view(dt).view(info.shape)

    def free(self, block):
        pass    # the last reference goes with the interpreter's table entry

    def swap_out(self, info, block):
        host = self._host.get(info.name)
        if host is None or host[1] < info.nbytes:
            if host is not None:
                k3.lms_host_free(host[0])
            host = self._host[info.name] = (k3.lms_host_alloc(info.nbytes), info.nbytes)
        return k3.lms_swap_out(self.lms, block.data_ptr(), info.nbytes, host[0])

    def release_after(self, h):
        k3.lms_release_after(self.lms, h)

    def prefetch_start(self, h, block):
        k3.lms_prefetch_start(self.lms, h, block.data_ptr())

    def wait_in(self, h):
        k3.lms_wait_in(self.lms, h)

    def evict(self, h):
        k3.lms_evict(self.lms, h)

    def release(self, h):
        """Handles are returned to the engine once their last copy has finished; asking earlier
        would block the host behind the GPU."""
        self._deferred.append(h)
        self._drain(False)

    def _drain(self, block):
        keep = []
        for h in self._deferred:
            if not block and k3.lms_handle_state(self.lms, h) in (k3.LMS_OUT_IN_FLIGHT, k3.LMS_IN_IN_FLIGHT):
                keep.append(h)
            else:
                k3.lms_release(self.lms, h)
        self._deferred = keep

    def call(self, c, t):
        if self.copies_only:   # measurement aid: the step's copy traffic without its kernels
            return
        a = c.args
        if c.fn == "conv_fwd":
            if a.get("bits") is None:
                k3.conv3d_fwd(t[a["x"]], self.w[c.layer], self.pk[c.layer], self.b[c.layer], a["relu"], t[a["y"]],
                              x2=t.get(a["x2"]))
            else:
                k3.conv3d_fwd_bits(t[a["x"]], self.w[c.layer], self.pk[c.layer], self.b[c.layer], a["relu"], t[a["y"]],
                                   t[a["bits"]], x2=t.get(a["x2"]))
        elif c.fn == "conv_wgrad":
            # g is the gradient of the layer's pre-activation: every producer of an activation
            # gradient applies the ReLU mask of the tensor it differentiates
            k3.conv3d_bwd_weight(t[a["x"]], t[a["g"]], None, self.gw[c.layer], self.gb[c.layer], self._ws, x2=t.get(a["x2"]))
        elif c.fn == "conv_dgrad":
            if a.get("mask_bits") is None:
                k3.conv3d_bwd_data(t[a["g"]], None, self.w[c.layer], self.pk[c.layer], t[a["dx"]], dx2=t.get(a["dx2"]),
                                   dx_mask=t.get(a["mask"]))
            else:
                k3.conv3d_bwd_data_bits(t[a["g"]], None, self.w[c.layer], self.pk[c.layer], t[a["dx"]], t[a["mask_bits"]],
                                        dx2=t.get(a["dx2"]))
        elif c.fn == "pool_fwd":
            if a.get("route") is None:
                k3.pool3d_fwd(t[a["x"]], t[a["y"]])
            else:
                k3.pool3d_fwd_bits(t[a["x"]], t[a["y"]], t[a["route"]])
        elif c.fn == "pool_bwd":
            if a.get("route") is None:
                k3.pool3d_bwd(t[a["x"]], t[a["dy"]], t.get(a["add"]), t[a["dx"]], relu_mask=a["relu_mask"])
            else:
                k3.pool3d_bwd_bits(t[a["route"]], t[a["dy"]], t[a["dx"]])
        elif c.fn == "up_fwd":
            k3.upconv3d_fwd(t[a["x"]], self.w[c.layer], self.pk[c.layer], self.b[c.layer], t[a["y"]])
        elif c.fn == "up_wgrad":
            k3.upconv3d_bwd_weight(t[a["x"]], t[a["dy"]], self.gw[c.layer], self.gb[c.layer], self._ws)
        elif c.fn == "up_dgrad":
            k3.upconv3d_bwd_data(t[a["dy"]], self.w[c.layer], self.pk[c.layer], t[a["dx"]], dx_mask=t.get(a["mask"]))
        elif c.fn == "head":
            if self.class_w is None:
                k3.head_softmax_ce_fwd_bwd(t[a["a"]], self.w["head"], self.b["head"], t["labels"], self.loss, t[a["da"]],
                                           self.gw["head"], self.gb["head"], None, self._ws, relu_mask=a["relu_mask"])
            else:
                k3.head_softmax_wce_fwd_bwd(t[a["a"]], self.w["head"], self.b["head"], t["labels"], self.class_w, self.loss,
                                            t[a["da"]], self.gw["head"], self.gb["head"], None, self._ws,
                                            relu_mask=a["relu_mask"])
        elif c.fn == "upsample_fwd":
            k3.upsample3d_fwd(t[a["x"]], t[a["y"]])
        elif c.fn == "upsample_bwd":
            k3.upsample3d_bwd(t[a["dy"]], t[a["dx"]], x_mask=t.get(a["mask"]))
        else:
            raise ValueError(c.fn)
        if self._timing is not None:
            ev = torch.cuda.Event(enable_timing=True)
            ev.record()
            self._timing.append(ev)

    # ------------------------------------------------------------------ the step
    def step(self, x, labels, swap=False, budget=None, keep_acts=False, timing=False):
        """Forward + backward on x (N,D,H,W,cin) and uint8 labels (N,D,H,W).

        Fills the gradient buffers and self.loss (device scalar); returns self.loss.
          swap=False        nothing leaves the GPU.
          swap=True         the stored encoder activations spend their idle gaps in host memory, under
                            the smallest budget that selection can run in.
          swap=<Plan>       a plan from planner.plan_for_budget / planner.swap_all.
        budget (bytes; with a plan the default is the budget the plan was made for) bounds the device
        memory of the step: its tensors then live in one slab of budget minus the fixed part (see
        fixed_bytes), and device copies of swapped tensors are dropped only when an allocation finds
        no room, oldest first.
        With keep_acts=True (swap must be off) the forward activations are returned too.
        With timing=True the per-call GPU durations (seconds) are left in self.call_seconds."""
        prog = self.program(x.shape, keep_acts)
        if swap is True:
            swap = self._default_plan(prog)
        plan = swap if swap else None
        if plan is not None and budget is None:
            budget = plan.budget
        if keep_acts and plan is not None:
            raise ValueError("keep_acts needs swap off")
        if plan is not None and self.lms is None:
            self.lms = k3.lms_create(0)
        need = self.workspace_bytes(prog)
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(need, device=self.dev, dtype=torch.uint8)
        if self.lms is not None:
            self._drain(False)
        ins = prog.instructions(plan.gaps, plan.lead, plan.at) if plan is not None else prog.instructions()
        ex = Executor(self, prog, budget=budget, eager=bool(plan is not None and plan.eager), fixed_bytes=self.fixed_bytes(prog))
        self._timing = [] if timing else None
        if timing:
            start = torch.cuda.Event(enable_timing=True)
            start.record()
        ex.run(ins, {"x": x, "labels": labels})
        self.last_run = ex
        if timing:
            torch.cuda.synchronize()
            evs = [start] + self._timing
            self.call_seconds = [evs[i].elapsed_time(evs[i + 1]) * 1e-3 for i in range(len(evs) - 1)]
            self._timing = None
        if self.lms is not None:
            self.last_stats = k3.lms_get_stats(self.lms)
        if keep_acts:
            return self.loss, self._name_acts(ex.kept)
        return self.loss

    def _name_acts(self, kept):
        return dict(kept)

    def _default_plan(self, prog):
        if getattr(prog, "_encoder_plan", None) is None:
            prog._encoder_plan = planner.swap_all(prog, only=self._swap_by_default, fixed_bytes=self.fixed_bytes(prog))
        return prog._encoder_plan

    def reset(self):
        """Wait for the copy streams and return every swap handle (after a step that ended in an error)."""
        if self.lms is not None:
            k3.lms_sync(self.lms)
            self._drain(True)

    def close(self):
        if self.lms is not None:
            torch.cuda.synchronize()
            k3.lms_sync(self.lms)
            self._drain(True)
        for ptr, _ in self._host.values():
            k3.lms_host_free(ptr)
        self._host = {}
        if self.lms is not None:
            k3.lms_destroy(self.lms)
            self.lms = None


class UNet3D(StepNet):
    def __init__(self, params, base=32, cin=1, levels=4, classes=3, dtype=torch.bfloat16, device="cuda", class_weights=None):
        """params: dict name -> float32 numpy array (see synth.unet_params)."""
        if classes != 3:
            raise ValueError("the head kernel is written for the paper's three classes")
        self.base, self.cin, self.levels = base, cin, levels
        super().__init__(params, dtype=dtype, device=device, class_weights=class_weights)

    _swap_by_default = staticmethod(planner.is_encoder_activation)

    def _build_program(self, x_shape, ebytes, keep_acts):
        n, d, h, w, c = x_shape
        if c != self.cin:
            raise ValueError("input channel count differs from the network's")
        return unet_program(self.base, self.cin, self.levels, n, d, h, w, ebytes=ebytes, keep_acts=keep_acts)

    def _name_acts(self, kept):
        names = {}
        for l in range(self.levels):
            names[f"a1_{l}"], names[f"a2_{l}"], names[f"p_{l}"] = f"enc{l}.a1", f"enc{l}.a2", f"enc{l}.pool"
            names[f"up_{l}"], names[f"da1_{l}"], names[f"da2_{l}"] = f"dec{l}.up", f"dec{l}.a1", f"dec{l}.a2"
        return {names[k]: v for k, v in kept.items() if k in names}


class EncoderDecoder3D(StepNet):
    """The section-4.1 model: two (conv, max-pool) encoder layers, two (conv, up-sampling) decoder
    layers, `channels` channels per voxel, three-class likelihoods, class-weighted loss."""

    def __init__(self, params, cin=1, channels=128, dtype=torch.bfloat16, device="cuda", class_weights=None):
        self.cin, self.channels = cin, channels
        super().__init__(params, dtype=dtype, device=device, class_weights=class_weights)

    @staticmethod
    def _swap_by_default(name):
        return name in ("a1", "p1", "a2", "p2", "a3", "u1", "a4")

    def _build_program(self, x_shape, ebytes, keep_acts):
        n, d, h, w, c = x_shape
        if c != self.cin:
            raise ValueError("input channel count differs from the network's")
        return bp_program(self.cin, self.channels, n, d, h, w, ebytes=ebytes, keep_acts=keep_acts)

    def classify(self, x):
        """Inference: forward pass and the most likely class per voxel (uint8), through the same kernels."""
        n, d, h, w, _ = x.shape
        C = self.channels

        def new(l):
            return torch.empty((n, d >> l, h >> l, w >> l, C), device=self.dev, dtype=self.dtype)

        def conv(name, src, dst):
            k3.conv3d_fwd(src, self.w[name], self.pk[name], self.b[name], True, dst)
            return dst
        a1 = conv("enc0.conv", x, new(0))
        p1 = new(1); k3.pool3d_fwd(a1, p1); del a1
        a2 = conv("enc1.conv", p1, new(1)); del p1
        p2 = new(2); k3.pool3d_fwd(a2, p2); del a2
        a3 = conv("dec1.conv", p2, new(2)); del p2
        u1 = new(1); k3.upsample3d_fwd(a3, u1); del a3
        a4 = conv("dec0.conv", u1, new(1)); del u1
        u2 = new(0); k3.upsample3d_fwd(a4, u2); del a4
        cls = torch.empty((n, d, h, w), device=self.dev, dtype=torch.uint8)
        k3.head_classify(u2, self.w["head"], self.b["head"], cls)
        return cls
