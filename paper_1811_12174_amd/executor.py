"""Interpreter of a step program (see program.py) with device-memory accounting.

The interpreter owns the policy of the LMS scheme (section 2.2 of the paper): which device
copies exist when.  It runs the same way against the GPU (the U-Net harness is the backend:
torch allocations, k3 kernels, the k3 swap engine) and against the planner's simulator
(virtual clocks), which is what makes the planner's memory figures exact.

Policy.  All decisions are taken in program order on the host, never by polling the GPU, so
the memory high-water mark is a property of the program and the budget, not of timing:
  * swap_out starts the device-to-host copy; the device copy stays for now.
  * evict marks the device copy as droppable.  It is dropped when an allocation would exceed
    the budget (oldest first); only then is the compute stream made to wait for that tensor's
    outgoing copy.  With `eager=True` it is dropped at once (smallest footprint).
  * prefetch brings a dropped tensor back into a fresh block (`prefetch_start`: the copy
    overlaps the kernels enqueued after it); a tensor that was never dropped is simply kept.
  * wait fences the compute stream behind the copy-in, right before the first reader.
  * A tensor that came back and is evicted again is dropped without a copy: its host copy is
    still valid because stored activations are never rewritten.
"""


class OutOfBudget(RuntimeError):
    def __init__(self, call_index, need, used, budget):
        super().__init__(f"device budget exceeded at call {call_index}: need {need} B with {used} B in use "
                         f"of {budget} B and nothing left to evict")
        self.call_index, self.need, self.used, self.budget = call_index, need, used, budget


class Executor:
    """backend interface:
         alloc(info) -> block, free(block), call(call, blocks: dict name -> block)
         swap_out(info, block) -> handle, release_after(handle), prefetch_start(handle, block),
         wait_in(handle), evict(handle), release(handle)"""

    def __init__(self, backend, program, budget=None, eager=False, fixed_bytes=0):
        self.be, self.prog = backend, program
        self.budget, self.eager, self.fixed = budget, eager, fixed_bytes
        self.used = fixed_bytes
        self.peak = fixed_bytes
        self.releases = 0           # device copies dropped while their outgoing copy may still run
        self.bytes_out = self.bytes_in = 0

    def _reserve(self, need, k):
        while self.budget is not None and self.used + need > self.budget:
            if not self._droppable:
                raise OutOfBudget(k, need, self.used, self.budget)
            self._drop(self._droppable.pop(0))
        self.used += need
        self.peak = max(self.peak, self.used)

    def _drop(self, t):
        """Drop the original device copy of a swapped-out tensor (compute waits for the copy-out)."""
        self.be.release_after(self._handle[t])
        self.be.free(self._blocks.pop(t))
        self.used -= self.prog.tensors[t].nbytes
        self._where[t] = "host"
        self.releases += 1

    def run(self, instructions, externals):
        prog = self.prog
        self._blocks = dict(externals)
        self._handle, self._where, self._droppable = {}, {}, []
        k = -1
        try:
            for ins in instructions:
                op, arg = ins
                if op == "call":
                    k += 1
                    self.be.call(arg, self._blocks)
                elif op == "alloc":
                    info = prog.tensors[arg]
                    self._reserve(info.nbytes, k + 1)
                    self._blocks[arg] = self.be.alloc(info)
                elif op == "free":
                    self._free(arg)
                elif op == "swap_out":
                    info = prog.tensors[arg]
                    self._handle[arg] = self.be.swap_out(info, self._blocks[arg])
                    self._where[arg] = "device"          # original copy, outgoing copy issued
                    self.bytes_out += info.nbytes
                elif op == "evict":
                    if self._where[arg] == "device":
                        if self.eager:
                            self._drop(arg)
                        else:
                            self._droppable.append(arg)
                    elif self._where[arg] == "back":
                        self.be.evict(self._handle[arg])
                        self.be.free(self._blocks.pop(arg))
                        self.used -= prog.tensors[arg].nbytes
                        self._where[arg] = "host"
                elif op == "prefetch":
                    if self._where[arg] == "device":
                        if arg in self._droppable:
                            self._droppable.remove(arg)   # never left: keep it
                    elif self._where[arg] == "host":
                        info = prog.tensors[arg]
                        self._reserve(info.nbytes, k + 1)
                        self._blocks[arg] = self.be.alloc(info)
                        self.be.prefetch_start(self._handle[arg], self._blocks[arg])
                        self._where[arg] = "incoming"
                        self.bytes_in += info.nbytes
                elif op == "wait":
                    if self._where[arg] == "incoming":
                        self.be.wait_in(self._handle[arg])
                        self._where[arg] = "back"
                else:
                    raise ValueError(op)
        finally:
            self._cleanup()
        return self

    def _free(self, t):
        if t in self._handle:
            h = self._handle.pop(t)
            if t in self._droppable:
                self._droppable.remove(t)
            if self._where.get(t) == "device":
                self.be.release_after(h)     # the block may be reused from here on
            self.be.release(h)
            self._where.pop(t, None)
        blk = self._blocks.pop(t, None)
        if blk is not None:
            self.be.free(blk)
            self.used -= self.prog.tensors[t].nbytes

    def _cleanup(self):
        """After a normal run everything is already freed except kept tensors; after an error the
        remaining handles and blocks are released here."""
        self.kept = {}
        for t in list(self._handle):
            h = self._handle.pop(t)
            if self._where.get(t) == "device":
                self.be.release_after(h)
            self.be.release(h)
        for t, blk in list(self._blocks.items()):
            info = self.prog.tensors[t]
            if info.external:
                continue
            if t in self.prog.keep:
                self.kept[t] = blk
            else:
                self.be.free(blk)
        self._blocks = {}
