"""Interpreter of a step program (see program.py) with device-memory accounting.

The interpreter owns the policy of the LMS scheme (section 2.2 of the paper): which device
copies exist when.  It runs the same way against the GPU (the U-Net harness is the backend:
torch allocations, k3 kernels, the k3 swap engine) and against the planner's simulator
(virtual clocks), which is what makes the planner's memory figures exact.

Policy.  All decisions are taken in program order on the host, never by polling the GPU, so
the memory high-water mark is a property of the program and the budget, not of timing:
  * swap_out starts the device-to-host copy; the device copy stays for now.
  * With a budget, every tensor of the step lives in one slab of (budget - fixed part) bytes
    whose address space is managed here (Arena), not by a caching allocator: what fits in the
    planner's simulation fits on the GPU, byte for byte and hole for hole.
  * evict marks the device copy as droppable.  It is dropped when no hole of the slab can take
    an allocation (oldest first, until one can); only then is the compute stream made to wait
    for that tensor's outgoing copy.  With `eager=True` it is dropped at once.
  * prefetch brings a dropped tensor back into a fresh block (`prefetch_start`: the copy
    overlaps the kernels enqueued after it); a tensor that was never dropped is simply kept.
  * wait fences the compute stream behind the copy-in, right before the first reader.
  * A tensor that came back and is evicted again is dropped without a copy: its host copy is
    still valid because stored activations are never rewritten (a tensor that a call rewrites
    in place is offered no gap: Program.gaps).
"""


class OutOfBudget(RuntimeError):
    def __init__(self, call_index, need, used, budget):
        super().__init__(f"device budget exceeded at call {call_index}: need {need} B with {used} B in use "
                         f"of {budget} B and nothing left to evict")
        self.call_index, self.need, self.used, self.budget = call_index, need, used, budget


class Arena:
    """Address space of the step's device slab: best-fit allocation (smallest hole that fits, lowest
    address on ties) with coalescing frees, 512-byte granules.  The same object runs in the GPU
    run and in the planner's simulation, so a plan that fits in simulation fits on the GPU,
    fragmentation included."""
    GRANULE = 512

    def __init__(self, size):
        self.size = max(0, int(size)) // self.GRANULE * self.GRANULE
        self.holes = [(0, self.size)] if self.size else []     # (offset, length), sorted by offset
        self.high_water = 0

    @classmethod
    def rounded(cls, n):
        return (int(n) + cls.GRANULE - 1) // cls.GRANULE * cls.GRANULE

    def alloc(self, n, top=False):
        """Best fit: the smallest hole that takes n bytes.  Large tensors are carved from the low
        end of their hole (lowest hole on ties), small ones (`top`) from the high end (highest hole
        on ties), so the two kinds grow towards each other and small tensors do not end up
        pinning the middle of the room a large one will need."""
        n = self.rounded(n)
        best = None
        for i, (off, ln) in enumerate(self.holes):
            if ln >= n and (best is None or ln < self.holes[best][1] or (top and ln == self.holes[best][1])):
                best = i
        if best is None:
            return None
        off, ln = self.holes[best]
        if ln == n:
            del self.holes[best]
            at = off
        elif top:
            self.holes[best] = (off, ln - n)
            at = off + ln - n
        else:
            self.holes[best] = (off + n, ln - n)
            at = off
        self.high_water = max(self.high_water, at + n)
        return at

    def free(self, off, n):
        n = self.rounded(n)
        lo, hi = 0, len(self.holes)
        while lo < hi:
            mid = (lo + hi) // 2
            if self.holes[mid][0] < off:
                lo = mid + 1
            else:
                hi = mid
        self.holes.insert(lo, (off, n))
        if lo + 1 < len(self.holes) and off + n == self.holes[lo + 1][0]:
            self.holes[lo] = (off, n + self.holes[lo + 1][1])
            del self.holes[lo + 1]
        if lo > 0 and self.holes[lo - 1][0] + self.holes[lo - 1][1] == off:
            self.holes[lo - 1] = (self.holes[lo - 1][0], self.holes[lo - 1][1] + self.holes[lo][1])
            del self.holes[lo]


class Executor:
    """backend interface:
         slab(nbytes) (called once per run when a budget is set), alloc(info, offset) -> block
         (offset into the slab, or None without a budget), free(block),
         call(call, blocks: dict name -> block)
         swap_out(info, block) -> handle, release_after(handle), prefetch_start(handle, block),
         wait_in(handle), evict(handle), release(handle)"""

    def __init__(self, backend, program, budget=None, eager=False, fixed_bytes=0):
        self.be, self.prog = backend, program
        self.budget, self.eager, self.fixed = budget, eager, fixed_bytes
        self.used = fixed_bytes
        self.peak = fixed_bytes
        self.arena = None if budget is None else Arena(budget - fixed_bytes)
        self._off = {}
        self._largest = max((i.nbytes for i in program.tensors.values() if not i.external), default=0)
        self.releases = 0           # device copies dropped while their outgoing copy may still run
        self.bytes_out = self.bytes_in = 0

    def _place(self, t, k):
        """Device block for tensor t: with a budget, an address range of the slab -- dropping the
        oldest droppable device copies until a hole is large enough."""
        info = self.prog.tensors[t]
        off = None
        if self.arena is not None:
            while True:
                off = self.arena.alloc(info.nbytes, top=2 * info.nbytes <= self._largest)
                if off is not None:
                    break
                if not self._droppable:
                    raise OutOfBudget(k, info.nbytes, self.used, self.budget)
                self._drop(self._droppable.pop(0))
            self._off[t] = off
        self.used += info.nbytes
        self.peak = max(self.peak, self.used)
        self._blocks[t] = self.be.alloc(info, off)

    def _unplace(self, t):
        self.be.free(self._blocks.pop(t))
        self.used -= self.prog.tensors[t].nbytes
        if self.arena is not None:
            self.arena.free(self._off.pop(t), self.prog.tensors[t].nbytes)

    def _drop(self, t):
        """Drop the original device copy of a swapped-out tensor (compute waits for the copy-out)."""
        self.be.release_after(self._handle[t])
        self._unplace(t)
        self._where[t] = "host"
        self.releases += 1

    def run(self, instructions, externals):
        prog = self.prog
        self._blocks = dict(externals)
        self._handle, self._where, self._droppable = {}, {}, []
        if self.arena is not None:
            self.be.slab(self.arena.size)
        k = -1
        try:
            for ins in instructions:
                op, arg = ins
                if op == "call":
                    k += 1
                    self.be.call(arg, self._blocks)
                elif op == "alloc":
                    self._place(arg, k + 1)
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
                        self._unplace(arg)
                        self._where[arg] = "host"
                elif op == "prefetch":
                    if self._where[arg] == "device":
                        if arg in self._droppable:
                            self._droppable.remove(arg)   # never left: keep it
                    elif self._where[arg] == "host":
                        self._place(arg, k + 1)
                        self.be.prefetch_start(self._handle[arg], self._blocks[arg])
                        self._where[arg] = "incoming"
                        self.bytes_in += prog.tensors[arg].nbytes
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
        if t in self._blocks:
            self._unplace(t)

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
