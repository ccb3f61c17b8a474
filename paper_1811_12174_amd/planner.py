"""Swap planner: which tensors of a step leave the GPU, and how far ahead they come back.

The paper's LMS module analyses the training graph before the run and inserts swap-out /
swap-in nodes, tuned by a few parameters per model and resolution (section 2.2; section 3
speaks of the optimal parameter settings per image resolution without listing them).  Here
the same job is done on the static step program: given a device-memory budget the planner
picks the idle gaps during which tensors live in host memory, and the prefetch lead, so that
the step fits the budget with the least predicted time.  Every candidate plan is judged by
running the real interpreter (executor.py) on a backend of virtual clocks: a compute stream,
a device-to-host stream and a host-to-device stream with the event ordering of the swap
engine.  The memory figures of that run are exact (the GPU run executes the same
instruction stream under the same accounting); the times come from a per-kernel cost model
and are estimates.

Selection is greedy: simulate; where the budget is first exceeded, add the gap spanning that
call that frees the most bytes (ties: the longest gap); repeat until the step fits.  A budget
that can hold the whole step selects nothing, so the overhead goes to zero as the budget
grows, and rises with the resolution at a fixed budget the way the paper reports it.
"""
from .executor import Executor, OutOfBudget

# Sustained rates measured on one MI355X with this library's kernels at U-Net layer sizes
# (FLOP/s for the matrix-core convolutions by narrower channel count; bytes/s for the
# HBM-bound kernels), and the pinned-memory host link with both directions busy.
CONV_RATE = {"conv_fwd": (0.62e15, 1.10e15, 1.27e15), "conv_dgrad": (0.55e15, 1.05e15, 1.25e15),
             "conv_wgrad": (0.50e15, 1.20e15, 1.27e15)}
STREAM_RATE = {"pool_fwd": 5.4e12, "pool_bwd": 5.4e12, "up_fwd": 4.0e12, "up_wgrad": 5.1e12, "up_dgrad": 2.8e12,
               "head": 3.5e12, "first_fwd": 3.1e12, "first_wgrad": 3.3e12, "upsample_fwd": 5.0e12, "upsample_bwd": 5.0e12}
LAUNCH_SECONDS = 12e-6
LINK_ONE_BYTES_PER_S = 55e9     # one copy direction busy
LINK_BOTH_BYTES_PER_S = 48.7e9  # each direction, both busy


def kernel_seconds(call):
    """Cost model of one call."""
    if call.fn in CONV_RATE:
        if call.ci < 16:   # first layer: HBM-bound gather kernels
            rate = STREAM_RATE["first_fwd" if call.fn == "conv_fwd" else "first_wgrad"]
            return LAUNCH_SECONDS + call.nbytes / rate
        c = min(call.ci, call.co)
        r = CONV_RATE[call.fn][0 if c < 64 else (1 if c < 128 else 2)]
        return LAUNCH_SECONDS + max(call.flops / r, call.nbytes / 4.0e12)
    return LAUNCH_SECONDS + call.nbytes / STREAM_RATE[call.fn]


class _Copy:
    __slots__ = ("ready", "dep", "left", "end")

    def __init__(self, ready, nbytes, dep=None):
        self.ready, self.dep, self.left, self.end = ready, dep, float(nbytes), None


class SimBackend:
    """Virtual-time backend: a compute clock and the two copy streams with the swap engine's
    ordering rules.  Each copy stream is a FIFO; a copy starts when its predecessor is done, the
    compute stream has reached the point it was issued at and (copy-in) the copy-out of the same
    tensor has finished.  The link is shared: a direction moves link_one bytes/s while the other
    is idle and link_both while both are busy (measured: 55 and 48.7 GB/s), so copy end times
    are resolved lazily, when the compute stream asks for them (a wait, or the end of the step)."""

    def __init__(self, seconds_of=kernel_seconds, link=None, durations=None, link_one=LINK_ONE_BYTES_PER_S,
                 link_both=LINK_BOTH_BYTES_PER_S):
        self.tc = 0.0
        self.stall = 0.0
        self.seconds_of, self.durations = seconds_of, durations
        self.r1, self.r2 = (link, link) if link is not None else (link_one, link_both)
        self._n = 0
        self.timeline = []     # compute clock after each call
        self._q = ([], [])     # pending copies: device-to-host, host-to-device (FIFO each)
        self._t = 0.0          # both streams are simulated up to here
        self.copy_end = 0.0    # end of the last finished copy

    def slab(self, nbytes):
        pass

    def alloc(self, info, offset):
        return info.name

    def free(self, block):
        pass

    def call(self, call, blocks):
        for t in call.touches():
            assert t in blocks, (call.fn, call.layer, t, "is not on the device")
        d = self.durations[self._n] if self.durations is not None else self.seconds_of(call)
        self._n += 1
        self.tc += d
        self.timeline.append(self.tc)

    # ---- the two copy streams
    def _advance(self, until, target=None):
        """Simulate both streams up to time `until` (no copy is issued meanwhile), or, with a
        target, until that copy has finished."""
        inf = float("inf")
        while True:
            heads = [q[0] if q else None for q in self._q]
            if heads[0] is None and heads[1] is None:
                break
            starts = []
            for h in heads:
                if h is None:
                    starts.append(inf)
                elif h.dep is not None and h.dep.end is None:
                    starts.append(inf)          # its copy-out is still queued on the other stream
                else:
                    starts.append(max(h.ready, h.dep.end if h.dep is not None else 0.0))
            active = [st <= self._t for st in starts]
            rate = self.r2 if (active[0] and active[1]) else self.r1
            nxt = until
            for h, st, a in zip(heads, starts, active):
                if a:
                    nxt = min(nxt, self._t + h.left / rate)
                elif st < inf:
                    nxt = min(nxt, st)
            if nxt == inf or nxt < self._t:
                break
            dt = nxt - self._t
            self._t = nxt
            for q, h, a in zip(self._q, heads, active):
                if a:
                    h.left -= dt * rate
                    if h.left <= 1e-3:
                        h.end = nxt
                        self.copy_end = max(self.copy_end, nxt)
                        q.pop(0)
            if target is not None and target.end is not None:
                return
            if self._t >= until:
                return
        if until < inf:
            self._t = max(self._t, until)

    def _end_of(self, c):
        self._advance(self.tc)
        if c.end is None:
            self._advance(float("inf"), target=c)
        return c.end

    def _wait(self, until):
        if until > self.tc:
            self.stall += until - self.tc
            self.tc = until

    def swap_out(self, info, block):
        c = _Copy(self.tc, info.nbytes)
        self._advance(self.tc)
        self._q[0].append(c)
        return {"out": c, "in": None, "bytes": info.nbytes}

    def release_after(self, h):
        self._wait(self._end_of(h["out"]))

    def prefetch_start(self, h, block):
        c = _Copy(self.tc, h["bytes"], dep=h["out"])
        self._advance(self.tc)
        self._q[1].append(c)
        h["in"] = c

    def wait_in(self, h):
        self._wait(self._end_of(h["in"]))

    def evict(self, h):
        self._wait(self._end_of(h["in"]))

    def release(self, h):
        pass

    @property
    def seconds(self):
        self._advance(self.tc)
        self._advance(float("inf"))
        return max(self.tc, self.copy_end)


class Plan:
    """gaps: the idle gaps spent in host memory; at: (tensor, gap index) -> call before which the
    prefetch is issued (gaps not listed use `lead` calls ahead of the reader)."""

    def __init__(self, gaps, lead, eager=False, at=None):
        self.gaps, self.lead, self.eager, self.at = list(gaps), lead, eager, dict(at or {})
        self.peak_bytes = self.seconds = self.stall_seconds = self.bytes_out = self.bytes_in = None
        self.no_swap_seconds = None
        self.budget = None      # the device budget the plan was made for

    def describe(self):
        names = sorted({g.tensor for g in self.gaps})
        leads = sorted(g.last - self.at.get((g.tensor, g.index), g.last - self.lead) for g in self.gaps)
        return {"swapped_tensors": names, "gaps": len(self.gaps), "prefetch_lead_calls": leads,
                "predicted_peak_gb": round(self.peak_bytes / 1e9, 3), "predicted_ms": round(self.seconds * 1e3, 2),
                "predicted_no_swap_ms": round(self.no_swap_seconds * 1e3, 2),
                "predicted_stall_ms": round(self.stall_seconds * 1e3, 2),
                "bytes_out": self.bytes_out, "bytes_in": self.bytes_in}


def simulate(program, gaps=(), lead=2, budget=None, eager=False, fixed_bytes=0, durations=None, at=None):
    """One virtual run; returns (executor, backend).  Raises OutOfBudget when the plan does not fit."""
    be = SimBackend(durations=durations)
    ex = Executor(be, program, budget=budget, eager=eager, fixed_bytes=fixed_bytes)
    ex.run(program.instructions(gaps, lead, at), {t: t for t, i in program.tensors.items() if i.external})
    return ex, be


def _fill(plan, ex, be):
    plan.peak_bytes, plan.seconds, plan.stall_seconds = ex.peak, be.seconds, be.stall
    plan.bytes_out, plan.bytes_in = ex.bytes_out, ex.bytes_in
    return plan


def swap_all(program, fixed_bytes=0, min_gap_calls=3, durations=None, only=None):
    """The plan that swaps without being asked to fit a budget: every idle gap (of the tensors
    whose names `only` accepts, when given) is spent in host memory.  Its peak_bytes is the
    smallest footprint that selection can reach (device copies dropped the moment they are
    swapped out, prefetches one call ahead); the plan is meant to run under that figure as the
    budget, where copies are dropped only when an allocation needs the room, and its prefetch
    points are advanced as far as that budget allows."""
    gaps = [g for g in program.gaps(min_gap_calls) if only is None or only(g.tensor)]
    floor = simulate(program, gaps, 1, None, True, fixed_bytes, durations)[0].peak

    def attempt(gs, at=None):
        try:
            return simulate(program, gs, 1, floor, False, fixed_bytes, durations, at), None
        except OutOfBudget as e:
            return None, e
    ok, err = attempt(gaps)
    while ok is None:      # the byte floor may not be reachable in address space: holes do not always line up
        floor = int(floor * 1.02)
        ok, err = attempt(gaps)
    at, ok = _advance_prefetches(program, gaps, attempt, ok)
    plan = _fill(Plan(gaps, 1, at=at), ok[0], ok[1])
    plan.budget = floor
    plan.no_swap_seconds = simulate(program, fixed_bytes=fixed_bytes, durations=durations)[1].seconds
    return plan


def is_encoder_activation(name):
    """The forward activations of the encoder: what a swap of the stored feature maps moves."""
    return name.startswith(("a1_", "a2_", "p_"))


def _advance_prefetches(program, chosen, attempt, ok):
    """In the order the readers run, move each gap's prefetch to the earliest call that still
    fits the budget and lowers the predicted time.  attempt(gaps, at) -> ((executor, backend)
    or None, error); ok is the result for the starting point (every prefetch one call ahead)."""
    at = {}
    for g in sorted(chosen, key=lambda g: g.last):
        best_pos = None
        for pos in range(g.last - 2, g.first, -1):
            trial = dict(at)
            trial[(g.tensor, g.index)] = pos
            r, _ = attempt(chosen, trial)
            if r is None:
                break
            if r[1].seconds < ok[1].seconds:
                ok, best_pos = r, pos
        if best_pos is not None:
            at[(g.tensor, g.index)] = best_pos
    return at, ok


def plan_for_budget(program, budget, fixed_bytes=0, min_gap_calls=3, durations=None):
    """Selection of gaps and prefetch points for a device budget, judged by simulation.
      1. Selection (prefetch one call ahead, which leaves every gap the most room): while the step
         does not fit, every gap that is idle at the failing call is tried; one that makes the
         step fit with the least predicted time is taken, else the one that moves the failure
         furthest down the program (ties: most bytes).
      2. Pruning: a gap whose removal keeps the step within budget and does not slow it is dropped.
      3. Prefetch points: in the order the readers run, each gap's prefetch is moved to the
         earliest call that still fits the budget and lowers the predicted time (copies come back
         in that order on the one host-to-device stream).
    Raises OutOfBudget when no selection fits."""
    all_gaps = program.gaps(min_gap_calls)
    base = simulate(program, fixed_bytes=fixed_bytes, durations=durations)[1].seconds

    def attempt(gaps, at=None):
        try:
            return simulate(program, gaps, 1, budget, False, fixed_bytes, durations, at), None
        except OutOfBudget as e:
            return None, e
    chosen = []
    ok, err = attempt(chosen)
    while ok is None:
        k = err.call_index
        have = {(g.tensor, g.index) for g in chosen}
        cands = [g for g in all_gaps if g.first < k < max(g.first + 1, g.last - 1) and (g.tensor, g.index) not in have]
        if not cands:
            raise err
        fits, moves = [], []
        for g in cands:
            r, e = attempt(chosen + [g])
            if r is not None:
                fits.append((r[1].seconds, -program.tensors[g.tensor].nbytes, g, r))
            else:
                moves.append((e.call_index, program.tensors[g.tensor].nbytes, g, e))
        if fits:
            _, _, g, ok = min(fits, key=lambda f: f[:2])
            chosen.append(g)
            break
        _, _, g, err = max(moves, key=lambda m: m[:2])
        chosen.append(g)
    for g in sorted(chosen, key=lambda g: -program.tensors[g.tensor].nbytes):
        rest = [c for c in chosen if c is not g]
        r, _ = attempt(rest)
        if r is not None and r[1].seconds <= ok[1].seconds:
            chosen, ok = rest, r
    at, ok = _advance_prefetches(program, chosen, attempt, ok)
    plan = _fill(Plan(chosen, 1, at=at), ok[0], ok[1])
    plan.budget = budget
    plan.no_swap_seconds = base
    return plan
