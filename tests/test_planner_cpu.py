"""Host-only tests of the step program, the interpreter's memory accounting and the swap planner."""
import pytest

from paper_1811_12174_amd import planner
from paper_1811_12174_amd.executor import Executor, OutOfBudget
from paper_1811_12174_amd.program import bp_program, unet_program


def _prog(levels=3, base=8, n=1, s=16):
    return unet_program(base, 1, levels, n, s, s, s)


@pytest.mark.parametrize("levels", [1, 2, 3, 4])
def test_program_is_well_formed(levels):
    """Every call finds its tensors on the device (the simulator asserts it), every step-owned
    tensor is allocated once and freed once after its last use, nothing is left at the end."""
    p = _prog(levels)
    # per level: 2 conv + (pool) forward, 2 x (wgrad + dgrad) (+ pool) backward, minus the input's dgrad;
    # per decoder level: up + 2 conv forward, 3 x (wgrad + dgrad) backward; the head
    assert len(p.calls) == 6 * levels - 1 + 2 * (levels - 1) + 9 * (levels - 1) + 1
    ins = p.instructions()
    allocs = [a for op, a in ins if op == "alloc"]
    frees = [a for op, a in ins if op == "free"]
    owned = [t for t, i in p.tensors.items() if not i.external]
    assert sorted(allocs) == sorted(owned) == sorted(frees)
    pos = {(op, a if op != "call" else id(a)): k for k, (op, a) in enumerate(ins)}
    for k, (op, a) in enumerate(ins):
        if op == "call":
            for t in a.touches():
                if not p.tensors[t].external:
                    assert pos[("alloc", t)] < k < pos[("free", t)]
    ex, be = planner.simulate(p, fixed_bytes=123)
    assert ex.used == 123 and ex.peak > 123


def test_single_level_peak_by_hand():
    # x -> a1 -> a2 -> head(g:a2) -> [a2 freed] wgrad2, dgrad2 (g:a1) -> [g:a2, a1... freed] wgrad1
    # live sets: {a1}, {a1,a2}, {a1,a2,g:a2} = 3 tensors, then {a1,g:a2,g:a1} = 3: peak is 3 tensors
    p = unet_program(8, 1, 1, 2, 8, 8, 8)
    one = 2 * 8 * 8 * 8 * 8 * 2
    assert planner.simulate(p)[0].peak == 3 * one


def test_gaps_of_the_stored_activations():
    p = _prog(3)
    gaps = {(g.tensor, g.index): g for g in p.gaps()}
    uses = p.uses()
    # a1_0: written by conv1, read by conv2, then idle until its weight-gradient / mask use in the last stage
    assert uses["a1_0"][:2] == [0, 1] and ("a1_0", 1) in gaps and gaps[("a1_0", 1)].last > len(p.calls) - 6
    # a2_0 (skip connection): idle encoder -> decoder forward, and again decoder backward -> pool backward
    a2 = [(g.first, g.last) for k, g in sorted(gaps.items()) if k[0] == "a2_0"]
    names = [[(p.calls[a].fn, p.calls[a].layer), (p.calls[b].fn, p.calls[b].layer)] for a, b in a2]
    assert names == [[("pool_fwd", None), ("conv_fwd", "dec0.conv1")],
                     [("conv_fwd", "dec0.conv1"), ("conv_wgrad", "dec0.conv1")],
                     [("conv_wgrad", "dec0.conv1"), ("pool_bwd", None)]]
    assert all(not p.tensors[g.tensor].external for g in gaps.values())


def test_encoder_decoder_program_keeps_routing_bits_instead_of_pooled_activations():
    """bf16 with whole 16-channel words: the encoder activations end with their pooling call (the
    backward pooling reads the routing bits, 1/16 of the bytes), so the step's peak is lower than
    in fp32 accounting scaled to the same element size; with 8 channels the activations stay."""
    p = bp_program(1, 32, 2, 16, 16, 16, ebytes=2)
    uses = p.uses()
    pool1 = next(k for k, c in enumerate(p.calls) if c.fn == "pool_fwd")
    assert uses["a1"][-1] == pool1 and p.tensors["r:a1"].kind == "bits"
    assert p.tensors["r:a1"].nbytes * 16 == p.tensors["a1"].nbytes
    back = [c for c in p.calls if c.fn == "pool_bwd"]
    assert [c.args["x"] for c in back] == [None, None] and [c.args["route"] for c in back] == ["r:a2", "r:a1"]
    assert all("a1" not in c.reads and "a2" not in c.reads for c in back)
    ins = p.instructions()
    assert sorted(a for op, a in ins if op == "alloc") == sorted(t for t, i in p.tensors.items() if not i.external)
    plain = bp_program(1, 8, 2, 16, 16, 16, ebytes=2)          # 8 channels: no whole word, x-reading pooling
    assert all(c.args["route"] is None for c in plain.calls if c.fn.startswith("pool"))
    assert plain.uses()["a1"][-1] > pool1
    peak = planner.simulate(p)[0].peak
    peak_plain = planner.simulate(plain)[0].peak * 4            # same program at 32 channels, activations kept
    assert peak < peak_plain


def test_head_gradient_replaces_its_input_and_that_tensor_is_never_swapped():
    """Without keep_acts the head writes its gradient over the last activation: one full-resolution
    tensor less at the peak (which sits at the head otherwise), and the rewritten tensor is offered
    no gap, whatever the minimum length, because a swapped tensor is copied out once only."""
    p = unet_program(8, 1, 3, 1, 16, 16, 16)
    kept = unet_program(8, 1, 3, 1, 16, 16, 16, keep_acts=True)
    head = next(c for c in p.calls if c.fn == "head")
    assert head.args["a"] == head.args["da"] == "da2_0" and "g:da2_0" not in p.tensors
    assert p.rewritten() == {"da2_0"} and kept.rewritten() == set()
    assert all(g.tensor != "da2_0" for g in p.gaps(1)) and any(g.tensor == "da2_0" for g in kept.gaps(1)) is False
    # bytes held while each call runs, from the instruction stream; with a separate gradient tensor
    # the head call would hold one more full-resolution tensor and be the step's peak
    p = unet_program(16, 1, 3, 1, 16, 16, 16)
    held, cur = {}, 0
    for op, a in p.instructions():
        if op == "alloc":
            cur += p.tensors[a].nbytes
        elif op == "free":
            cur -= p.tensors[a].nbytes
        elif op == "call":
            held[(a.fn, a.layer)] = cur
    peak = planner.simulate(p)[0].peak
    assert peak == max(held.values())
    assert held[("head", "head")] <= peak < held[("head", "head")] + p.tensors["da2_0"].nbytes
    q = bp_program(1, 32, 2, 16, 16, 16)
    assert q.rewritten() == {"u2"} and "g:u2" not in q.tensors
    assert next(c for c in q.calls if c.fn == "upsample_bwd").args["dy"] == "u2"


def test_rewrite_places_swap_instructions():
    p = _prog(3)
    gs = [g for g in p.gaps() if g.tensor in ("a1_0", "a2_0")]
    ins = p.instructions(gs, lead=2)
    ops = [(op, a) for op, a in ins if op != "call" and a in ("a1_0", "a2_0")]
    assert sum(1 for op, a in ops if op == "swap_out") == 2            # once per tensor, however many gaps
    assert sum(1 for op, a in ops if op == "evict") == len(gs) == sum(1 for op, a in ops if op == "prefetch")
    # per tensor the order is alloc, swap_out, (evict, prefetch, wait)*, free
    for t in ("a1_0", "a2_0"):
        seq = [op for op, a in ops if a == t]
        assert seq[0] == "alloc" and seq[1] == "swap_out" and seq[-1] == "free"
        body = seq[2:-1]
        assert body == ["evict", "prefetch", "wait"] * (len(body) // 3)
    # a wait sits directly in front of (the allocations of) the call that reads the tensor
    for k, (op, a) in enumerate(ins):
        if op == "wait":
            nxt = next(x for x in ins[k:] if x[0] == "call")[1]
            assert a in nxt.touches()


def test_budget_is_respected_and_loose_budgets_swap_nothing():
    p = unet_program(32, 1, 4, 1, 64, 64, 64)
    need = planner.simulate(p)[0].peak
    plan = planner.plan_for_budget(p, need)
    assert plan.gaps == [] and plan.bytes_out == 0 and plan.seconds == plan.no_swap_seconds
    last_time = plan.seconds
    for frac in (0.95, 0.85, 0.75):
        plan = planner.plan_for_budget(p, int(frac * need))
        assert plan.peak_bytes <= int(frac * need) and plan.gaps
        assert plan.seconds >= plan.no_swap_seconds
        # the executor under that budget, on a fresh simulator, reproduces the plan's figures
        ex, be = planner.simulate(p, plan.gaps, plan.lead, int(frac * need), at=plan.at)
        assert (ex.peak, ex.bytes_out, ex.bytes_in) == (plan.peak_bytes, plan.bytes_out, plan.bytes_in)
        assert abs(be.seconds - plan.seconds) < 1e-12
        last_time = plan.seconds
    with pytest.raises(OutOfBudget):
        planner.plan_for_budget(p, int(0.3 * need))
    with pytest.raises(OutOfBudget):
        planner.simulate(p, budget=need - 1)


def test_fixed_bytes_count_against_the_budget():
    p = _prog(3)
    need = planner.simulate(p)[0].peak
    assert planner.simulate(p, fixed_bytes=1000)[0].peak == need + 1000
    with pytest.raises(OutOfBudget):
        planner.simulate(p, budget=need + 999, fixed_bytes=1000)
    planner.simulate(p, budget=need + 1000, fixed_bytes=1000)


def test_lazy_and_eager_drops():
    p = unet_program(32, 1, 4, 1, 64, 64, 64)
    gaps = [g for g in p.gaps() if planner.is_encoder_activation(g.tensor)]
    lazy, _ = planner.simulate(p, gaps, 2)                       # no budget: nothing is ever dropped
    eager, be_e = planner.simulate(p, gaps, 1, eager=True)
    none, be_n = planner.simulate(p)
    assert lazy.peak == none.peak and lazy.releases == 0 and lazy.bytes_in == 0 and lazy.bytes_out > 0
    assert eager.peak < none.peak and eager.releases > 0 and eager.bytes_in > 0
    # the plan that swaps all of them runs in (nearly) the eager footprint -- the byte floor, or some
    # percent more where the holes of the slab do not line up -- with drops only where needed
    plan = planner.swap_all(p, only=planner.is_encoder_activation)
    assert eager.peak <= plan.budget <= 1.2 * eager.peak and plan.peak_bytes <= plan.budget < none.peak
    assert plan.seconds <= be_e.seconds + 1e-12
    ex, be = planner.simulate(p, plan.gaps, plan.lead, plan.budget, at=plan.at)
    assert ex.peak == plan.peak_bytes and abs(be.seconds - plan.seconds) < 1e-12
    assert ex.arena.high_water <= plan.budget


def test_arena_best_fit_and_coalescing():
    from paper_1811_12174_amd.executor import Arena
    a = Arena(10 * 512 + 100)                 # rounded down to whole granules
    assert a.size == 10 * 512
    x = a.alloc(3 * 512); y = a.alloc(2 * 512); z = a.alloc(1); w = a.alloc(4 * 512)
    assert (x, y, z, w) == (0, 3 * 512, 5 * 512, 6 * 512) and a.alloc(1) is None
    a.free(y, 2 * 512); a.free(w, 4 * 512)
    assert a.holes == [(3 * 512, 2 * 512), (6 * 512, 4 * 512)]
    assert a.alloc(2 * 512) == 3 * 512        # best fit: the smaller hole, though the larger comes later
    assert a.alloc(5 * 512) is None           # 4 granules free in one piece, 5 asked
    a.free(z, 1)
    a.free(3 * 512, 2 * 512)                  # the three frees meet: one hole from 3 to 10
    assert a.holes == [(3 * 512, 7 * 512)]
    a.free(x, 3 * 512)
    assert a.holes == [(0, 10 * 512)] and a.high_water == 10 * 512


def test_a_budget_counts_address_space_not_only_bytes():
    """Two live tensors pin the slab so that the free bytes are split in two holes: an allocation
    of their sum must fail in simulation exactly as it would on the GPU."""
    from paper_1811_12174_amd.executor import Arena
    a = Arena(8 * 512)
    t0 = a.alloc(2 * 512); t1 = a.alloc(2 * 512); t2 = a.alloc(2 * 512); t3 = a.alloc(2 * 512)
    a.free(t0, 2 * 512); a.free(t2, 2 * 512)
    assert sum(ln for _, ln in a.holes) == 4 * 512 and a.alloc(4 * 512) is None and a.alloc(2 * 512) == t0


def test_simulated_stream_ordering():
    """A device copy is dropped only after its copy-out (the compute clock waits), a copy-in
    starts after the copy-out and after the compute point it was issued at, and a reader waits
    for the copy-in: forced with a slow link."""
    from paper_1811_12174_amd.program import TensorInfo
    be = planner.SimBackend(link=1e6)
    info = TensorInfo("t", (1, 1, 1, 1, 500000), 2)               # 1 MB: one second on this link
    be.tc = 0.25
    h = be.swap_out(info, None)
    be.release_after(h)
    assert h["out"].end == pytest.approx(1.25)
    assert be.tc == pytest.approx(1.25) and be.stall == pytest.approx(1.0)
    be.tc = 1.5
    be.prefetch_start(h, None)
    be.tc = 2.0                                                    # kernels overlapped the copy-in
    be.wait_in(h)
    assert h["in"].end == pytest.approx(2.5)
    assert be.tc == pytest.approx(2.5) and be.stall == pytest.approx(1.5)
    assert be.seconds == pytest.approx(2.5)
    # a copy-in issued while the copy-out of the same tensor is still running starts when that ends
    be = planner.SimBackend(link=1e6)
    h = be.swap_out(info, None)                                    # runs 0 .. 1
    be.tc = 0.5
    be.prefetch_start(h, None)                                     # may start at 1.0, ends 2.0
    be.wait_in(h)
    assert be.tc == pytest.approx(2.0)


def test_the_two_directions_share_the_link():
    """One direction alone moves link_one bytes/s, both together link_both each; a copy that
    overlaps the other direction for part of its life is priced piecewise."""
    from paper_1811_12174_amd.program import TensorInfo
    a = TensorInfo("a", (1, 1, 1, 1, 500000), 2)                   # 1 MB
    b = TensorInfo("b", (1, 1, 1, 1, 500000), 2)
    be = planner.SimBackend(link_one=1e6, link_both=0.5e6)
    ha = be.swap_out(a, None); be.release_after(ha)                # a goes out alone: 0 .. 1
    assert be.tc == pytest.approx(1.0)
    be.prefetch_start(ha, None)                                    # a comes back from t = 1 ...
    hb = be.swap_out(b, None)                                      # ... while b goes out: both at half rate
    be.wait_in(ha)
    assert be.tc == pytest.approx(3.0)                             # 1 MB at 0.5 MB/s
    be.release_after(hb)
    assert be.tc == pytest.approx(3.0)                             # b finished at the same moment
    # unequal overlap: c alone for 0.5 s (0.5 MB), then shares with d
    be = planner.SimBackend(link_one=1e6, link_both=0.5e6)
    hc = be.swap_out(a, None); be.release_after(hc)                # out: 0 .. 1
    be.prefetch_start(hc, None)                                    # in from 1.0
    be.tc = 1.5
    hd = be.swap_out(b, None)                                      # out from 1.5: both busy
    be.wait_in(hc)                                                 # 0.5 MB alone + 0.5 MB at half rate = 1.0 .. 2.5
    assert be.tc == pytest.approx(2.5)
    be.release_after(hd)                                           # d: 0.5 MB shared until 2.5, then 0.5 MB alone
    assert be.tc == pytest.approx(3.0)


def test_cost_model_orders_of_magnitude():
    p = unet_program(64, 1, 4, 2, 256, 256, 256)
    t = planner.simulate(p)[1].seconds
    assert 0.1 < t < 0.25      # measured on the GPU: 0.145 s


def test_arena_random_sequences_never_overlap_and_coalesce_fully():
    """Random allocation / free traffic: live ranges never overlap, stay inside the slab, a request
    fails only when no hole can take it, and freeing everything leaves one hole."""
    import random
    from paper_1811_12174_amd.executor import Arena
    rng = random.Random(1811)
    for trial in range(30):
        size = rng.randrange(20, 200) * 512
        a = Arena(size)
        live = {}
        for step in range(300):
            if live and (rng.random() < 0.45 or len(live) > 40):
                key = rng.choice(list(live))
                off, n = live.pop(key)
                a.free(off, n)
            else:
                n = rng.randrange(1, size // 3)
                top = rng.random() < 0.5
                biggest = max((ln for _, ln in a.holes), default=0)
                off = a.alloc(n, top=top)
                if off is None:
                    assert biggest < Arena.rounded(n)
                    continue
                assert biggest >= Arena.rounded(n)
                assert 0 <= off and off + Arena.rounded(n) <= a.size and off % 512 == 0
                for o2, n2 in live.values():
                    assert off + Arena.rounded(n) <= o2 or o2 + Arena.rounded(n2) <= off
                live[step] = (off, n)
            # holes are sorted, disjoint, not adjacent (fully coalesced), and complement the live ranges
            for (o1, l1), (o2, l2) in zip(a.holes, a.holes[1:]):
                assert o1 + l1 < o2
            assert sum(ln for _, ln in a.holes) + sum(Arena.rounded(n) for _, n in live.values()) == a.size
        for off, n in live.values():
            a.free(off, n)
        assert a.holes == [(0, a.size)]


def test_random_plans_keep_the_interpreter_consistent():
    """Random gap selections and prefetch points on a small program, with and without a budget: every
    call finds its tensors on the device (the simulator asserts it), the accounting returns to the
    fixed part, the peak respects the budget, and bytes in never exceed what the gaps allow."""
    import random
    rng = random.Random(12174)
    p = unet_program(16, 1, 3, 1, 32, 32, 32)
    gaps = p.gaps()
    need = planner.simulate(p)[0].peak
    ran = refused = 0
    for trial in range(60):
        chosen = [g for g in gaps if rng.random() < 0.4]
        at = {(g.tensor, g.index): rng.randrange(g.first + 1, g.last + 1) for g in chosen if rng.random() < 0.7}
        budget = None if trial % 3 == 0 else int(need * rng.uniform(0.6, 1.1))
        eager = trial % 5 == 0
        try:
            ex, be = planner.simulate(p, chosen, rng.randrange(1, 6), budget, eager, fixed_bytes=1000, at=at)
        except OutOfBudget:
            refused += 1
            assert budget is not None
            continue
        ran += 1
        assert ex.used == 1000 and ex.peak >= 1000
        if budget is not None:
            assert ex.peak <= budget and ex.arena.high_water <= budget - 1000
        assert ex.bytes_out == sum(p.tensors[t].nbytes for t in {g.tensor for g in chosen})
        assert ex.bytes_in <= sum(p.tensors[g.tensor].nbytes for g in chosen)
        assert be.seconds >= planner.simulate(p, fixed_bytes=1000)[1].seconds - 1e-12
    assert ran > 20 and refused > 0


class _FenceCheckingBackend:
    """Backend that tracks, per tensor, whether its copy-in has been fenced on the compute stream:
    a call that touches a tensor whose prefetch was started and not waited for is a read-before-copy."""

    def __init__(self):
        self.unfenced = set()     # handles with a prefetch started and no wait yet
        self.handle_of = {}       # block serial -> handle
        self.serial = 0
        self.next_handle = 0
        self.violations = []

    def slab(self, nbytes):
        pass

    def alloc(self, info, offset):
        self.serial += 1
        return (info.name, self.serial)

    def free(self, block):
        pass

    def swap_out(self, info, block):
        self.next_handle += 1
        return self.next_handle

    def release_after(self, h):
        pass

    def prefetch_start(self, h, block):
        self.unfenced.add(h)
        self.handle_of[block[1]] = h

    def wait_in(self, h):
        self.unfenced.discard(h)

    def evict(self, h):
        pass

    def release(self, h):
        pass

    def call(self, c, blocks):
        for t in c.touches():
            b = blocks.get(t)
            if b is not None and self.handle_of.get(b[1]) in self.unfenced:
                self.violations.append((c.fn, c.layer, t))


def test_every_reader_of_an_incoming_tensor_is_fenced_even_with_zero_lead():
    """Prefetch positions equal to the reader call (gaps(min_calls=1), lead 0, explicit at = last):
    the wait must come after the prefetch it fences, or the reader runs before its copy."""
    p = unet_program(8, 1, 3, 1, 16, 16, 16)
    for gaps, lead, at in [(p.gaps(1), 1, None), (p.gaps(), 0, None),
                           (p.gaps(), 2, {(g.tensor, g.index): g.last for g in p.gaps()})]:
        ins = p.instructions(gaps, lead, at)
        # static order: no ("wait", t) directly precedes the ("prefetch", t) it belongs to
        for i in range(len(ins) - 1):
            assert not (ins[i][0] == "wait" and ins[i + 1] == ("prefetch", ins[i][1])), ins[i]
        be = _FenceCheckingBackend()
        ex = Executor(be, p, budget=None, eager=True)
        ex.run(ins, {"x": ("x", -1), "labels": ("labels", -2)})
        assert not be.violations, be.violations[:3]
        assert ex.bytes_in > 0
