"""Offload-amount planner: the reference against hand-worked cases and a brute-force search, and the
library's ssdt_plan against the reference (host logic, no GPU)."""
import itertools
import math

import numpy as np
import pytest

from oracle import planner_oracle as po
from paper_2408_10013_amd import binding as sb


# ---- the reference against what the rules fix ------------------------------------------------------

def test_uniform_layers_worked_by_hand():
    # 4 layers, 1 s forward and 2 s backward each, 10 bytes each, store 5 B/s, load 100 B/s, last layer kept.
    # Stores: layer 0 ready at 1 s, done at 3 s; layer 1 ready at 2 s, starts at 3 s, would end at 5 s > 4 s:
    # (4 - 3) s * 5 B/s = 5 bytes of it count; layer 2 is not reached.
    p = po.plan([10] * 4, [1.0] * 4, [2.0] * 4, 5.0, 100.0, 1.0, 1)
    assert p == po.Plan(15, 1, 5, 1, 4.0)
    # store so fast that everything eligible leaves in time: 3 layers
    p = po.plan([10] * 4, [1.0] * 4, [2.0] * 4, 1e3, 100.0, 1.0, 1)
    assert (p.budget_bytes, p.layers, p.partial_bytes, p.prefetch_distance) == (30, 3, 0, 1)
    assert p.store_done_s == pytest.approx(3.01)
    # nothing eligible / nothing drains in time
    assert po.plan([10] * 4, [1.0] * 4, [2.0] * 4, 5.0, 100.0, 1.0, 4).budget_bytes == 0
    assert po.plan([10, 10], [1.0, 1e-9], [1.0, 1.0], 1.0, 1.0, 1.0, 1).budget_bytes == 0


def test_slow_loads_raise_the_distance_then_cut_the_amount():
    # loads at 4 B/s: a 10-byte layer needs 2.5 s but one backward layer lasts 2 s.
    # distance 1: layer 2 issued at end of forward (t=4, layer 3 kept and running), done 6.5 > start of bwd(2)=6
    # distance 2 is no better for layer 2 (issued at t=4 either way): the top layer has to go.
    p = po.plan([10] * 4, [1.0] * 4, [2.0] * 4, 1e3, 4.0, 1.0, 1)
    # layers 0,1: distance 1: layer 1 issued at bwd_start(2)=6, done 8.5 > bwd_start(1)=8 -> no;
    # distance 2: layer 1 issued at bwd_start(3)=4, done 6.5 <= 8; layer 0 issued at bwd_start(2)=6, starts 6.5, done 9 <= 10 -> yes
    assert (p.budget_bytes, p.layers, p.prefetch_distance) == (20, 2, 2)
    # safety scales both rates
    q = po.plan([10] * 4, [1.0] * 4, [2.0] * 4, 2e3, 8.0, 0.5, 1)
    assert (q.budget_bytes, q.layers, q.prefetch_distance) == (20, 2, 2)


def simulate(amount, layer_bytes, fwd_s, bwd_s, w, r, d):
    """Independent event-by-event timeline (one tick = 1/64 s) used only by the brute-force test."""
    n = len(fwd_s)
    tick = 1.0 / 64
    t_fwd = sum(fwd_s)
    ends = np.cumsum(fwd_s)
    left = list(amount)
    t = 0.0
    while any(x > 1e-9 for x in left) and t < t_fwd - 1e-12:
        for l in range(len(left)):
            if left[l] > 1e-9:
                if ends[l] <= t + 1e-12:
                    left[l] -= w * tick
                break
        t += tick
    stored_in_time = all(x <= 1e-9 for x in left)
    bwd_start = {}
    tt = t_fwd
    for l in range(n - 1, -1, -1):
        bwd_start[l] = tt
        tt += bwd_s[l]
    qf, ok = 0.0, True
    for l in range(len(amount) - 1, -1, -1):
        issue = bwd_start[l + d] if l + d < n else t_fwd
        qf = max(qf, issue) + amount[l] / r
        ok = ok and qf <= bwd_start[l] + 1e-12
    return stored_in_time, ok


def test_plan_is_feasible_and_maximal_on_small_cases():
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(2, 6))
        # dyadic times and rates keep every quantity exact in binary floating point
        fwd = [int(rng.integers(1, 9)) / 8 for _ in range(n)]
        bwd = [2 * f for f in fwd]
        lb = [int(rng.integers(1, 9)) * 64 for _ in range(n)]
        w = float(2 ** int(rng.integers(5, 10)))
        r = float(2 ** int(rng.integers(5, 10)))
        keep = int(rng.integers(0, 2))
        p = po.plan(lb, fwd, bwd, w, r, 1.0, keep)
        amount = lb[:p.layers] + ([p.partial_bytes] if p.partial_bytes else [])
        assert sum(amount) == p.budget_bytes and p.layers + (1 if p.partial_bytes else 0) <= n - keep
        if not amount:
            continue
        s_ok, l_ok = simulate(amount, lb, fwd, bwd, w, r, p.prefetch_distance)
        assert s_ok and l_ok, (lb, fwd, w, r, keep, p)
        if p.prefetch_distance > 1:   # the distance is the smallest that works
            assert not simulate(amount, lb, fwd, bwd, w, r, p.prefetch_distance - 1)[1]
        # maximal among store-feasible prefixes whose loads can be hidden: one more 64-byte unit breaks something
        grown = list(amount)
        if p.partial_bytes or p.layers < n - keep:
            if p.partial_bytes and p.partial_bytes + 64 <= lb[p.layers]:
                grown[-1] += 64
            elif p.partial_bytes:
                continue
            else:
                grown.append(64)
            feas = [simulate(grown, lb, fwd, bwd, w, r, d) for d in range(1, n + 1)]
            stores_fit = feas[0][0]
            loads_fit = any(f[1] for f in feas)
            cut_back = amount != po.store_prefix(lb, fwd, n - keep, w)[0]
            assert (not stores_fit) or (not loads_fit) or cut_back, (lb, fwd, w, r, keep, p)


def test_unequal_layers_worked_by_hand():
    """Two cases with layers of different lengths and sizes, worked on paper from the rules (stores: one queue in
    forward order, a layer's bytes available when its forward ends, counted only if gone by the end of forward;
    loads: one queue in reverse order, layer l issued when backward of layer l+d starts, due when backward of layer l
    starts).  Both the reference and the library must give the paper result."""
    # (A) forward 1, 2, 1 s (ends at 1, 3, 4), backward 2, 4, 2 s; 8, 4, 6 bytes; store 4 B/s, load 2 B/s; last kept.
    #     stores: layer 0 from 1 s to 3 s; layer 1 from 3 s to 4 s = end of forward: both whole, 12 bytes, done at 4 s.
    #     backward starts: layer 2 at 4 s, layer 1 at 6 s, layer 0 at 10 s.  distance 1: layer 1 issued at 4 s, 2 s
    #     long, done at 6 s (due 6 s); layer 0 issued at 6 s, 4 s long, done at 10 s (due 10 s): hidden.
    a = ([8, 4, 6], [1.0, 2.0, 1.0], [2.0, 4.0, 2.0], 4.0, 2.0, 1.0, 1)
    want_a = (12, 2, 0, 1, 4.0)
    # (B) forward 2, 1, 1, 2 s (ends at 2, 3, 4, 6), backward 4, 2, 2, 4 s; 6, 8, 4, 10 bytes; store 2 B/s; last kept.
    #     stores: layer 0 from 2 s to 5 s; layer 1 starts at 5 s and would need 4 s: (6 - 5) s * 2 B/s = 2 bytes count;
    #     amount 6 + 2, last store done at 6 s.  backward starts: layer 3 at 6 s, 2 at 10 s, 1 at 12 s, 0 at 14 s.
    #     load 1 B/s: distance 1: layer 1 (2 B) issued at 10 s, done 12 s; layer 0 (6 B) issued at 12 s, done 18 s > 14 s.
    #     distance 2: layer 1 issued at 6 s, done 8 s; layer 0 issued at 10 s, done 16 s > 14 s.  distance 3: layer 1
    #     issued at the end of forward (6 s), done 8 s; layer 0 issued at 6 s, waits for the queue, 8 s .. 14 s: hidden.
    b1 = ([6, 8, 4, 10], [2.0, 1.0, 1.0, 2.0], [4.0, 2.0, 2.0, 4.0], 2.0, 1.0, 1.0, 1)
    want_b1 = (8, 1, 2, 3, 6.0)
    #     load 0.75 B/s: layer 1 takes 2.67 s, layer 0 8 s: even issued together at 6 s they end at 16.67 s > 14 s, so
    #     the partial layer is given up; layer 0 alone: issued at 12 s (distance 1) or 10 s (distance 2) it is late,
    #     issued at 6 s (distance 3) it is done at 14 s: hidden.  Its store is done at 5 s.
    b2 = ([6, 8, 4, 10], [2.0, 1.0, 1.0, 2.0], [4.0, 2.0, 2.0, 4.0], 2.0, 0.75, 1.0, 1)
    want_b2 = (6, 1, 0, 3, 5.0)
    for args, want in ((a, want_a), (b1, want_b1), (b2, want_b2)):
        p = po.plan(*args)
        assert (p.budget_bytes, p.layers, p.partial_bytes, p.prefetch_distance, p.store_done_s) == want, (args, p)
        g = sb.ssdt_plan(*args)
        assert (g["budget_bytes"], g["layers"], g["partial_bytes"], g["prefetch_distance"], g["store_done_s"]) == want, (args, g)


class Timeline:
    """The rules of the planner played out tick by tick (1/64 s), with no arithmetic shared with the reference or the
    library: a store queue that moves `w` bytes per second of the oldest unfinished layer once that layer's forward
    has ended, a load queue that moves `r` bytes per second of the oldest issued request.  All quantities in the
    tests that use it are dyadic, so every comparison is exact."""
    TICK = 1.0 / 64

    def __init__(self, fwd_s, bwd_s):
        self.n = len(fwd_s)
        self.fwd_end = [sum(fwd_s[:l + 1]) for l in range(self.n)]
        self.t_fwd = self.fwd_end[-1]
        self.bwd_start = {}
        t = self.t_fwd
        for l in range(self.n - 1, -1, -1):
            self.bwd_start[l] = t
            t += bwd_s[l]
        self.t_end = t

    def drained_by_end_of_forward(self, layer_bytes, eligible, w):
        """Bytes of each eligible layer that have left the device when the forward pass ends (whole bytes)."""
        left = [float(b) for b in layer_bytes[:eligible]]
        t = 0.0
        while t < self.t_fwd:
            for l in range(eligible):
                if left[l] > 0:
                    if self.fwd_end[l] <= t:          # available during this whole tick
                        left[l] = max(0.0, left[l] - w * self.TICK)
                    break                             # first in, first out: nobody overtakes
            t += self.TICK
        out = []
        for l in range(eligible):
            gone = int(layer_bytes[l] - left[l])
            if gone <= 0:
                break
            out.append(gone)
            if left[l] > 0:
                break
        return out

    def loads_hidden(self, amount, r, d):
        left = {l: float(a) for l, a in enumerate(amount)}
        order = sorted(left, reverse=True)
        issue = {l: (self.bwd_start[l + d] if l + d < self.n else self.t_fwd) for l in order}
        t = self.t_fwd
        while t < self.t_end:
            for l in order:
                if left[l] > 0 and t >= self.bwd_start[l]:
                    return False                      # its backward starts and it is not back
            for l in order:
                if left[l] > 0:
                    if issue[l] <= t:
                        left[l] = max(0.0, left[l] - r * self.TICK)
                    break
            t += self.TICK
        return all(v <= 0 for v in left.values())


def test_library_plan_against_the_tick_by_tick_timeline():
    """ssdt_plan's own output on 200 seeded dyadic cases: what it offloads is exactly what the store queue drains by
    the end of forward, cut back from the top only as far as the loads demand, with the smallest prefetch distance
    that hides them."""
    rng = np.random.default_rng(17)
    seen_cut = seen_far = 0
    for _ in range(200):
        n = int(rng.integers(2, 6))
        fwd = [int(rng.integers(1, 9)) / 8 for _ in range(n)]
        bwd = [2 * f for f in fwd]
        lb = [int(rng.integers(1, 9)) * 64 for _ in range(n)]
        w = float(2 ** int(rng.integers(5, 10)))
        r = float(2 ** int(rng.integers(4, 10)))
        keep = int(rng.integers(0, 2))
        g = sb.ssdt_plan(lb, fwd, bwd, w, r, 1.0, keep)
        got = lb[:g["layers"]] + ([g["partial_bytes"]] if g["partial_bytes"] else [])
        assert sum(got) == g["budget_bytes"]
        tl = Timeline(fwd, bwd)
        prefix = tl.drained_by_end_of_forward(lb, n - keep, w)
        want, want_d = [], 0
        for k in range(len(prefix), 0, -1):          # give up the partial layer first, then layers from the top
            ds = [d for d in range(1, n + 1) if tl.loads_hidden(prefix[:k], r, d)]
            if ds:
                want, want_d = prefix[:k], ds[0]
                break
        assert got == want and g["prefetch_distance"] == want_d, (lb, fwd, w, r, keep, g, prefix, want, want_d)
        seen_cut += len(want) < len(prefix)
        seen_far += want_d > 1
    assert seen_cut >= 5 and seen_far >= 5           # the cases do exercise both rules


# ---- the library against the reference ---------------------------------------------------------------

def cases():
    rng = np.random.default_rng(11)
    out = [([10] * 4, [1.0] * 4, [2.0] * 4, 5.0, 100.0, 1.0, 1), ([10] * 4, [1.0] * 4, [2.0] * 4, 1e3, 4.0, 1.0, 1),
           ([10] * 4, [1.0] * 4, [2.0] * 4, 5.0, 100.0, 1.0, 4)]
    for _ in range(300):
        n = int(rng.integers(1, 13))
        fwd = list(rng.uniform(1e-3, 5e-2, n))
        bwd = list(2 * np.array(fwd) * rng.uniform(0.8, 1.2, n))
        lb = [int(x) for x in rng.integers(1 << 20, 1 << 33, n)]
        out.append((lb, fwd, bwd, float(rng.uniform(5e9, 6e10)), float(rng.uniform(5e9, 6e10)),
                    float(rng.uniform(0.5, 1.0)), int(rng.integers(0, 3))))
    # the headline shape: 8 layers of 8.6 GB, 55 ms forward each, 57 GB/s each way
    out.append(([8_602_517_504] * 8, [0.055] * 8, [0.11] * 8, 57e9, 57e9, 0.85, 1))
    return out


def test_library_plan_equals_reference():
    for lb, fwd, bwd, w, r, s, keep in cases():
        ref = po.plan(lb, fwd, bwd, w, r, s, keep)
        got = sb.ssdt_plan(lb, fwd, bwd, w, r, s, keep)
        assert (got["budget_bytes"], got["layers"], got["partial_bytes"], got["prefetch_distance"]) == \
               (ref.budget_bytes, ref.layers, ref.partial_bytes, ref.prefetch_distance), (lb, fwd, w, r, s, keep)
        assert got["store_done_s"] == pytest.approx(ref.store_done_s, rel=1e-12, abs=1e-15)


def test_library_plan_rejects_bad_input():
    for bad in (dict(store_Bps=0.0), dict(load_Bps=-1.0), dict(safety=0.0), dict(safety=1.5), dict(keep_last=-1)):
        kw = dict(layer_bytes=[10, 10], fwd_s=[1.0, 1.0], bwd_s=[2.0, 2.0], store_Bps=5.0, load_Bps=5.0, safety=1.0, keep_last=1)
        kw.update(bad)
        with pytest.raises(sb.SsdtError) as e:
            sb.ssdt_plan(**kw)
        assert e.value.status == sb.E_INVAL
    with pytest.raises(sb.SsdtError):
        sb.ssdt_plan([], [], [], 1.0, 1.0, 1.0, 0)
    with pytest.raises(sb.SsdtError):
        sb.ssdt_plan([10], [-1.0], [1.0], 1.0, 1.0, 1.0, 0)
