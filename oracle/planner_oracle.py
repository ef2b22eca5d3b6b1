"""Test infrastructure only: reference for the choice of the per-step offload amount.

SSDTrain sets the amount of activations to offload from the model's amount of computation and
activation size, the GPU throughput and the I/O bandwidth (Sec. 3.1, workflow paragraph), so that the
transfers stay hidden behind computation; tensors are then offloaded in forward order until the
amount is reached (Sec. 3.2, first condition of the pack hook).  The paper gives no formula.  The
reading fixed here (and listed among the readings of the design notes):

* stores: one FIFO queue; the tensors of layer l become available when layer l's forward ends and
  drain at `safety * store_Bps`; a byte counts towards the amount only if it has left the device by the
  end of the forward pass (only then does it lower the activation peak, which is reached there);
* loads: one FIFO queue, layers in reverse order; the load of layer l is issued when the backward of
  layer l+d starts (at the end of forward if there is no such layer) and must be complete when the
  backward of layer l starts; d is the smallest prefetch distance for which this holds, and if no
  distance works the amount shrinks (first the partial layer, then whole layers from the top);
* the last `keep_last` layers are never offloaded (Sec. 3.3.2).

The function below does this by explicit simulation of the two queues, one candidate after another,
with no closed forms, so that it can be checked by eye against the rules above.
"""
import math
from typing import List, NamedTuple, Sequence


class Plan(NamedTuple):
    budget_bytes: int
    layers: int             # leading layers entirely within the amount
    partial_bytes: int      # bytes of layer `layers` also within the amount
    prefetch_distance: int  # 0 when nothing is offloaded
    store_done_s: float     # completion time of the last store, from the start of the step


def store_prefix(layer_bytes: Sequence[int], fwd_s: Sequence[float], eligible: int, rate: float):
    """Bytes per layer that leave the device before the forward pass ends."""
    out: List[int] = []
    queue_free, done = 0.0, 0.0
    ends = []
    acc = 0.0
    for t in fwd_s:   # times accumulate left to right in double precision
        acc += t
        ends.append(acc)
    t_fwd = acc
    for l in range(eligible):
        start = max(queue_free, ends[l])
        finish = start + layer_bytes[l] / rate
        if finish <= t_fwd:
            out.append(int(layer_bytes[l]))
            queue_free = done = finish
            continue
        part = int(math.floor((t_fwd - start) * rate)) if t_fwd > start else 0
        part = max(0, min(part, int(layer_bytes[l])))
        if part:
            out.append(part)
            done = start + part / rate
        break
    return out, done


def loads_hidden(amount: Sequence[int], fwd_s: Sequence[float], bwd_s: Sequence[float], rate: float, d: int) -> bool:
    n = len(fwd_s)
    t_fwd = 0.0
    for x in fwd_s:
        t_fwd += x
    bwd_start = [0.0] * n   # backward runs layer n-1 first
    t = t_fwd
    for l in range(n - 1, -1, -1):
        bwd_start[l] = t
        t += bwd_s[l]
    queue_free = 0.0
    for l in range(len(amount) - 1, -1, -1):
        issue = bwd_start[l + d] if l + d < n else t_fwd
        finish = max(queue_free, issue) + amount[l] / rate
        if finish > bwd_start[l]:
            return False
        queue_free = finish
    return True


def last_store_end(amount: Sequence[int], fwd_s: Sequence[float], rate: float) -> float:
    queue_free, acc = 0.0, 0.0
    for l, a in enumerate(amount):
        acc += fwd_s[l]
        queue_free = max(queue_free, acc) + a / rate
    return queue_free


def plan(layer_bytes: Sequence[int], fwd_s: Sequence[float], bwd_s: Sequence[float], store_Bps: float,
         load_Bps: float, safety: float = 1.0, keep_last: int = 1) -> Plan:
    n = len(layer_bytes)
    eligible = max(0, n - keep_last)
    amount, _ = store_prefix(layer_bytes, fwd_s, eligible, safety * store_Bps)
    while amount:
        for d in range(1, n + 1):
            if loads_hidden(amount, fwd_s, bwd_s, safety * load_Bps, d):
                full = sum(1 for l, a in enumerate(amount) if a == layer_bytes[l])
                part = amount[full] if full < len(amount) else 0
                return Plan(sum(amount), full, part, d, last_store_end(amount, fwd_s, safety * store_Bps))
        # no distance hides the loads: give up the partial layer first, then the topmost layer
        amount = amount[:-1]
    return Plan(0, 0, 0, 0, 0.0)
