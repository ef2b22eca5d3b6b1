"""Reference (test-only) simulation of the tensor cache's bookkeeping.

THIS IS TEST INFRASTRUCTURE; the product never imports it and it shares no code with
the C library.

It replays a sequence of events -- scope begin/end and "tensor saved for backward" --
through the rules of the paper's pack hook (Algorithm 1; Sec. 3.2 for scopes, the
offload amount and the kept last module; Sec. 3.3.1 for identity and weight exclusion)
and produces, for every unique storage, the record the library must also produce:
stamp, class, owning scope, byte size and offsets inside the host pool.

Rules, in the order the pack hook applies them to one save call:
  1. the storage is a registered weight                      -> bypass (nothing recorded)
  2. the view has fewer than `min_offload_elems` elements    -> bypass, but the storage is
     still tracked (class SMALL) so that its device memory is released with its scopes
  3. identity: a storage seen for the first time gets the next value of a counter that
     starts at 1 and is never reused; any later save of any view of that storage is a
     dedup hit and inherits the class chosen at the first save
  4. the current scope (top of the forward scope stack) is added to the record's scopes
  5. the storage is KEPT when its layer is among the last `keep_last` layers of the
     step, or when `offloaded_so_far + bytes > budget_bytes`, or when its pack would
     overflow the host pool, or when the save happens inside backward propagation (a
     checkpointed module recomputing its activations: second condition of the pack
     hook's keep test, Sec. 3.2); otherwise it is OFFLOADED and `offloaded_so_far += bytes`

Micro-batches (Sec. 3.1: individual records are kept for each micro-batch and the cache switches
records when the micro-batch changes): `micro_batch(mb)` makes every later scope id refer to that
micro-batch, so the same layer ids can be open for several micro-batches at once; the keep-last
rule can be overridden per micro-batch (the paper keeps the last module only where its backward
follows its forward immediately); stamps, the offload amount and the pool cursor run across
micro-batches.

Host-pool layout: the OFFLOADED storages of one layer (the scope at the bottom of the
scope stack) form a pack, in first-save order, each starting at the next multiple of
256 bytes (of 4096 bytes when the pool is backed by a spill file, whose direct I/O works in
whole blocks: `tensor_align`); a pack's size is rounded up to 4096 bytes; packs follow each
other in the order their layers first appear.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

ALIGN_TENSOR = 256
ALIGN_PACK = 4096

WEIGHT, SMALL, KEPT, OFFLOADED = "weight", "small", "kept", "offloaded"


def _up(v: int, a: int) -> int:
    return (v + a - 1) // a * a


@dataclass
class Record:
    stamp: int
    cls: str
    layer: int                 # owning layer (bottom of scope stack at first save)
    bytes: int
    pack_offset: int = -1      # offset inside the layer's pack (OFFLOADED only)
    pool_offset: int = -1      # offset inside the host pool   (OFFLOADED only)
    scopes: List[int] = field(default_factory=list)
    micro_batch: int = 0


@dataclass
class Counters:
    save_calls: int = 0
    unique: int = 0
    dedup_hits: int = 0
    bypass_weight: int = 0
    bypass_small: int = 0
    kept: int = 0
    offloaded: int = 0
    bytes_small: int = 0
    bytes_kept: int = 0
    bytes_offloaded: int = 0
    pool_bytes_used: int = 0


class RegistryOracle:
    def __init__(self, num_layers: int, min_offload_elems: int = 1 << 20,
                 budget_bytes: Optional[int] = None, keep_last: int = 1,
                 pool_bytes: Optional[int] = None, tensor_align: int = ALIGN_TENSOR):
        self.tensor_align = tensor_align
        self.num_layers = num_layers
        self.min_elems = min_offload_elems
        self.budget = budget_bytes
        self.keep_last = keep_last
        self.pool_bytes = pool_bytes
        self.weights = set()
        self.stack: List[int] = []
        self.next_stamp = 1
        self.by_storage: Dict[object, Record] = {}
        self.records: List[Record] = []
        self.c = Counters()
        self.pack_cursor: Dict[int, int] = {}     # layer -> bytes used inside its pack
        self.pack_base: Dict[int, int] = {}       # layer -> pool offset of its pack
        self.pool_cursor = 0
        self.in_backward = 0                      # depth of open backward scopes
        self.cur_mb = 0
        self.mb_keep_last: Dict[int, int] = {}

    # -- events ------------------------------------------------------------------------
    def register_weight(self, storage) -> None:
        self.weights.add(storage)

    def micro_batch(self, mb: int, keep_last: Optional[int] = None) -> None:
        assert not self.stack and self.in_backward == 0
        self.cur_mb = mb
        if keep_last is not None:
            self.mb_keep_last[mb] = keep_last

    def scope_begin(self, scope: int) -> None:
        scope = (self.cur_mb, scope)
        if not self.stack and scope not in self.pack_base:
            # a new layer: its pack starts where the previous layer's (rounded) pack ended
            self.pool_cursor = _up(self.pool_cursor, ALIGN_PACK)
            self.pack_base[scope] = self.pool_cursor
            self.pack_cursor[scope] = 0
        self.stack.append(scope)

    def backward_begin(self) -> None:
        self.in_backward += 1

    def backward_end(self) -> None:
        assert self.in_backward > 0
        self.in_backward -= 1

    def scope_end(self, scope: int) -> None:
        scope = (self.cur_mb, scope)
        assert self.stack and self.stack[-1] == scope
        self.stack.pop()
        if not self.stack:
            self.pool_cursor = _up(self.pack_base[scope] + self.pack_cursor[scope], ALIGN_PACK)

    def save(self, storage, storage_bytes: int, numel: int) -> int:
        """Returns the stamp (0 when bypassed)."""
        c = self.c
        c.save_calls += 1
        if storage in self.weights:
            c.bypass_weight += 1
            return 0
        scope, layer = self.stack[-1], self.stack[0]
        rec = self.by_storage.get(storage)
        if rec is not None:
            c.dedup_hits += 1
            assert rec.micro_batch == scope[0], "a storage is saved from one micro-batch only"
            if scope[1] not in rec.scopes:
                rec.scopes.append(scope[1])
            return 0 if rec.cls == SMALL else rec.stamp
        rec = Record(stamp=self.next_stamp, cls=KEPT, layer=layer[1], micro_batch=layer[0], bytes=storage_bytes,
                     scopes=[scope[1]])
        self.next_stamp += 1
        self.by_storage[storage] = rec
        self.records.append(rec)
        c.unique += 1
        if numel < self.min_elems:
            rec.cls = SMALL
            c.bypass_small += 1
            c.bytes_small += storage_bytes
            return 0
        in_last = layer[1] >= self.num_layers - self.mb_keep_last.get(layer[0], self.keep_last)
        over = self.budget is not None and c.bytes_offloaded + storage_bytes > self.budget
        off = _up(self.pack_cursor[layer], self.tensor_align)
        nomem = (self.pool_bytes is not None and
                 _up(self.pack_base[layer] + off + storage_bytes, ALIGN_PACK) > self.pool_bytes)
        if in_last or over or nomem or self.in_backward > 0:
            c.kept += 1
            c.bytes_kept += storage_bytes
            return rec.stamp
        rec.cls = OFFLOADED
        rec.pack_offset = off
        rec.pool_offset = self.pack_base[layer] + off
        self.pack_cursor[layer] = off + storage_bytes
        c.offloaded += 1
        c.bytes_offloaded += storage_bytes
        c.pool_bytes_used = _up(self.pack_base[layer] + self.pack_cursor[layer], ALIGN_PACK)
        return rec.stamp

    # -- backward side -----------------------------------------------------------------
    def prefetch_order(self, layer: int) -> List[int]:
        """Stamps of a layer's OFFLOADED records in the order they are loaded: the reverse
        of the order they were saved in, because backward consumes them last-in-first-out
        (Sec. 3.1 step 5; Sec. 3.3.2)."""
        return [r.stamp for r in reversed(self.records)
                if r.layer == layer and r.micro_batch == self.cur_mb and r.cls == OFFLOADED]

    def release(self, scope: int) -> List[int]:
        """Backward of `scope` finished: drop it from every scope list; returns the stamps
        whose list became empty (their memory is freed) -- Sec. 3.2, backward hook pair."""
        freed = []
        for r in self.records:
            if r.micro_batch == self.cur_mb and scope in r.scopes:
                r.scopes.remove(scope)
                if not r.scopes:
                    freed.append(r.stamp)
        return freed


# --------------------------------------------------------------------------------------
# the save sequence of one layer
# --------------------------------------------------------------------------------------

def saved_trace(arch: str, norm: str, act: str, T: int, H: int, F: int, B: int, A: int, S: int,
                esize: int, T_enc: int = 0) -> List[Tuple[str, str, int, int]]:
    """The save calls one layer issues in forward order, as (tensor name, storage name,
    storage bytes, view elements).  This is what autograd would keep for the operators of
    the layer (Sec. 3.2: every tensor registered on the graph goes through the pack hook):
    each norm keeps its input and per-row statistics, each linear its input, attention its
    q, k, v (three views of the one projection output), its output and the per-row
    log-sum-exp (fused attention keeps no S x S tensor, Sec. 4.3), the activation its
    input (GELU) or output (ReLU).  Statistics and lse are fp32."""
    ln = norm == "layernorm"
    tr: List[Tuple[str, str, int, int]] = []

    def t(name, storage, sbytes, numel):
        tr.append((name, storage, sbytes, numel))

    def stats(tag):
        if ln:
            t("mean" + tag, "mean" + tag, T * 4, T)
        t("rstd" + tag, "rstd" + tag, T * 4, T)

    def self_attn():
        for n in ("q", "k", "v"):
            t(n, "qkv", T * 3 * H * esize, T * H)
        t("o", "o", T * H * esize, T * H)
        t("lse", "lse", B * A * S * 4, B * A * S)
        t("o", "o", T * H * esize, T * H)                 # out-projection input

    def act_and_fc2():
        if act == "gelu":
            t("h1", "h1", T * F * esize, T * F)           # activation input
        else:
            t("g", "g", T * F * esize, T * F)             # ReLU keeps its output
        t("g", "g", T * F * esize, T * F)                 # FC2 input

    if arch == "bert_postln":
        t("x", "x", T * H * esize, T * H)                 # QKV-projection input
        self_attn()
        t("r1", "r1", T * H * esize, T * H); stats("1")   # norm-1 input = x + attn
        t("x1", "x1", T * H * esize, T * H)               # FC1 input
        act_and_fc2()
        t("r2", "r2", T * H * esize, T * H); stats("2")
        return tr

    t("x", "x", T * H * esize, T * H); stats("1")          # norm-1 input
    t("a", "a", T * H * esize, T * H)                      # QKV-projection input
    self_attn()
    t("x1", "x1", T * H * esize, T * H)
    if arch == "t5_dec":
        stats("x")                                         # cross-attention norm over x1
        t("ax", "ax", T * H * esize, T * H)                # Q-projection input
        t("enc", "enc", T_enc * H * esize, T_enc * H)      # K|V-projection input (encoder output)
        t("qx", "qx", T * H * esize, T * H)
        t("kx", "kvx", T_enc * 2 * H * esize, T_enc * H)
        t("vx", "kvx", T_enc * 2 * H * esize, T_enc * H)
        t("ox", "ox", T * H * esize, T * H)
        t("lsex", "lsex", B * A * S * 4, B * A * S)
        t("ox", "ox", T * H * esize, T * H)
        t("x2", "x2", T * H * esize, T * H)                # norm-2 input
    stats("2")
    t("m", "m", T * H * esize, T * H)
    act_and_fc2()
    return tr
