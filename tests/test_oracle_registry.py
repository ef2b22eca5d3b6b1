"""Pins for the bookkeeping checker (no GPU): closed forms, hand-worked traces, and the
paper's Table 3 as a sanity ratio."""
import json
import os

import pytest

from oracle import registry_oracle as ro

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run_layers(reg, traces, shared=()):
    """traces: list over layers of saved_trace() lists.  Storage key = (layer, name) unless
    the storage name is in `shared` (then it is one storage for the whole step)."""
    stamps = []
    for l, tr in enumerate(traces):
        reg.scope_begin(l)
        for name, storage, sbytes, numel in tr:
            key = storage if storage in shared else (l, storage)
            stamps.append(reg.save(key, sbytes, numel))
        reg.scope_end(l)
    return stamps


def gpt_trace(T, H, F, B, A, S, e):
    return ro.saved_trace("gpt_preln", "layernorm", "gelu", T, H, F, B, A, S, e)


def test_gpt_layer_counts_and_bytes_closed_form():
    B, S, H, A, F, e = 2, 128, 256, 4, 1024, 4
    T = B * S
    reg = ro.RegistryOracle(num_layers=1, min_offload_elems=0, keep_last=0)
    run_layers(reg, [gpt_trace(T, H, F, B, A, S, e)])
    c = reg.c
    assert (c.save_calls, c.unique, c.dedup_hits) == (16, 13, 3)
    assert c.offloaded == 13 and c.kept == 0 and c.bypass_small == 0
    payload = (8 * T * H + 2 * T * F) * e + 4 * T * 4 + B * A * S * 4
    assert c.bytes_offloaded == payload == 4202496


def test_bf16_payload_is_32TH_plus_stats():
    B, S, H, A, F, e = 4, 1024, 2048, 16, 8192, 2
    T = B * S
    reg = ro.RegistryOracle(num_layers=2, min_offload_elems=0, keep_last=0)
    run_layers(reg, [gpt_trace(T, H, F, B, A, S, e)] * 2)
    per_layer = 32 * T * H + 4 * T * 4 + B * A * S * 4
    assert reg.c.bytes_offloaded == 2 * per_layer
    assert abs(per_layer / 269e6 - 1) < 0.01


def test_other_archs_counts():
    T, H, F, B, A, S = 64, 32, 64, 2, 4, 32
    tr = ro.saved_trace("bert_postln", "layernorm", "gelu", T, H, F, B, A, S, 2)
    assert len(tr) == 16 and len({s for _, s, _, _ in tr}) == 13
    tr = ro.saved_trace("t5_enc", "rmsnorm", "relu", T, H, F, B, A, S, 2)
    assert len(tr) == 14 and len({s for _, s, _, _ in tr}) == 10
    tr = ro.saved_trace("t5_dec", "rmsnorm", "relu", T, H, F, B, A, S, 2, T_enc=128)
    names = [s for _, s, _, _ in tr]
    assert names.count("enc") == 1 and names.count("kvx") == 2


def test_default_threshold_bypasses_small_tensors():
    # 2**20-element threshold of the pack hook: statistics and lse stay, big tensors go
    B, S, H, A, F, e = 4, 1024, 2048, 16, 8192, 2
    T = B * S
    reg = ro.RegistryOracle(num_layers=2, keep_last=0)
    stamps = run_layers(reg, [gpt_trace(T, H, F, B, A, S, e)] * 2)
    c = reg.c
    assert c.bypass_small == 2 * 5 and c.offloaded == 2 * 8
    assert c.bytes_offloaded == 2 * 32 * T * H
    assert stamps[1] == 0 and stamps[0] == 1       # mean1 bypassed -> id 0; x -> first stamp


def test_hand_worked_offsets_budget_keep_last_and_weights():
    reg = ro.RegistryOracle(num_layers=3, min_offload_elems=10, budget_bytes=2000, keep_last=1)
    reg.register_weight("W")
    reg.scope_begin(0)
    assert reg.save("W", 4000, 1000) == 0            # weight: bypassed, not recorded
    assert reg.save("a", 300, 150) == 1              # pack offset 0
    assert reg.save("s", 16, 4) == 0                 # small: tracked, id 0
    assert reg.save("b", 1000, 500) == 3             # offset up(300,256)=512
    assert reg.save("a", 300, 75) == 1               # view of a: dedup hit
    reg.scope_end(0)
    reg.scope_begin(1)
    assert reg.save("c", 600, 300) == 4              # 300+1000+600 = 1900 <= 2000 -> offloaded
    assert reg.save("d", 200, 100) == 5              # 2100 > 2000 -> kept
    assert reg.save("e", 100, 50) == 6               # 2000 <= 2000 -> offloaded, offset up(600,256)=768
    reg.scope_end(1)
    reg.scope_begin(2)
    assert reg.save("f", 50, 25) == 7                # last layer: kept
    reg.scope_end(2)
    r = {x.stamp: x for x in reg.records}
    assert (r[1].cls, r[1].pack_offset, r[1].pool_offset) == (ro.OFFLOADED, 0, 0)
    assert (r[3].cls, r[3].pack_offset, r[3].pool_offset) == (ro.OFFLOADED, 512, 512)
    assert r[2].cls == ro.SMALL
    # layer 0's pack is 1512 bytes -> rounded to 4096; layer 1's pack starts there
    assert (r[4].cls, r[4].pack_offset, r[4].pool_offset) == (ro.OFFLOADED, 0, 4096)
    assert r[5].cls == ro.KEPT and r[5].pool_offset == -1
    assert (r[6].cls, r[6].pack_offset, r[6].pool_offset) == (ro.OFFLOADED, 768, 4096 + 768)
    assert r[7].cls == ro.KEPT
    c = reg.c
    assert (c.save_calls, c.unique, c.dedup_hits, c.bypass_weight, c.bypass_small) == (9, 7, 1, 1, 1)
    assert (c.offloaded, c.kept, c.bytes_offloaded, c.bytes_kept, c.bytes_small) == (4, 2, 2000, 250, 16)
    assert c.pool_bytes_used == 8192
    assert reg.prefetch_order(0) == [3, 1] and reg.prefetch_order(1) == [6, 4]


def test_pool_overflow_falls_back_to_kept():
    reg = ro.RegistryOracle(num_layers=2, min_offload_elems=0, keep_last=0, pool_bytes=8192)
    reg.scope_begin(0)
    reg.save("a", 4000, 1)
    reg.save("b", 200, 1)                            # 4096+200 -> pack 8192 fits
    reg.scope_end(0)
    reg.scope_begin(1)
    reg.save("c", 10, 1)                             # pack would start at 8192: no room
    reg.scope_end(1)
    assert [r.cls for r in reg.records] == [ro.OFFLOADED, ro.OFFLOADED, ro.KEPT]


def test_shared_encoder_output_stored_once_and_released_last():
    B, S, Se, H, A, F = 8, 128, 512, 2048, 32, 5120
    T, Te = B * S, B * Se
    tr = ro.saved_trace("t5_dec", "rmsnorm", "relu", T, H, F, B, A, S, 2, T_enc=Te)
    reg = ro.RegistryOracle(num_layers=2, min_offload_elems=0, keep_last=0)
    run_layers(reg, [tr, tr], shared=("enc",))
    enc = [r for r in reg.records if r.bytes == Te * H * 2 and r.scopes == [0, 1]]
    assert len(enc) == 1 and enc[0].layer == 0 and enc[0].cls == ro.OFFLOADED
    assert abs(enc[0].bytes / 16.8e6 - 1) < 0.01
    # per layer: k, v (views of qkv), o again, vx (view of kvx), ox again, g again = 6; plus enc once
    assert reg.c.dedup_hits == 2 * 6 + 1
    assert reg.c.save_calls == 2 * 24 and reg.c.unique == 2 * 18 - 1
    freed1 = reg.release(1)
    assert enc[0].stamp not in freed1
    freed0 = reg.release(0)
    assert enc[0].stamp in freed0


def test_stamps_are_never_reused():
    reg = ro.RegistryOracle(num_layers=1, min_offload_elems=0, keep_last=0)
    reg.scope_begin(0)
    s1 = reg.save(("addr", 0x1000, "gen0"), 64, 16)
    s2 = reg.save(("addr", 0x1000, "gen1"), 64, 16)  # same address, a new storage
    assert s1 != s2 and s2 == s1 + 1


def test_table3_sanity_ratio():
    """The paper's measured per-GPU amounts are with tensor parallelism 2, which shards some
    saved tensors and replicates others; the unsharded payload of all L layers must therefore
    lie between 1x and 2x the paper's figure (how much of the last layer the paper kept is not
    stated, so no layer is kept here)."""
    with open(os.path.join(GOLDEN, "paper_table3.json")) as f:
        cases = json.load(f)["cases"]
    for cse in cases:
        H, L = cse["H"], cse["L"]
        B, S, A = 16, 1024, H // 128
        T = B * S
        tr = ro.saved_trace("bert_postln", "layernorm", "gelu", T, H, 4 * H, B, A, S, 2)
        reg = ro.RegistryOracle(num_layers=L, keep_last=0)
        run_layers(reg, [tr] * L)
        ratio = reg.c.bytes_offloaded / (cse["offloaded_GB"] * 1e9)
        assert 1.0 <= ratio <= 2.0, (H, ratio)


def test_saves_during_backward_are_kept_hand_worked():
    """Layerwise recomputation (Sec. 3.2, second condition of the keep test; Sec. 4.3): forward registers only
    each layer's input; the recomputed activations registered inside backward never go to the pool."""
    reg = ro.RegistryOracle(num_layers=2, min_offload_elems=0, budget_bytes=None, keep_last=0, pool_bytes=1 << 20)
    for l in range(2):                                   # forward: one 1000-byte input per layer
        reg.scope_begin(l)
        assert reg.save(("x", l), 1000, 500) == l + 1
        reg.scope_end(l)
    assert (reg.c.offloaded, reg.c.bytes_offloaded, reg.c.kept) == (2, 2000, 0)
    assert [r.pool_offset for r in reg.records] == [0, 4096]
    reg.backward_begin()                                 # backward of layer 1: recompute, then backward
    reg.scope_begin(1)
    assert reg.save(("x", 1), 1000, 500) == 2            # the input again: the same record
    assert reg.save(("h", 1), 3000, 1500) == 3           # recomputed activation: new stamp, kept
    assert reg.save(("h", 1), 3000, 750) == 3
    reg.scope_end(1)
    reg.backward_end()
    c = reg.c
    assert (c.save_calls, c.unique, c.dedup_hits, c.offloaded, c.kept, c.bytes_kept, c.bytes_offloaded) == \
           (5, 3, 2, 2, 1, 3000, 2000)
    h = reg.records[2]
    assert (h.cls, h.layer, h.pack_offset, h.pool_offset, h.scopes) == (ro.KEPT, 1, -1, -1, [1])
    assert c.pool_bytes_used == 8192                     # the pool layout of the forward pass is untouched
    # outside backward the same save is offloaded again
    reg.scope_begin(1)
    assert reg.save(("g", 1), 100, 50) == 4 and reg.records[3].cls == ro.OFFLOADED


def test_two_micro_batches_in_flight_hand_worked():
    """Individual records per micro-batch (Sec. 3.1): forward of micro-batch 0, forward of micro-batch 1, then the
    backwards in reverse.  Same layer ids, separate records; stamps, the offload amount and the pool run across both;
    the last layer is kept only for the micro-batch whose backward follows at once."""
    reg = ro.RegistryOracle(num_layers=2, min_offload_elems=0, budget_bytes=2500, keep_last=1, pool_bytes=1 << 20)
    reg.micro_batch(0, keep_last=0)               # its backward is far away: nothing kept for being last
    for l in range(2):
        reg.scope_begin(l)
        assert reg.save(("a", 0, l), 1000, 500) == l + 1
        reg.scope_end(l)
    reg.micro_batch(1)                            # default keep_last = 1
    for l in range(2):
        reg.scope_begin(l)
        assert reg.save(("a", 1, l), 1000, 500) == l + 3
        reg.scope_end(l)
    rec = reg.records
    assert [(r.micro_batch, r.layer, r.cls) for r in rec] == \
        [(0, 0, ro.OFFLOADED), (0, 1, ro.OFFLOADED), (1, 0, ro.KEPT), (1, 1, ro.KEPT)]
    # micro-batch 1, layer 0: 2000 + 1000 > 2500 -> over the amount; layer 1: last layer of its micro-batch
    assert [r.pool_offset for r in rec] == [0, 4096, -1, -1]
    assert reg.c.pool_bytes_used == 8192 and reg.c.bytes_offloaded == 2000 and reg.c.bytes_kept == 2000
    # releases address the current micro-batch only
    assert reg.release(1) == [4] and reg.release(0) == [3]
    reg.micro_batch(0)
    assert reg.prefetch_order(1) == [2] and reg.prefetch_order(0) == [1]
    assert reg.release(1) == [2] and reg.release(0) == [1]
    assert all(not r.scopes for r in rec)
