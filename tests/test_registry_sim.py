"""Host logic of the tensor cache, exercised without a GPU through the simulated copy
backend (copies complete when the test says so), and compared with the bookkeeping checker."""
import ctypes
import re
import os

import numpy as np
import pytest

from oracle import registry_oracle as ro
from paper_2408_10013_amd import binding as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


class Arena:
    def __init__(self, nbytes):
        self.buf = np.zeros(nbytes + 256, dtype=np.uint8)
        addr = self.buf.ctypes.data
        self.base = (addr + 255) // 256 * 256
        self.nbytes = nbytes

    def view(self, ptr, n):
        off = ptr - self.buf.ctypes.data
        return self.buf[off:off + n]


def make(arena_bytes=1 << 20, pool_bytes=1 << 20, **kw):
    ar = Arena(arena_bytes)
    kw.setdefault("min_offload_elems", 0)
    kw.setdefault("keep_last", 0)
    ctx = sb.ssdt_ctx_create(backend=sb.BACKEND_SIM, arena_base=ar.base, arena_bytes=arena_bytes,
                             pool_bytes=pool_bytes, **kw)
    return ctx, ar


def records(ctx):
    return [sb.ssdt_get_record(ctx, i) for i in range(sb.ssdt_num_records(ctx))]


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ssdt.h")).read()
    declared = set(re.findall(r"\b(ssdt_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(sb.exported_symbols())
    l = sb.lib()
    for name in declared:
        assert hasattr(l, name), name
    assert "gfx950" in sb.ssdt_version()


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(sb.ssdt_config) == 64
    assert ctypes.sizeof(sb.ssdt_stats) == 22 * 8
    assert ctypes.sizeof(sb.ssdt_record) == 64
    assert ctypes.sizeof(sb.ssdt_layer_desc) == 64
    assert ctypes.sizeof(sb.ssdt_layer_weights) == 20 * 8
    assert ctypes.sizeof(sb.ssdt_layer_saved) == 8 + 24 * sb.SV_COUNT
    assert sb.SV_COUNT == 24


def test_layer_entry_points_refuse_the_simulated_backend():
    ctx, ar = make()
    d = sb.make_desc(B=1, S=4, H=8, A=2, F=16)
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_layer_fwd(ctx, d, sb.make_weights({}), 0, ar.base, 0, 0, ar.base, 0)
    assert e.value.status == sb.E_UNSUPPORTED
    sb.ssdt_ctx_destroy(ctx)


def replay(ctx, reg, events, ptrs):
    """events: ('begin', s) | ('end', s) | ('save', key, bytes, numel) | ('weight', key).  `ptrs` maps
    key -> (device pointer, bytes)."""
    out = []
    for ev in events:
        if ev[0] == "begin":
            sb.ssdt_scope_begin(ctx, ev[1]); reg.scope_begin(ev[1])
        elif ev[0] == "end":
            sb.ssdt_scope_end(ctx, ev[1]); reg.scope_end(ev[1])
        elif ev[0] == "weight":
            sb.ssdt_register_weight(ctx, ptrs[ev[1]][0], ptrs[ev[1]][1]); reg.register_weight(ev[1])
        else:
            _, key, nbytes, numel = ev
            got = sb.ssdt_save(ctx, ptrs[key][0], nbytes, 0, [numel], sb.F32 if numel * 4 <= nbytes else sb.BF16)
            want = reg.save(key, nbytes, numel)
            out.append((got, want))
    return out


def compare(ctx, reg):
    st = sb.ssdt_get_stats(ctx)
    for k, v in vars(reg.c).items():
        assert st[k] == v, (k, st[k], v)
    recs = records(ctx)
    assert len(recs) == len(reg.records)
    cls = {ro.SMALL: sb.CLS_SMALL, ro.KEPT: sb.CLS_KEPT, ro.OFFLOADED: sb.CLS_OFFLOADED}
    for g, w in zip(recs, reg.records):
        assert (g["tid"], g["layer"], g["cls"], g["bytes"], g["pack_offset"], g["pool_offset"], g["n_scopes"]) == \
               (w.stamp, w.layer, cls[w.cls], w.bytes, w.pack_offset, w.pool_offset, len(w.scopes))


def test_hand_worked_trace_matches_checker():
    ctx, ar = make(min_offload_elems=10, budget_bytes=2000, keep_last=1)
    sb.ssdt_step_begin(ctx, 3)
    reg = ro.RegistryOracle(3, 10, 2000, 1, 1 << 20)
    wbuf = np.zeros(4000, dtype=np.uint8)
    ptrs = {"W": (wbuf.ctypes.data, 4000)}
    for key, n in (("a", 300), ("s", 16), ("b", 1000), ("c", 600), ("d", 200), ("e", 100), ("f", 50)):
        ptrs[key] = (sb.ssdt_arena_alloc(ctx, n), n)
    ev = [("weight", "W"), ("begin", 0), ("save", "W", 4000, 1000), ("save", "a", 300, 150), ("save", "s", 16, 4),
          ("save", "b", 1000, 500), ("save", "a", 300, 75), ("end", 0),
          ("begin", 1), ("save", "c", 600, 300), ("save", "d", 200, 100), ("save", "e", 100, 50), ("end", 1),
          ("begin", 2), ("save", "f", 50, 25), ("end", 2)]
    pairs = replay(ctx, reg, ev, ptrs)
    assert all(g == w for g, w in pairs), pairs
    assert [g for g, _ in pairs] == [0, 1, 0, 3, 1, 4, 5, 6, 7]
    compare(ctx, reg)
    sb.ssdt_ctx_destroy(ctx)


@pytest.mark.parametrize("arch,norm,act", [("gpt_preln", "layernorm", "gelu"), ("bert_postln", "layernorm", "gelu"),
                                           ("t5_enc", "rmsnorm", "relu")])
def test_layer_traces_match_checker(arch, norm, act):
    B, S, H, A, F, e, L = 2, 16, 32, 4, 128, 2, 3
    T = B * S
    tr = ro.saved_trace(arch, norm, act, T, H, F, B, A, S, e)
    for kw in (dict(min_offload_elems=0, keep_last=0, budget_bytes=-1), dict(min_offload_elems=T * H, keep_last=1, budget_bytes=-1),
               dict(min_offload_elems=0, keep_last=0, budget_bytes=3 * T * H * e)):
        ctx, ar = make(arena_bytes=4 << 20, pool_bytes=2 << 20, **kw)
        sb.ssdt_step_begin(ctx, L)
        reg = ro.RegistryOracle(L, kw["min_offload_elems"], None if kw["budget_bytes"] < 0 else kw["budget_bytes"],
                                kw["keep_last"], 2 << 20)
        for l in range(L):
            ptrs, events = {}, [("begin", l)]
            for name, storage, sbytes, numel in tr:
                if storage not in ptrs:
                    ptrs[storage] = (sb.ssdt_arena_alloc(ctx, sbytes), sbytes)
                events.append(("save", storage, sbytes, numel))
            events.append(("end", l))
            # storages are per layer: rename keys for the checker
            for evn in events:
                if evn[0] == "begin": reg.scope_begin(l); sb.ssdt_scope_begin(ctx, l)
                elif evn[0] == "end": reg.scope_end(l); sb.ssdt_scope_end(ctx, l)
                else:
                    _, key, nb, ne = evn
                    dt = sb.F32 if key.startswith(("mean", "rstd", "lse")) else sb.BF16
                    got = sb.ssdt_save(ctx, ptrs[key][0], nb, 0, [ne], dt)
                    assert got == reg.save((l, key), nb, ne)
        compare(ctx, reg)
        if arch == "gpt_preln" and kw["min_offload_elems"] == 0 and kw["budget_bytes"] < 0:
            st = sb.ssdt_get_stats(ctx)
            assert (st["save_calls"], st["unique"], st["dedup_hits"]) == (16 * L, 13 * L, 3 * L)
        sb.ssdt_ctx_destroy(ctx)


def test_views_share_an_id_and_weight_views_are_excluded():
    ctx, ar = make()
    sb.ssdt_step_begin(ctx, 1)
    T, H = 8, 4
    qkv = sb.ssdt_arena_alloc(ctx, T * 3 * H * 2)
    w = np.zeros(64, dtype=np.float32)
    sb.ssdt_register_weight(ctx, w.ctypes.data, w.nbytes)
    sb.ssdt_scope_begin(ctx, 0)
    ids = [sb.ssdt_save(ctx, qkv, T * 3 * H * 2, off, [T, H], sb.BF16) for off in (0, 0, 0)]
    # a "transposed" weight is another view of the weight's storage (Sec. 3.3.1)
    assert sb.ssdt_save(ctx, w.ctypes.data, w.nbytes, 0, [8, 8], sb.F32) == 0
    assert sb.ssdt_save(ctx, w.ctypes.data + 64, w.nbytes - 64, 0, [4, 4], sb.F32) == 0
    sb.ssdt_scope_end(ctx, 0)
    st = sb.ssdt_get_stats(ctx)
    assert ids[0] == ids[1] == ids[2] != 0
    assert (st["unique"], st["dedup_hits"], st["bypass_weight"], st["bytes_offloaded"]) == (1, 2, 2, T * 3 * H * 2)
    sb.ssdt_ctx_destroy(ctx)


def test_address_reuse_gets_a_new_stamp_and_store_completion_frees_the_slot():
    ctx, ar = make(arena_bytes=4096)
    sb.ssdt_step_begin(ctx, 2)
    a = sb.ssdt_arena_alloc(ctx, 4096)
    ar.view(a, 4096)[:] = 7
    sb.ssdt_scope_begin(ctx, 0)
    ta = sb.ssdt_save(ctx, a, 4096, 0, [1024], sb.F32)
    sb.ssdt_scope_end(ctx, 0)
    sb.ssdt_arena_free(ctx, a)                       # caller's reference gone, registry's remains
    assert sb.ssdt_get_stats(ctx)["arena_in_use"] == 4096
    sb.ssdt_offload(ctx, 0)
    assert records(ctx)[0]["state"] == sb.ST_STORING
    assert sb.ssdt_get_stats(ctx)["arena_in_use"] == 4096     # not reusable before the store completes
    assert sb.ssdt_sim_complete(ctx, 0, 1) == 1
    sb.ssdt_sync_io(ctx)
    assert records(ctx)[0]["state"] == sb.ST_OFFLOADED and records(ctx)[0]["device_ptr"] is None
    assert sb.ssdt_get_stats(ctx)["arena_in_use"] == 0
    b = sb.ssdt_arena_alloc(ctx, 4096)
    assert b == a                                    # same address, a different storage
    ar.view(b, 4096)[:] = 9
    sb.ssdt_scope_begin(ctx, 1)
    tb = sb.ssdt_save(ctx, b, 4096, 0, [1024], sb.F32)
    sb.ssdt_scope_end(ctx, 1)
    assert tb == ta + 1 and sb.ssdt_get_stats(ctx)["dedup_hits"] == 0
    assert sb.ssdt_pool_read(ctx, 0, 4096) == bytes([7]) * 4096
    sb.ssdt_ctx_destroy(ctx)


def test_fifo_stores_reverse_prefetch_forwarding_and_release():
    ctx, ar = make(arena_bytes=1 << 16)
    sb.ssdt_step_begin(ctx, 2)
    ptrs, tids = {}, {}
    for l, names in ((0, "abc"), (1, "de")):
        sb.ssdt_scope_begin(ctx, l)
        for i, n in enumerate(names):
            p = sb.ssdt_arena_alloc(ctx, 1024)
            ar.view(p, 1024)[:] = ord(n)
            ptrs[n] = p
            tids[n] = sb.ssdt_save(ctx, p, 1024, 0, [256], sb.F32)
            sb.ssdt_arena_free(ctx, p)
        sb.ssdt_scope_end(ctx, l)
        sb.ssdt_offload(ctx, l)
    # stores complete in submission order: after 2 completions exactly a and b are off the device
    assert sb.ssdt_sim_complete(ctx, 0, 2) == 2
    sb.ssdt_prefetch(ctx, 1)                          # d, e still being stored -> forwarded
    s = sb.ssdt_get_stats(ctx)
    assert s["forwarded"] == 2 and s["loads"] == 0
    assert sb.ssdt_get(ctx, tids["d"]) == ptrs["d"] and sb.ssdt_get(ctx, tids["e"]) == ptrs["e"]
    sb.ssdt_prefetch(ctx, 0)                          # c forwarded; b then a loaded, in that order
    s = sb.ssdt_get_stats(ctx)
    assert s["forwarded"] == 3 and s["loads"] == 2
    rec = {r["tid"]: r for r in records(ctx)}
    assert rec[tids["a"]]["state"] == sb.ST_LOADING and rec[tids["b"]]["state"] == sb.ST_LOADING
    assert sb.ssdt_sim_complete(ctx, 1, 1) == 1       # the first load to finish is b's (reverse order)
    pb = rec[tids["b"]]["device_ptr"]; pa = rec[tids["a"]]["device_ptr"]
    assert bytes(ar.view(pb, 1024)) == b"b" * 1024
    assert bytes(ar.view(pa, 1024)) != b"a" * 1024
    assert sb.ssdt_get(ctx, tids["a"]) == pa          # get waits for the load
    assert bytes(ar.view(pa, 1024)) == b"a" * 1024
    # release: memory returns, later use is an error
    before = sb.ssdt_get_stats(ctx)["arena_in_use"]
    sb.ssdt_release(ctx, 1)
    assert sb.ssdt_get_stats(ctx)["arena_in_use"] == before - 2048
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_get(ctx, tids["d"])
    assert e.value.status == sb.E_STATE
    sb.ssdt_release(ctx, 0)
    assert sb.ssdt_get_stats(ctx)["arena_in_use"] == 0 and sb.ssdt_get_stats(ctx)["released"] == 5
    sb.ssdt_step_begin(ctx, 2)                        # a clean step can start
    sb.ssdt_ctx_destroy(ctx)


def test_shared_storage_released_after_its_last_scope_and_caller_reference_keeps_it():
    ctx, ar = make(arena_bytes=1 << 16)
    sb.ssdt_step_begin(ctx, 2)
    enc = sb.ssdt_arena_alloc(ctx, 2048)
    ar.view(enc, 2048)[:] = 5
    sb.ssdt_scope_begin(ctx, 0); t0 = sb.ssdt_save(ctx, enc, 2048, 0, [512], sb.F32); sb.ssdt_scope_end(ctx, 0)
    sb.ssdt_offload(ctx, 0)
    sb.ssdt_sim_complete(ctx, 0, 1); sb.ssdt_sync_io(ctx)
    # the store is done but the caller still holds the block: it must not be reused
    assert sb.ssdt_get_stats(ctx)["arena_in_use"] == 2048
    other = sb.ssdt_arena_alloc(ctx, 2048)
    assert other != enc
    sb.ssdt_scope_begin(ctx, 1); t1 = sb.ssdt_save(ctx, enc, 2048, 0, [512], sb.F32); sb.ssdt_scope_end(ctx, 1)
    assert t1 == t0 and sb.ssdt_get_stats(ctx)["dedup_hits"] == 1 and sb.ssdt_get_stats(ctx)["bytes_offloaded"] == 2048
    sb.ssdt_offload(ctx, 1)                           # nothing new to store
    assert sb.ssdt_sim_complete(ctx, 0, 5) == 0
    sb.ssdt_arena_free(ctx, enc)
    sb.ssdt_prefetch(ctx, 0)
    p = sb.ssdt_get(ctx, t0)
    assert bytes(ar.view(p, 2048)) == bytes([5]) * 2048
    sb.ssdt_release(ctx, 1)
    assert records(ctx)[0]["state"] == sb.ST_RESIDENT and records(ctx)[0]["n_scopes"] == 1
    sb.ssdt_release(ctx, 0)
    assert records(ctx)[0]["state"] == sb.ST_RELEASED
    sb.ssdt_ctx_destroy(ctx)


def test_arena_pressure_waits_for_the_oldest_store():
    ctx, ar = make(arena_bytes=2048)
    sb.ssdt_step_begin(ctx, 2)
    a = sb.ssdt_arena_alloc(ctx, 1024); ar.view(a, 1024)[:] = 1
    b = sb.ssdt_arena_alloc(ctx, 1024); ar.view(b, 1024)[:] = 2
    sb.ssdt_scope_begin(ctx, 0)
    ta = sb.ssdt_save(ctx, a, 1024, 0, [256], sb.F32); tb = sb.ssdt_save(ctx, b, 1024, 0, [256], sb.F32)
    sb.ssdt_scope_end(ctx, 0)
    sb.ssdt_arena_free(ctx, a); sb.ssdt_arena_free(ctx, b)
    sb.ssdt_offload(ctx, 0)
    c = sb.ssdt_arena_alloc(ctx, 1024)                # full: waits for a's store, then reuses a's block
    assert c == a and records(ctx)[0]["state"] == sb.ST_OFFLOADED and records(ctx)[1]["state"] == sb.ST_STORING
    assert sb.ssdt_pool_read(ctx, 0, 1024) == bytes([1]) * 1024
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_arena_alloc(ctx, 4096)
    assert e.value.status == sb.E_NOMEM
    sb.ssdt_ctx_destroy(ctx)


def test_error_paths():
    ctx, ar = make()
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_scope_begin(ctx, 0)                   # no step
    assert e.value.status == sb.E_STATE
    sb.ssdt_step_begin(ctx, 1)
    p = sb.ssdt_arena_alloc(ctx, 256)
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_save(ctx, p, 256, 0, [64], sb.F32)    # outside a scope
    assert e.value.status == sb.E_STATE
    sb.ssdt_scope_begin(ctx, 0)
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_save(ctx, p, 256, 0, [65], sb.F32)    # view larger than storage
    assert e.value.status == sb.E_INVAL
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_scope_end(ctx, 3)
    assert e.value.status == sb.E_STATE
    assert sb.ssdt_get_stats(ctx)["save_calls"] == 0  # failed calls left no trace
    t = sb.ssdt_save(ctx, p, 256, 0, [64], sb.F32)
    sb.ssdt_scope_end(ctx, 0)
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_get(ctx, 999)
    assert e.value.status == sb.E_NOTFOUND
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_step_begin(ctx, 1)                    # previous step not released
    assert e.value.status == sb.E_STATE
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_arena_free(ctx, p + 64)
    assert e.value.status == sb.E_STATE
    sb.ssdt_release(ctx, 0)
    sb.ssdt_ctx_destroy(ctx)
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_ctx_create(backend=sb.BACKEND_SIM, arena_base=ar.base + 8, arena_bytes=1024)
    assert e.value.status == sb.E_INVAL
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_ctx_create(backend=sb.BACKEND_SIM, spill_path="/nonexistent-dir/spill.bin")
    assert e.value.status == sb.E_IO


def _spill_step(ctx, ar, fill):
    """Two layers of three 1 KiB tensors each; returns {name: (tid, pool_offset)}."""
    sb.ssdt_step_begin(ctx, 2)
    out = {}
    for l, names in ((0, "abc"), (1, "def")):
        sb.ssdt_scope_begin(ctx, l)
        for n in names:
            p = sb.ssdt_arena_alloc(ctx, 1024)
            ar.view(p, 1024)[:] = fill[n]
            out[n] = sb.ssdt_save(ctx, p, 1024, 0, [256], sb.F32)
            sb.ssdt_arena_free(ctx, p)
        sb.ssdt_scope_end(ctx, l)
        sb.ssdt_offload(ctx, l)
    rec = {r["tid"]: r for r in records(ctx)}
    return {n: (t, rec[t]["pool_offset"]) for n, t in out.items()}


def test_spill_file_is_the_store_and_reloads_are_bit_identical(tmp_path):
    path = str(tmp_path / "spill.bin")
    ctx, ar = make(arena_bytes=1 << 16, spill_path=path)
    for step in range(2):                               # the second step reuses the same file offsets
        fill = {n: (ord(n) + 7 * step) & 0xFF for n in "abcdef"}
        t = _spill_step(ctx, ar, fill)
        assert sb.ssdt_sim_complete(ctx, 0, 4) == 4     # a..d are off the device, e and f still on their way
        sb.ssdt_prefetch(ctx, 1)                        # f, e forwarded; d comes back from the file
        sb.ssdt_prefetch(ctx, 0)
        s = sb.ssdt_get_stats(ctx)
        assert s["forwarded"] == 2 and s["loads"] == 4
        for n in "fedcba":
            p = sb.ssdt_get(ctx, t[n][0])
            assert bytes(ar.view(p, 1024)) == bytes([fill[n]]) * 1024, n
        sb.ssdt_sync_io(ctx)
        w, r = sb.ssdt_spill_stats(ctx)
        assert (w, r) == (4096 * (step + 1), 4096 * (step + 1))   # forwarded tensors never reach the file
        with open(path, "rb") as f:
            blob = f.read()
        for n in "abcd":
            off = t[n][1]
            assert blob[off:off + 1024] == bytes([fill[n]]) * 1024
            assert sb.ssdt_pool_read(ctx, off, 1024) == bytes([fill[n]]) * 1024
        sb.ssdt_release(ctx, 1)
        sb.ssdt_release(ctx, 0)
        assert sb.ssdt_get_stats(ctx)["arena_in_use"] == 0
    sb.ssdt_ctx_destroy(ctx)


def test_spill_layout_is_block_aligned_and_io_is_chunked(tmp_path):
    """With a spill file every tensor starts on a 4096-byte boundary of pool and file (the bookkeeping checker with
    tensor_align = 4096 gives the same offsets), the file is served by the configured number of threads, and a tensor
    larger than one request (8 MiB) is written and read back in several chunks, bit for bit."""
    big = (20 << 20) + 1024                                  # three requests, the last one short and padded
    ar = Arena((64 << 20) + 4096)
    ctx = sb.ssdt_ctx_create(backend=sb.BACKEND_SIM, keep_last=0, min_offload_elems=0, budget_bytes=-1,
                             arena_base=ar.base, arena_bytes=64 << 20, pool_bytes=48 << 20,
                             spill_path=str(tmp_path / "big.bin"), spill_threads=3)
    info = sb.ssdt_spill_info(ctx)
    assert info["threads"] == 3 and info["direct_io"] in (0, 1)
    sizes = [1024, big, 768, 4096]
    rng = np.random.default_rng(3)
    sb.ssdt_step_begin(ctx, 1)
    sb.ssdt_scope_begin(ctx, 0)
    tids, data = [], []
    reg = ro.RegistryOracle(1, 0, None, 0, 48 << 20, tensor_align=4096)
    reg.scope_begin(0)
    for i, n in enumerate(sizes):
        p = sb.ssdt_arena_alloc(ctx, n)
        blob = rng.integers(0, 256, n, dtype=np.uint8)
        ar.view(p, n)[:] = blob
        data.append(blob.tobytes())
        tids.append(sb.ssdt_save(ctx, p, n, 0, [n // 4], sb.F32))
        reg.save(("t", i), n, n // 4)
        sb.ssdt_arena_free(ctx, p)
    sb.ssdt_scope_end(ctx, 0)
    reg.scope_end(0)
    recs = records(ctx)
    assert [(r["pack_offset"], r["pool_offset"]) for r in recs] == [(r.pack_offset, r.pool_offset) for r in reg.records]
    assert all(r["pool_offset"] % 4096 == 0 for r in recs)
    sb.ssdt_offload(ctx, 0)
    assert sb.ssdt_sim_complete(ctx, 0, 4) == 4
    sb.ssdt_sync_io(ctx)                                     # copies done, all four written
    for r, blob in zip(recs, data):                          # the file holds them; the pool copies are gone
        assert sb.ssdt_pool_read(ctx, r["pool_offset"], r["bytes"]) == blob
    sb.ssdt_prefetch(ctx, 0)
    for t, blob in zip(tids, data):
        p = sb.ssdt_get(ctx, t)
        assert bytes(ar.view(p, len(blob))) == blob
    info = sb.ssdt_spill_info(ctx)
    assert info["bytes_written"] == sum(sizes) and info["bytes_read"] == sum(sizes)
    assert info["write_busy_ns"] > 0 and info["read_busy_ns"] > 0
    sb.ssdt_release(ctx, 0)
    sb.ssdt_ctx_destroy(ctx)


def test_spill_release_before_the_read_was_used_and_demand_load(tmp_path):
    ctx, ar = make(arena_bytes=1 << 16, spill_path=str(tmp_path / "s.bin"))
    fill = {n: ord(n) for n in "abcdef"}
    t = _spill_step(ctx, ar, fill)
    sb.ssdt_sync_io(ctx)                                # everything stored and written
    p = sb.ssdt_get(ctx, t["e"][0])                     # nobody prefetched it: demand load through the file
    assert bytes(ar.view(p, 1024)) == b"e" * 1024
    assert sb.ssdt_get_stats(ctx)["demand_loads"] == 1
    sb.ssdt_prefetch(ctx, 0)                            # reads requested ...
    sb.ssdt_release(ctx, 0)                             # ... and the scope released before any copy was issued
    sb.ssdt_release(ctx, 1)
    assert sb.ssdt_get_stats(ctx)["arena_in_use"] == 0
    sb.ssdt_step_begin(ctx, 2)
    sb.ssdt_ctx_destroy(ctx)


def test_spill_write_failure_is_reported():
    ctx, ar = make(arena_bytes=1 << 16, spill_path="/dev/full")    # every write fails with ENOSPC
    t = _spill_step(ctx, ar, {n: ord(n) for n in "abcdef"})
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_sync_io(ctx)
    assert e.value.status == sb.E_IO and "spill write" in str(e.value)
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_prefetch(ctx, 1)
    assert e.value.status == sb.E_IO
    sb.ssdt_ctx_destroy(ctx)


def test_recompute_inside_backward_keeps_everything_and_matches_checker():
    """Layerwise full recomputation through the registry: forward saves only each layer's input, the
    layer's own saves repeat inside its backward scope and stay on the device (Sec. 3.2, Sec. 4.3)."""
    B, S, H, A, F, e, L = 2, 16, 32, 4, 128, 2, 3
    T = B * S
    tr = ro.saved_trace("gpt_preln", "layernorm", "gelu", T, H, F, B, A, S, e)
    ctx, ar = make(arena_bytes=4 << 20, pool_bytes=2 << 20, min_offload_elems=0, keep_last=1, budget_bytes=-1)
    sb.ssdt_step_begin(ctx, L)
    reg = ro.RegistryOracle(L, 0, None, 1, 2 << 20)
    xs = {}
    for l in range(L):                                    # forward: inputs only
        xs[l] = sb.ssdt_arena_alloc(ctx, T * H * e)
        sb.ssdt_scope_begin(ctx, l); reg.scope_begin(l)
        assert sb.ssdt_save(ctx, xs[l], T * H * e, 0, [T * H], sb.BF16) == reg.save((l, "x"), T * H * e, T * H)
        sb.ssdt_scope_end(ctx, l); reg.scope_end(l)
        sb.ssdt_offload(ctx, l)
        sb.ssdt_arena_free(ctx, xs[l])                    # the caller's reference; the record keeps its own
    sb.ssdt_sync_io(ctx)
    st = sb.ssdt_get_stats(ctx)
    assert st["offloaded"] == L - 1 and st["kept"] == 1 and st["arena_in_use"] == T * H * e  # the kept last input
    for l in range(L - 1, -1, -1):                        # backward: reload the input, recompute, release
        sb.ssdt_prefetch(ctx, l)
        sb.ssdt_scope_begin(ctx, l, sb.BWD); reg.backward_begin()
        tid = [r for r in records(ctx) if r["layer"] == l][0]["tid"]
        x = sb.ssdt_get(ctx, tid)
        ptrs = {"x": x}
        sb.ssdt_scope_begin(ctx, l); reg.scope_begin(l)
        for name, storage, sbytes, numel in tr:
            if storage not in ptrs:
                ptrs[storage] = sb.ssdt_arena_alloc(ctx, sbytes)
            dt = sb.F32 if storage.startswith(("mean", "rstd", "lse")) else sb.BF16
            assert sb.ssdt_save(ctx, ptrs[storage], sbytes, 0, [numel], dt) == reg.save((l, storage), sbytes, numel)
        sb.ssdt_scope_end(ctx, l); reg.scope_end(l)
        for k, p in ptrs.items():
            if k != "x":
                sb.ssdt_arena_free(ctx, p)
        sb.ssdt_scope_end(ctx, l, sb.BWD); reg.backward_end()
        sb.ssdt_release(ctx, l)
    compare_counts = sb.ssdt_get_stats(ctx)
    for k, v in vars(reg.c).items():
        assert compare_counts[k] == v, (k, compare_counts[k], v)
    recs = records(ctx)
    assert len(recs) == len(reg.records) == L * 13
    assert [r["cls"] for r in recs[L:]] == [sb.CLS_KEPT if w.cls == ro.KEPT else sb.CLS_SMALL for w in reg.records[L:]]
    assert all(w.cls != ro.OFFLOADED for w in reg.records[L:])
    assert compare_counts["offloaded"] == L - 1 and compare_counts["loads"] == L - 1
    assert compare_counts["arena_in_use"] == 0
    sb.ssdt_ctx_destroy(ctx)


def test_layer_descriptors_are_validated_without_a_gpu():
    """ssdt_layer_workspace checks a descriptor with the same rules as the layer entry points."""
    good = dict(arch="gpt_preln", dtype="bf16", B=2, S=128, H=256, A=4, F=1024)
    f, b = sb.ssdt_layer_workspace(sb.make_desc(**good))
    assert f > 0 and b >= f                      # transposed-operand scratch; backward needs the gradient temporaries too
    for bad in (dict(B=0), dict(S=0), dict(H=0), dict(A=0), dict(F=0), dict(A=3), dict(B=-1), dict(eps=0.0)):
        with pytest.raises(sb.SsdtError) as e:
            sb.ssdt_layer_workspace(sb.make_desc(**{**good, **bad}))
        assert e.value.status == sb.E_INVAL, bad
    d = sb.make_desc(**good)
    d.arch = 17
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_layer_workspace(d)
    assert e.value.status == sb.E_INVAL
    with pytest.raises(sb.SsdtError) as e:       # a decoder layer needs the encoder length
        sb.ssdt_layer_workspace(sb.make_desc(**{**good, "arch": "t5_dec", "S_kv": 0}))
    assert e.value.status == sb.E_INVAL
    with pytest.raises(sb.SsdtError) as e:       # more tokens than the kernels index
        sb.ssdt_layer_workspace(sb.make_desc(**{**good, "B": 1 << 20, "S": 1 << 12}))
    assert e.value.status == sb.E_UNSUPPORTED


def test_records_per_micro_batch_match_checker():
    """Two micro-batches between forward and backward at the same time (Sec. 3.1): forward 0, forward 1, backward
    1, backward 0, with the layer traces of a GPT layer; bookkeeping against the checker, and the data of each
    micro-batch comes back to its own records."""
    B, S, H, A, F, e, L = 2, 16, 32, 4, 128, 2, 2
    T = B * S
    tr = ro.saved_trace("gpt_preln", "layernorm", "gelu", T, H, F, B, A, S, e)
    ctx, ar = make(arena_bytes=4 << 20, pool_bytes=2 << 20, min_offload_elems=0, keep_last=1, budget_bytes=-1)
    sb.ssdt_step_begin(ctx, L)
    reg = ro.RegistryOracle(L, 0, None, 1, 2 << 20)
    tids = {}
    for mb, kl in ((0, 0), (1, -1)):
        sb.ssdt_micro_batch(ctx, mb, kl); reg.micro_batch(mb, None if kl < 0 else kl)
        for l in range(L):
            sb.ssdt_scope_begin(ctx, l); reg.scope_begin(l)
            ptrs = {}
            for name, storage, sbytes, numel in tr:
                if storage not in ptrs:
                    ptrs[storage] = sb.ssdt_arena_alloc(ctx, sbytes)
                    ar.view(ptrs[storage], sbytes)[:] = (17 * mb + 5 * l + len(ptrs)) & 0xFF
                dt = sb.F32 if storage.startswith(("mean", "rstd", "lse")) else sb.BF16
                got = sb.ssdt_save(ctx, ptrs[storage], sbytes, 0, [numel], dt)
                assert got == reg.save((mb, l, storage), sbytes, numel)
                tids[(mb, l, storage)] = (got, sbytes, (17 * mb + 5 * l + list(ptrs).index(storage) + 1) & 0xFF)
            sb.ssdt_scope_end(ctx, l); reg.scope_end(l)
            sb.ssdt_offload(ctx, l)
            for p in ptrs.values():
                sb.ssdt_arena_free(ctx, p)
    compare(ctx, reg)
    recs = records(ctx)
    assert [r["micro_batch"] for r in recs] == [0] * 26 + [1] * 26
    assert sum(1 for r in recs if r["cls"] == sb.CLS_KEPT) == 13         # only the last layer of micro-batch 1
    sb.ssdt_sync_io(ctx)
    for mb in (1, 0):
        sb.ssdt_micro_batch(ctx, mb)
        for l in (1, 0):
            sb.ssdt_prefetch(ctx, l)
            for (m2, l2, storage), (tid, sbytes, fill) in tids.items():
                if (m2, l2) == (mb, l):
                    p = sb.ssdt_get(ctx, tid)
                    assert bytes(ar.view(p, sbytes)) == bytes([fill]) * sbytes, (mb, l, storage)
            sb.ssdt_release(ctx, l)
    st = sb.ssdt_get_stats(ctx)
    assert st["arena_in_use"] == 0 and st["released"] == 52 and st["loads"] == 39
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_micro_batch(ctx, -1)
    assert e.value.status == sb.E_INVAL
    sb.ssdt_scope_begin(ctx, 0)
    with pytest.raises(sb.SsdtError) as e:
        sb.ssdt_micro_batch(ctx, 1)
    assert e.value.status == sb.E_STATE
    sb.ssdt_scope_end(ctx, 0)
    sb.ssdt_step_begin(ctx, L)
    sb.ssdt_ctx_destroy(ctx)


def test_random_traces_match_checker_and_reload_bit_exactly():
    """Seeded random sequences of scopes, saves (views, repeats, weights, small tensors), budgets, kept layers and
    micro-batches, with stores and loads completing in random amounts: bookkeeping equals the checker's record by
    record, no two live arena blocks overlap, and every tensor fetched in backward holds the bytes it was saved
    with."""
    rng = np.random.default_rng(20240810)
    for trial in range(40):
        L = int(rng.integers(1, 5))
        n_mb = int(rng.integers(1, 3))
        kw = dict(min_offload_elems=int(rng.choice([0, 64, 1 << 20])), keep_last=int(rng.integers(0, 2)),
                  budget_bytes=int(rng.choice([-1, 0, 3000, 20000])))
        pool = int(rng.choice([1 << 12, 1 << 16, 1 << 20]))
        ctx, ar = make(arena_bytes=1 << 20, pool_bytes=pool, **kw)
        sb.ssdt_step_begin(ctx, L)
        reg = ro.RegistryOracle(L, kw["min_offload_elems"], None if kw["budget_bytes"] < 0 else kw["budget_bytes"],
                                kw["keep_last"], pool)
        wbuf = np.zeros(4096, dtype=np.uint8)
        sb.ssdt_register_weight(ctx, wbuf.ctypes.data, 4096); reg.register_weight("W")
        live = {}                                   # (mb, layer, name) -> (tid, ptr, bytes, fill)
        for mb in range(n_mb):
            klo = int(rng.integers(-1, 2))
            sb.ssdt_micro_batch(ctx, mb, klo); reg.micro_batch(mb, None if klo < 0 else klo)
            for l in range(L):
                sb.ssdt_scope_begin(ctx, l); reg.scope_begin(l)
                mine = {}
                for s_i in range(int(rng.integers(1, 7))):
                    kind = rng.integers(0, 10)
                    if kind == 0:                   # a weight: bypassed
                        assert sb.ssdt_save(ctx, wbuf.ctypes.data, 4096, 0, [1024], sb.F32) == 0
                        assert reg.save("W", 4096, 1024) == 0
                        continue
                    if kind <= 2 and mine:          # another view of a storage saved before
                        name = list(mine)[int(rng.integers(0, len(mine)))]
                    else:
                        name = "t%d" % s_i
                        nbytes = int(rng.choice([64, 256, 1000, 4096, 10000]))
                        p = sb.ssdt_arena_alloc(ctx, nbytes)
                        fill = int(rng.integers(1, 255))
                        ar.view(p, nbytes)[:] = fill
                        mine[name] = (p, nbytes, fill)
                    p, nbytes, fill = mine[name]
                    numel = int(rng.integers(1, nbytes // 4 + 1))
                    got = sb.ssdt_save(ctx, p, nbytes, 0, [numel], sb.F32)
                    assert got == reg.save((mb, l, name), nbytes, numel)
                    live[(mb, l, name)] = (got, p, nbytes, fill)
                sb.ssdt_scope_end(ctx, l); reg.scope_end(l)
                sb.ssdt_offload(ctx, l)
                for p, _, _ in mine.values():
                    sb.ssdt_arena_free(ctx, p)
                sb.ssdt_sim_complete(ctx, 0, int(rng.integers(0, 4)))
        compare(ctx, reg)
        recs = records(ctx)
        spans = sorted((r["device_ptr"], r["bytes"]) for r in recs if r["device_ptr"])
        for (a, na), (b, _) in zip(spans, spans[1:]):
            assert a + na <= b, "live arena blocks overlap"
        sb.ssdt_sim_complete(ctx, 0, int(rng.choice([0, 1, 2, 50])))   # some stores are still in flight: forwarding
        for mb in reversed(range(n_mb)):
            sb.ssdt_micro_batch(ctx, mb)
            for l in reversed(range(L)):
                if rng.integers(0, 2):
                    sb.ssdt_prefetch(ctx, l)
                sb.ssdt_sim_complete(ctx, 1, int(rng.integers(0, 3)))
                for (m2, l2, name), (tid, p, nbytes, fill) in live.items():
                    if (m2, l2) != (mb, l):
                        continue
                    q = sb.ssdt_get(ctx, tid) if tid else p      # bypassed tensors stay where they were
                    assert bytes(ar.view(q, nbytes)) == bytes([fill]) * nbytes, (trial, mb, l, name)
                sb.ssdt_release(ctx, l)
        st = sb.ssdt_get_stats(ctx)
        assert st["arena_in_use"] == 0 and st["released"] == st["unique"], (trial, st)
        assert st["loads"] + st["forwarded"] <= st["offloaded"] + st["demand_loads"]
        sb.ssdt_step_begin(ctx, L)
        sb.ssdt_ctx_destroy(ctx)
