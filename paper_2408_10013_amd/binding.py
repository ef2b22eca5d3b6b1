"""ctypes binding of libssdt.so: the same names as the C ABI, argument marshalling only.

Every function raises SsdtError on a non-zero status.  Device pointers are plain integers
(e.g. torch.Tensor.data_ptr()); streams are hipStream_t values as integers
(torch.cuda.Stream.cuda_stream), 0 for the default stream.  There is no fallback: if the
library has not been built, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libssdt.so")

OK, E_INVAL, E_NOMEM, E_HIP, E_IO, E_STATE, E_NOTFOUND, E_UNSUPPORTED = 0, -1, -2, -3, -4, -5, -6, -7
BACKEND_HIP, BACKEND_SIM = 0, 1
FWD, BWD = 0, 1
F32, BF16 = 0, 1
CLS_SMALL, CLS_KEPT, CLS_OFFLOADED = 1, 2, 3
ST_RESIDENT, ST_STORING, ST_OFFLOADED, ST_LOADING, ST_RELEASED = 1, 2, 3, 4, 5
ARCH = {"gpt_preln": 0, "bert_postln": 1, "t5_enc": 2, "t5_dec": 3}
ACT = {"gelu": 0, "relu": 1}
NORM = {"layernorm": 0, "rmsnorm": 1}
MASK = {"none": 0, "causal": 1, "keypad": 2}
DTYPE = {"f32": 0, "bf16": 1}

SV_NAMES = ["x", "mean1", "rstd1", "a", "qkv", "o", "lse", "r1", "x1", "meanx", "rstdx", "ax", "enc", "qx", "kvx",
            "ox", "lsex", "x2", "mean2", "rstd2", "m", "h1", "g", "r2"]
SV_COUNT = len(SV_NAMES)
WEIGHT_NAMES = ["ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "lnx_g", "lnx_b", "w_qx", "b_qx", "w_kvx", "b_kvx",
                "w_ox", "b_ox", "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2"]


class SsdtError(RuntimeError):
    def __init__(self, status: int, where: str, msg: str = ""):
        super().__init__("%s failed with status %d%s" % (where, status, (": " + msg) if msg else ""))
        self.status = status


class ssdt_config(C.Structure):
    _fields_ = [("backend", C.c_int32), ("keep_last", C.c_int32), ("min_offload_elems", C.c_int64),
                ("budget_bytes", C.c_int64), ("arena_base", C.c_void_p), ("arena_bytes", C.c_size_t),
                ("pool_bytes", C.c_size_t), ("spill_path", C.c_char_p), ("measure_waits", C.c_int32),
                ("spill_threads", C.c_int32)]


class ssdt_stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "save_calls", "unique", "dedup_hits", "bypass_weight", "bypass_small", "kept", "offloaded",
        "bytes_small", "bytes_kept", "bytes_offloaded", "pool_bytes_used",
        "loads", "bytes_loaded", "forwarded", "demand_loads", "released",
        "arena_in_use", "arena_high_water", "arena_peak_in_use", "arena_allocs",
        "exposed_load_wait_ns", "exposed_store_wait_ns")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class ssdt_record(C.Structure):
    _fields_ = [("tid", C.c_uint64), ("layer", C.c_int32), ("cls", C.c_int32), ("state", C.c_int32),
                ("n_scopes", C.c_int32), ("bytes", C.c_uint64), ("pack_offset", C.c_int64),
                ("pool_offset", C.c_int64), ("device_ptr", C.c_void_p), ("micro_batch", C.c_int32),
                ("reserved", C.c_int32)]


class ssdt_spill_info_t(C.Structure):
    _fields_ = [("direct_io", C.c_int32), ("threads", C.c_int32), ("bytes_written", C.c_uint64),
                ("bytes_read", C.c_uint64), ("write_busy_ns", C.c_uint64), ("read_busy_ns", C.c_uint64)]


class ssdt_plan_in(C.Structure):
    _fields_ = [("num_layers", C.c_int32), ("keep_last", C.c_int32), ("layer_bytes", C.POINTER(C.c_uint64)),
                ("fwd_s", C.POINTER(C.c_double)), ("bwd_s", C.POINTER(C.c_double)), ("store_Bps", C.c_double),
                ("load_Bps", C.c_double), ("safety", C.c_double)]


class ssdt_plan_out(C.Structure):
    _fields_ = [("budget_bytes", C.c_int64), ("layers", C.c_int32), ("prefetch_distance", C.c_int32),
                ("partial_bytes", C.c_uint64), ("store_done_s", C.c_double), ("fwd_total_s", C.c_double)]


class ssdt_kernel_time(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_uint64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


class ssdt_layer_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("arch", "dtype", "act", "norm", "mask", "has_bias", "B", "S", "S_kv", "H",
                                         "A", "F")] + [("eps", C.c_float), ("softmax_scale", C.c_float),
                                                        ("checkpoint", C.c_int32), ("accumulate", C.c_int32)]


class ssdt_bwd_temporaries(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("d_h1", "t0", "t1", "t2", "d_qkv", "d_kvx")]


class ssdt_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_NAMES]


class ssdt_saved_entry(C.Structure):
    _fields_ = [("tid", C.c_uint64), ("ptr", C.c_void_p), ("bytes", C.c_uint64)]


class ssdt_layer_saved(C.Structure):
    _fields_ = [("scope", C.c_int32), ("reserved", C.c_int32), ("e", ssdt_saved_entry * SV_COUNT)]


_lib = None

_PROTOS = {
    "ssdt_last_error": (C.c_char_p, [C.c_void_p]),
    "ssdt_version": (C.c_char_p, []),
    "ssdt_ctx_create": (C.c_int32, [C.POINTER(ssdt_config), C.POINTER(C.c_void_p)]),
    "ssdt_ctx_destroy": (C.c_int32, [C.c_void_p]),
    "ssdt_step_begin": (C.c_int32, [C.c_void_p, C.c_int32]),
    "ssdt_micro_batch": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32]),
    "ssdt_set_budget": (C.c_int32, [C.c_void_p, C.c_int64]),
    "ssdt_arena_alloc": (C.c_int32, [C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]),
    "ssdt_arena_free": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p]),
    "ssdt_register_weight": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_size_t]),
    "ssdt_scope_begin": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32]),
    "ssdt_scope_end": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32]),
    "ssdt_save": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_size_t, C.c_size_t, C.POINTER(C.c_int64), C.c_int32,
                              C.c_int32, C.POINTER(C.c_uint64)]),
    "ssdt_offload": (C.c_int32, [C.c_void_p, C.c_int32, C.c_void_p]),
    "ssdt_prefetch": (C.c_int32, [C.c_void_p, C.c_int32]),
    "ssdt_get": (C.c_int32, [C.c_void_p, C.c_uint64, C.c_void_p, C.POINTER(C.c_void_p)]),
    "ssdt_release": (C.c_int32, [C.c_void_p, C.c_int32, C.c_void_p]),
    "ssdt_get_stats": (C.c_int32, [C.c_void_p, C.POINTER(ssdt_stats)]),
    "ssdt_num_records": (C.c_int32, [C.c_void_p, C.POINTER(C.c_uint32)]),
    "ssdt_get_record": (C.c_int32, [C.c_void_p, C.c_uint32, C.POINTER(ssdt_record)]),
    "ssdt_pool_read": (C.c_int32, [C.c_void_p, C.c_size_t, C.c_void_p, C.c_size_t]),
    "ssdt_sim_complete": (C.c_int32, [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]),
    "ssdt_sync_io": (C.c_int32, [C.c_void_p]),
    "ssdt_plan": (C.c_int32, [C.POINTER(ssdt_plan_in), C.POINTER(ssdt_plan_out)]),
    "ssdt_spill_info": (C.c_int32, [C.c_void_p, C.POINTER(ssdt_spill_info_t)]),
    "ssdt_spill_stats": (C.c_int32, [C.c_void_p, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]),
    "ssdt_profile": (C.c_int32, [C.c_void_p, C.c_int32]),
    "ssdt_profile_read": (C.c_int32, [C.c_void_p, C.POINTER(ssdt_kernel_time), C.c_uint32, C.POINTER(C.c_uint32)]),
    "ssdt_sgd_update": (C.c_int32, [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_float, C.c_void_p]),
    "ssdt_layer_workspace": (C.c_int32, [C.POINTER(ssdt_layer_desc), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "ssdt_layer_bwd_temporaries": (C.c_int32, [C.POINTER(ssdt_layer_desc), C.POINTER(ssdt_bwd_temporaries)]),
    "ssdt_layer_fwd": (C.c_int32, [C.c_void_p, C.POINTER(ssdt_layer_desc), C.POINTER(ssdt_layer_weights), C.c_int32,
                                   C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p),
                                   C.POINTER(ssdt_layer_saved), C.c_void_p, C.c_size_t, C.c_void_p]),
    "ssdt_layer_bwd_static": (C.c_int32, [C.c_void_p, C.POINTER(ssdt_layer_desc), C.POINTER(ssdt_layer_weights),
                                          C.POINTER(ssdt_layer_saved), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.POINTER(ssdt_layer_weights), C.c_void_p]),
    "ssdt_layer_bwd": (C.c_int32, [C.c_void_p, C.POINTER(ssdt_layer_desc), C.POINTER(ssdt_layer_weights),
                                   C.POINTER(ssdt_layer_saved), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.POINTER(ssdt_layer_weights), C.c_void_p, C.c_size_t, C.c_void_p]),
}


def lib():
    """Opens libssdt.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError("%s is missing: build it with `python -m paper_2408_10013_amd.build`" % LIB_PATH)
        l = C.CDLL(LIB_PATH)
        for name, (res, args) in _PROTOS.items():
            f = getattr(l, name)
            f.restype, f.argtypes = res, args
        _lib = l
    return _lib


def exported_symbols():
    return list(_PROTOS)


def _check(ctx, status, where):
    if status != OK:
        msg = ""
        if ctx:
            m = lib().ssdt_last_error(ctx)
            msg = m.decode() if m else ""
        raise SsdtError(status, where, msg)


# ---- thin wrappers, same names as the C entry points ----------------------------------------

def ssdt_version() -> str:
    return lib().ssdt_version().decode()


def ssdt_ctx_create(backend=BACKEND_HIP, keep_last=1, min_offload_elems=1 << 20, budget_bytes=-1, arena_base=0,
                    arena_bytes=0, pool_bytes=0, spill_path: Optional[str] = None, measure_waits=0,
                    spill_threads=0) -> int:
    cfg = ssdt_config(backend, keep_last, min_offload_elems, budget_bytes, arena_base or None, arena_bytes, pool_bytes,
                      spill_path.encode() if spill_path else None, measure_waits, spill_threads)
    out = C.c_void_p()
    _check(None, lib().ssdt_ctx_create(C.byref(cfg), C.byref(out)), "ssdt_ctx_create")
    return out.value


def ssdt_ctx_destroy(ctx):
    _check(None, lib().ssdt_ctx_destroy(ctx), "ssdt_ctx_destroy")


def ssdt_step_begin(ctx, num_layers):
    _check(ctx, lib().ssdt_step_begin(ctx, num_layers), "ssdt_step_begin")


def ssdt_micro_batch(ctx, mb, keep_last=-1):
    _check(ctx, lib().ssdt_micro_batch(ctx, mb, keep_last), "ssdt_micro_batch")


def ssdt_set_budget(ctx, budget_bytes):
    _check(ctx, lib().ssdt_set_budget(ctx, budget_bytes), "ssdt_set_budget")


def ssdt_arena_alloc(ctx, nbytes, stream=0) -> int:
    out = C.c_void_p()
    _check(ctx, lib().ssdt_arena_alloc(ctx, nbytes, stream or None, C.byref(out)), "ssdt_arena_alloc")
    return out.value


def ssdt_arena_free(ctx, ptr, stream=0):
    _check(ctx, lib().ssdt_arena_free(ctx, ptr, stream or None), "ssdt_arena_free")


def ssdt_register_weight(ctx, base, nbytes):
    _check(ctx, lib().ssdt_register_weight(ctx, base, nbytes), "ssdt_register_weight")


def ssdt_scope_begin(ctx, scope, phase=FWD):
    _check(ctx, lib().ssdt_scope_begin(ctx, scope, phase), "ssdt_scope_begin")


def ssdt_scope_end(ctx, scope, phase=FWD):
    _check(ctx, lib().ssdt_scope_end(ctx, scope, phase), "ssdt_scope_end")


def ssdt_save(ctx, storage_base, storage_bytes, view_offset, shape: Sequence[int], dtype) -> int:
    shp = (C.c_int64 * len(shape))(*shape)
    out = C.c_uint64()
    _check(ctx, lib().ssdt_save(ctx, storage_base, storage_bytes, view_offset, shp, len(shape), dtype, C.byref(out)),
           "ssdt_save")
    return out.value


def ssdt_offload(ctx, scope, producer=0):
    _check(ctx, lib().ssdt_offload(ctx, scope, producer or None), "ssdt_offload")


def ssdt_prefetch(ctx, scope):
    _check(ctx, lib().ssdt_prefetch(ctx, scope), "ssdt_prefetch")


def ssdt_get(ctx, tid, consumer=0) -> int:
    out = C.c_void_p()
    _check(ctx, lib().ssdt_get(ctx, tid, consumer or None, C.byref(out)), "ssdt_get")
    return out.value


def ssdt_release(ctx, scope, stream=0):
    _check(ctx, lib().ssdt_release(ctx, scope, stream or None), "ssdt_release")


def ssdt_get_stats(ctx) -> dict:
    st = ssdt_stats()
    _check(ctx, lib().ssdt_get_stats(ctx, C.byref(st)), "ssdt_get_stats")
    return st.as_dict()


def ssdt_num_records(ctx) -> int:
    n = C.c_uint32()
    _check(ctx, lib().ssdt_num_records(ctx, C.byref(n)), "ssdt_num_records")
    return n.value


def ssdt_get_record(ctx, index) -> dict:
    r = ssdt_record()
    _check(ctx, lib().ssdt_get_record(ctx, index, C.byref(r)), "ssdt_get_record")
    return {n: getattr(r, n) for n, _ in r._fields_}


def ssdt_pool_read(ctx, pool_offset, nbytes) -> bytes:
    buf = C.create_string_buffer(nbytes)
    _check(ctx, lib().ssdt_pool_read(ctx, pool_offset, buf, nbytes), "ssdt_pool_read")
    return buf.raw


def ssdt_sim_complete(ctx, direction, n) -> int:
    done = C.c_int32()
    _check(ctx, lib().ssdt_sim_complete(ctx, direction, n, C.byref(done)), "ssdt_sim_complete")
    return done.value


def ssdt_sync_io(ctx):
    _check(ctx, lib().ssdt_sync_io(ctx), "ssdt_sync_io")


def ssdt_plan(layer_bytes, fwd_s, bwd_s, store_Bps, load_Bps, safety=1.0, keep_last=1) -> dict:
    n = len(layer_bytes)
    if not (len(fwd_s) == len(bwd_s) == n):
        raise ValueError("ssdt_plan: per-layer arrays differ in length")
    lb = (C.c_uint64 * max(n, 1))(*[int(b) for b in layer_bytes])
    fw = (C.c_double * max(n, 1))(*[float(t) for t in fwd_s])
    bw = (C.c_double * max(n, 1))(*[float(t) for t in bwd_s])
    pin = ssdt_plan_in(n, keep_last, lb, fw, bw, store_Bps, load_Bps, safety)
    out = ssdt_plan_out()
    _check(None, lib().ssdt_plan(C.byref(pin), C.byref(out)), "ssdt_plan")
    return {f: getattr(out, f) for f, _ in ssdt_plan_out._fields_}


def ssdt_spill_stats(ctx):
    w, r = C.c_uint64(0), C.c_uint64(0)
    _check(ctx, lib().ssdt_spill_stats(ctx, C.byref(w), C.byref(r)), "ssdt_spill_stats")
    return w.value, r.value


def ssdt_spill_info(ctx) -> dict:
    out = ssdt_spill_info_t()
    _check(ctx, lib().ssdt_spill_info(ctx, C.byref(out)), "ssdt_spill_info")
    return {n: int(getattr(out, n)) for n, _ in out._fields_}


def ssdt_profile(ctx, enable: bool):
    _check(ctx, lib().ssdt_profile(ctx, int(bool(enable))), "ssdt_profile")


def ssdt_profile_read(ctx) -> list:
    buf = (ssdt_kernel_time * 16)()
    n = C.c_uint32()
    _check(ctx, lib().ssdt_profile_read(ctx, buf, 16, C.byref(n)), "ssdt_profile_read")
    return [dict(name=buf[i].name.decode(), launches=int(buf[i].launches), ms=buf[i].ms, flops=buf[i].flops,
                 bytes=buf[i].bytes) for i in range(n.value)]


def make_desc(arch="gpt_preln", dtype="f32", act="gelu", norm="layernorm", mask="causal", has_bias=True, B=1, S=1,
              S_kv=0, H=1, A=1, F=1, eps=1e-5, softmax_scale=0.0, checkpoint=False, accumulate=False) -> ssdt_layer_desc:
    return ssdt_layer_desc(ARCH[arch], DTYPE[dtype], ACT[act], NORM[norm], MASK[mask], int(bool(has_bias)), B, S, S_kv,
                           H, A, F, eps, softmax_scale, int(bool(checkpoint)), int(bool(accumulate)))


def make_weights(ptrs: dict) -> ssdt_layer_weights:
    w = ssdt_layer_weights()
    for n in WEIGHT_NAMES:
        setattr(w, n, ptrs.get(n) or None)
    return w


def ssdt_sgd_update(ctx, w, g, numel, dtype, lr, stream=0):
    _check(ctx, lib().ssdt_sgd_update(ctx, w, g, numel, dtype, lr, stream or None), "ssdt_sgd_update")


def ssdt_layer_workspace(desc: ssdt_layer_desc):
    f, b = C.c_size_t(), C.c_size_t()
    _check(None, lib().ssdt_layer_workspace(C.byref(desc), C.byref(f), C.byref(b)), "ssdt_layer_workspace")
    return f.value, b.value


def ssdt_layer_bwd_temporaries(desc: ssdt_layer_desc) -> dict:
    out = ssdt_bwd_temporaries()
    _check(None, lib().ssdt_layer_bwd_temporaries(C.byref(desc), C.byref(out)), "ssdt_layer_bwd_temporaries")
    return {n: int(getattr(out, n)) for n, _ in out._fields_}


def ssdt_layer_fwd(ctx, desc, weights, scope, x, enc_out, kv_len, ws, ws_bytes, stream=0):
    """Returns (y device pointer, ssdt_layer_saved)."""
    y = C.c_void_p()
    saved = ssdt_layer_saved()
    _check(ctx, lib().ssdt_layer_fwd(ctx, C.byref(desc), C.byref(weights), scope, x, enc_out or None, kv_len or None,
                                     C.byref(y), C.byref(saved), ws, ws_bytes, stream or None), "ssdt_layer_fwd")
    return y.value, saved


def ssdt_layer_bwd(ctx, desc, weights, saved, kv_len, dy, dx, d_enc_out, grads, ws, ws_bytes, stream=0):
    _check(ctx, lib().ssdt_layer_bwd(ctx, C.byref(desc), C.byref(weights), C.byref(saved), kv_len or None, dy, dx,
                                     d_enc_out or None, C.byref(grads), ws, ws_bytes, stream or None),
           "ssdt_layer_bwd")


STATIC_WS_BYTES = 64 << 20


def ssdt_layer_bwd_static(ctx, desc, weights, saved, kv_len, dy, dx, d_enc_out, grads, stream=0):
    _check(ctx, lib().ssdt_layer_bwd_static(ctx, C.byref(desc), C.byref(weights), C.byref(saved), kv_len or None, dy, dx,
                                            d_enc_out or None, C.byref(grads), stream or None),
           "ssdt_layer_bwd_static")
