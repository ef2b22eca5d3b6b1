"""Shared by the GPU parity tests: builds a seeded case, runs the CPU checker and the GPU
library on the same bytes, and compares tensor by tensor."""
import numpy as np
import torch

from oracle import layer_oracle as lo
from oracle import registry_oracle as ro
from paper_2408_10013_amd import binding as sb
from paper_2408_10013_amd import runner, synth

TOL = {"f32": 1e-4, "bf16": 2e-2}   # max |gpu - ref| / max |ref| per tensor


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if not np.isfinite(ref).all():
        # -inf entries (empty softmax rows) must match exactly; compare the rest
        assert (np.isfinite(ref) == np.isfinite(got)).all()
        m = np.isfinite(ref)
        got, ref = got[m], ref[m]
        if ref.size == 0:
            return 0.0
    assert np.isfinite(got).all()
    denom = np.abs(ref).max()
    return float(np.abs(got - ref).max() / denom) if denom > 0 else float(np.abs(got).max())


def rel_l2(got: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64).ravel()
    got = np.asarray(got, dtype=np.float64).ravel()
    n = np.linalg.norm(ref)
    return float(np.linalg.norm(got - ref) / n) if n > 0 else float(np.linalg.norm(got))


def oracle_desc(l: runner.Layer) -> lo.LayerDesc:
    return lo.LayerDesc(arch=l.arch, B=l.B, S=l.S, S_kv=l.S_kv, H=l.H, A=l.A, F=l.F, act=l.act, norm=l.norm,
                        mask=l.mask, has_bias=l.has_bias, eps=l.eps)


def make_layer_case(l: runner.Layer, seed: int, bias_std=0.05, kv_len_range=None):
    shapes = lo.weight_shapes(oracle_desc(l))
    assert list(shapes) == list(l.shapes)
    return synth.make_case(shapes, l.T, l.H, seed, l.dtype, T_enc=l.B * l.S_kv, bias_std=bias_std, B=l.B,
                           kv_len_range=kv_len_range)


def load_weights(l: runner.Layer, w: dict, dev):
    l.set_weights({k: runner.to_device(v, l.dtype, dev) for k, v in w.items()})


SAVED_SHAPES = {"lse": lambda l: (l.B, l.A, l.S), "lsex": lambda l: (l.B, l.A, l.S)}


def fetch_saved(st: runner.Stack, l: runner.Layer):
    """Reads a layer's saved tensors from the device right after its forward (before they leave)."""
    out = {}
    T, H, F, Te = l.T, l.H, l.F, l.B * l.S_kv
    shp = {"x": (T, H), "a": (T, H), "qkv": (T, 3 * H), "o": (T, H), "r1": (T, H), "x1": (T, H), "ax": (T, H),
           "enc": (Te, H), "qx": (T, H), "kvx": (Te, 2 * H), "ox": (T, H), "x2": (T, H), "m": (T, H), "h1": (T, F),
           "g": (T, F), "r2": (T, H)}
    for i, name in enumerate(sb.SV_NAMES):
        e = l.saved.e[i]
        if not e.bytes:
            continue
        if name in shp:
            out[name] = runner.to_host(st.view(e.ptr, shp[name]))
        elif name.startswith("lse"):
            out[name] = runner.to_host(st.view(e.ptr, (l.B, l.A, l.S), torch.float32))
        else:
            out[name] = runner.to_host(st.view(e.ptr, (T,), torch.float32))
    return out


def registry_expectation(layers, keep_last, min_offload_elems, budget_bytes, pool_bytes, shared_enc=False):
    reg = ro.RegistryOracle(len(layers), min_offload_elems, None if budget_bytes < 0 else budget_bytes, keep_last,
                            pool_bytes)
    for i, l in enumerate(layers):
        e = 4 if l.dtype == "f32" else 2
        tr = ro.saved_trace(l.arch, l.norm, l.act, l.T, l.H, l.F, l.B, l.A, l.S, e, T_enc=l.B * l.S_kv)
        reg.scope_begin(i)
        for name, storage, sbytes, numel in tr:
            if storage == "enc":
                key = "enc"
            else:
                key = (i, storage)
            reg.save(key, sbytes, numel)
        reg.scope_end(i)
    return reg


def compare_registry(stack: runner.Stack, reg):
    st = stack.stats()
    for k, v in vars(reg.c).items():
        assert st[k] == v, (k, st[k], v)
    recs = stack.records()
    cls = {ro.SMALL: sb.CLS_SMALL, ro.KEPT: sb.CLS_KEPT, ro.OFFLOADED: sb.CLS_OFFLOADED}
    assert len(recs) == len(reg.records)
    for g, w in zip(recs, reg.records):
        assert (g["tid"], g["layer"], g["cls"], g["bytes"], g["pack_offset"], g["pool_offset"]) == \
               (w.stamp, w.layer, cls[w.cls], w.bytes, w.pack_offset, w.pool_offset)


def layer_bwd_same_relu_decisions(d, w, sv, dy, kv_len, g_gpu):
    """The checker's backward with ReLU's 0/1 derivative decided on the activation values the GPU stored.

    ReLU's derivative is an integer decision on the sign of a computed value; with bf16 storage a pre-activation
    within rounding distance of zero can come out on either side, and both are valid.  Both sides must then take
    the decision from the same numbers: the GPU's backward decides on its stored activation output g (> 0), so
    the checker is given that g in place of its own pre-activation for this one decision.  Everything else
    (every matrix product, the norms, attention, the other saved tensors) stays the checker's own."""
    if d.act != "relu":
        return lo.layer_bwd(d, w, sv, dy, kv_len)
    sv2 = dict(sv)
    sv2["h1"] = np.asarray(g_gpu, dtype=np.float64)
    return lo.layer_bwd(d, w, sv2, dy, kv_len)
