"""A thin driver of the C ABI for a stack of layers: the role the training framework's
scheduler plays in the paper (Sec. 3.1): it calls the layers in order, starts each layer's
offload when its forward has been enqueued, prefetches the previous layer before each
layer's backward and releases a layer when its backward has been enqueued.

All arithmetic happens in libssdt.so.  PyTorch provides device memory (weights, the
activation arena, workspaces) and the stream.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as sb
from . import synth


def weight_shapes(arch: str, norm: str, has_bias: bool, H: int, F: int) -> Dict[str, tuple]:
    """Name -> shape of every parameter a layer variant has, in ssdt_layer_weights order."""
    out: Dict[str, tuple] = {}

    def nrm(p):
        out[p + "_g"] = (H,)
        if norm == "layernorm":
            out[p + "_b"] = (H,)

    def lin(wn, bn, i, o):
        out[wn] = (i, o)
        if has_bias:
            out[bn] = (o,)

    nrm("ln1"); lin("w_qkv", "b_qkv", H, 3 * H); lin("w_o", "b_o", H, H)
    if arch == "t5_dec":
        nrm("lnx"); lin("w_qx", "b_qx", H, H); lin("w_kvx", "b_kvx", H, 2 * H); lin("w_ox", "b_ox", H, H)
    nrm("ln2"); lin("w_1", "b_1", H, F); lin("w_2", "b_2", F, H)
    return out


def _tdtype(dtype: str):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def to_device(a: np.ndarray, dtype: str, device) -> torch.Tensor:
    """Host fp32 array (already bf16-representable when dtype is bf16) -> device tensor, exact."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(device=device, dtype=_tdtype(dtype))


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


class Layer:
    def __init__(self, arch, dtype, B, S, H, A, F, act, norm, mask, has_bias, eps, S_kv=0):
        self.arch, self.dtype, self.B, self.S, self.H, self.A, self.F, self.S_kv = arch, dtype, B, S, H, A, F, S_kv
        self.act, self.norm, self.mask, self.has_bias, self.eps = act, norm, mask, has_bias, eps
        self.desc = sb.make_desc(arch=arch, dtype=dtype, act=act, norm=norm, mask=mask, has_bias=has_bias, B=B, S=S,
                                 S_kv=S_kv, H=H, A=A, F=F, eps=eps)
        self.desc_acc = sb.make_desc(arch=arch, dtype=dtype, act=act, norm=norm, mask=mask, has_bias=has_bias, B=B, S=S,
                                     S_kv=S_kv, H=H, A=A, F=F, eps=eps, accumulate=True)
        self.desc_ckpt = sb.make_desc(arch=arch, dtype=dtype, act=act, norm=norm, mask=mask, has_bias=has_bias, B=B,
                                      S=S, S_kv=S_kv, H=H, A=A, F=F, eps=eps, checkpoint=True)
        self.shapes = weight_shapes(arch, norm, has_bias, H, F)
        self.w: Dict[str, torch.Tensor] = {}
        self.g: Dict[str, torch.Tensor] = {}
        self.saved = None

    @property
    def T(self):
        return self.B * self.S

    def set_weights(self, w: Dict[str, torch.Tensor]):
        self.w = w
        self.g = {k: torch.empty_like(v) for k, v in w.items()}
        self.wstruct = sb.make_weights({k: v.data_ptr() for k, v in self.w.items()})
        self.gstruct = sb.make_weights({k: v.data_ptr() for k, v in self.g.items()})


class Stack:
    """A stack of layers on one GPU with its tensor-cache context."""

    def __init__(self, layers: List[Layer], arena_bytes: int, pool_bytes: int, device="cuda:0", keep_last=1,
                 min_offload_elems=1 << 20, budget_bytes=-1, measure_waits=0, spill_path=None, spill_threads=0):
        self.layers = layers
        self.dev = torch.device(device)
        self.dtype = layers[0].dtype
        self.esize = 4 if self.dtype == "f32" else 2
        self.arena = torch.empty(arena_bytes, dtype=torch.uint8, device=self.dev)
        base = self.arena.data_ptr()
        self.arena_base = (base + 255) // 256 * 256
        self.ctx = sb.ssdt_ctx_create(backend=sb.BACKEND_HIP, keep_last=keep_last, min_offload_elems=min_offload_elems,
                                      budget_bytes=budget_bytes, arena_base=self.arena_base,
                                      arena_bytes=arena_bytes - (self.arena_base - base), pool_bytes=pool_bytes,
                                      measure_waits=measure_waits, spill_path=spill_path,
                                      spill_threads=spill_threads)
        fb = bb = 0
        for l in layers:
            f, b = sb.ssdt_layer_workspace(l.desc)
            fb, bb = max(fb, f), max(bb, b)
        self.ws_bytes = max(fb, bb)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=self.dev)
        self.ws_ptr = (self.ws.data_ptr() + 255) // 256 * 256
        self.stream = torch.cuda.current_stream(self.dev).cuda_stream
        self.prefetch_distance = 1
        # layerwise full recomputation (the comparison arm of Sec. 4.3): forward registers only each layer's
        # input, backward re-runs the layer's forward inside its backward scope
        self.recompute = False
        self.mb_saved: Dict[int, list] = {}
        # set to a dict to keep copies of every layer's output ("y"), activation output ("g") and input gradient
        # ("dx") of the next forward / backward pass, and the accumulated encoder-output gradient ("d_enc")
        self.capture: Optional[dict] = None

    def close(self):
        if self.ctx:
            torch.cuda.synchronize(self.dev)
            sb.ssdt_ctx_destroy(self.ctx)
            self.ctx = None

    def register_weights(self):
        for l in self.layers:
            for t in l.w.values():
                sb.ssdt_register_weight(self.ctx, t.data_ptr(), t.numel() * t.element_size())

    # -- arena views -------------------------------------------------------------------------
    def view(self, ptr: int, shape, dtype=None) -> torch.Tensor:
        dtype = dtype or _tdtype(self.dtype)
        n = int(np.prod(shape)) * torch.empty(0, dtype=dtype).element_size()
        off = ptr - self.arena.data_ptr()
        assert 0 <= off and off + n <= self.arena.numel()
        return self.arena[off:off + n].view(dtype).reshape(shape)

    def arena_tensor(self, shape, dtype=None):
        dtype = dtype or _tdtype(self.dtype)
        n = int(np.prod(shape)) * torch.empty(0, dtype=dtype).element_size()
        p = sb.ssdt_arena_alloc(self.ctx, n, self.stream)
        return p, self.view(p, shape, dtype)

    # -- one pass ----------------------------------------------------------------------------
    def forward(self, x: torch.Tensor, enc_x: Optional[torch.Tensor] = None, kv_len: Optional[torch.Tensor] = None,
                offload=True, micro_batch: Optional[int] = None, keep_last: int = -1):
        """x: input of the first layer of the (decoder) stack; enc_x: input of the encoder stack for
        an encoder-decoder.  Returns the device pointer of the output (owned by the caller)."""
        ctx, L = self.ctx, len(self.layers)
        if micro_batch is None:
            sb.ssdt_step_begin(ctx, L)
        else:   # the caller has begun the step; this pass belongs to one of its micro-batches
            sb.ssdt_micro_batch(ctx, micro_batch, keep_last)
        self.kv_len = kv_len
        kvp = kv_len.data_ptr() if kv_len is not None else 0
        n_enc = sum(1 for l in self.layers if l.arch == "t5_enc") if enc_x is not None else 0
        self.n_enc = n_enc
        enc_ptr = 0

        def run(lo, hi, inp, enc):
            p, v = self.arena_tensor(tuple(inp.shape))
            v.copy_(inp)
            for i in range(lo, hi):
                l = self.layers[i]
                y, l.saved = sb.ssdt_layer_fwd(ctx, l.desc_ckpt if self.recompute else l.desc, l.wstruct, i, p, enc, kvp,
                                               self.ws_ptr, self.ws_bytes, self.stream)
                if self.capture is not None:
                    self.capture.setdefault("y", {})[i] = self.view(y, (l.T, l.H)).clone()
                    ge = l.saved.e[sb.SV_NAMES.index("g")]
                    if l.act == "relu" and ge.ptr and ge.bytes:
                        self.capture.setdefault("g", {})[i] = self.view(ge.ptr, (l.T, l.F)).clone()
                if offload:
                    sb.ssdt_offload(ctx, i, self.stream)
                sb.ssdt_arena_free(ctx, p, self.stream)   # drop the caller's reference on the layer input
                p = y
            return p

        if n_enc:
            enc_ptr = run(0, n_enc, enc_x, 0)
        y = run(n_enc, L, x, enc_ptr)
        if enc_ptr:
            sb.ssdt_arena_free(ctx, enc_ptr, self.stream)
        if micro_batch is not None:
            self.mb_saved[micro_batch] = [l.saved for l in self.layers]
        return y

    def backward(self, dy: torch.Tensor, dx_out: Optional[torch.Tensor] = None, micro_batch: Optional[int] = None,
                 accumulate: bool = False):
        """Runs backward through the stack; gradients land in each layer's .g; returns dx of the
        first (decoder) layer and, for an encoder-decoder, dx of the encoder input."""
        ctx, L = self.ctx, len(self.layers)
        if micro_batch is not None:
            sb.ssdt_micro_batch(ctx, micro_batch)
            for l, sv in zip(self.layers, self.mb_saved.pop(micro_batch)):
                l.saved = sv
        kvp = self.kv_len.data_ptr() if self.kv_len is not None else 0
        n_enc = self.n_enc
        bufs = [torch.empty_like(dy), torch.empty_like(dy)]
        d_enc = None
        if n_enc:
            le = self.layers[0]
            d_enc = torch.zeros(le.T, le.H, dtype=dy.dtype, device=self.dev)
        for k in range(self.prefetch_distance):
            if L - 1 - k >= 0:
                sb.ssdt_prefetch(ctx, L - 1 - k)

        def run(hi, lo, grad, denc_ptr):
            cur, flip = grad, 0
            for i in range(hi - 1, lo - 1, -1):
                l = self.layers[i]
                nxt = i - self.prefetch_distance
                if nxt >= 0:
                    sb.ssdt_prefetch(ctx, nxt)
                out = bufs[flip] if cur.shape == bufs[flip].shape else torch.empty_like(cur)
                if out.data_ptr() == cur.data_ptr():
                    out = torch.empty_like(cur)
                if self.recompute:
                    # saves made while a backward scope is open are kept on the device (Sec. 3.2)
                    sb.ssdt_scope_begin(ctx, i, sb.BWD)
                    ins = []
                    for name in ("x", "enc"):
                        ent = l.saved.e[sb.SV_NAMES.index(name)]
                        ins.append(sb.ssdt_get(ctx, ent.tid, self.stream) if ent.tid else (ent.ptr or 0))
                    y2, l.saved = sb.ssdt_layer_fwd(ctx, l.desc, l.wstruct, i, ins[0], ins[1], kvp, self.ws_ptr,
                                                    self.ws_bytes, self.stream)
                    sb.ssdt_arena_free(ctx, y2, self.stream)
                sb.ssdt_layer_bwd(ctx, l.desc_acc if accumulate else l.desc, l.wstruct, l.saved, kvp, cur.data_ptr(),
                                  out.data_ptr(), denc_ptr, l.gstruct, self.ws_ptr, self.ws_bytes, self.stream)
                if self.recompute:
                    sb.ssdt_scope_end(ctx, i, sb.BWD)
                sb.ssdt_release(ctx, i, self.stream)
                if self.capture is not None:
                    self.capture.setdefault("dx", {})[i] = out.clone()
                cur, flip = out, flip ^ 1
            return cur

        dx = run(L, n_enc, dy, d_enc.data_ptr() if d_enc is not None else 0)
        if self.capture is not None and d_enc is not None:
            self.capture["d_enc"] = d_enc
        if n_enc:
            dx_enc = run(n_enc, 0, d_enc, 0)
            return dx, dx_enc
        return dx, None

    def train_step(self, xs: List[torch.Tensor], dys: List[torch.Tensor], lr: float, in_flight: int = 1):
        """One training step with gradient accumulation over the micro-batches xs[i] (dys[i] stands for the loss
        gradient) followed by a plain SGD update of every parameter (Sec. 1, Sec. 4.1).  in_flight = 1 runs forward
        and backward of each micro-batch back to back; in_flight = 2 runs two forwards before their backwards
        (newest first), which needs the cache's per-micro-batch records (Sec. 3.1).  Returns the outputs' pointers'
        contents as tensors (cloned) for checking."""
        ctx, L = self.ctx, len(self.layers)
        sb.ssdt_step_begin(ctx, L)
        ys, first = [], True
        for g0 in range(0, len(xs), in_flight):
            group = list(range(g0, min(g0 + in_flight, len(xs))))
            outs = {}
            for mb in group:
                # only the micro-batch whose backward follows at once keeps its last layer on the device
                outs[mb] = self.forward(xs[mb], micro_batch=mb, keep_last=-1 if mb == group[-1] else 0)
            for mb in reversed(group):
                ys.append((mb, self.view(outs[mb], tuple(xs[mb].shape)).clone()))
                self.backward(dys[mb], micro_batch=mb, accumulate=not first)
                sb.ssdt_arena_free(ctx, outs[mb], self.stream)
                first = False
        dt = sb.F32 if self.dtype == "f32" else sb.BF16
        for l in self.layers:
            for k, w in l.w.items():
                sb.ssdt_sgd_update(ctx, w.data_ptr(), l.g[k].data_ptr(), w.numel(), dt, lr, self.stream)
        return [y for _, y in sorted(ys, key=lambda t: t[0])]

    def stats(self):
        return sb.ssdt_get_stats(self.ctx)

    def records(self):
        return [sb.ssdt_get_record(self.ctx, i) for i in range(sb.ssdt_num_records(self.ctx))]


def layers_from_config(cfg: dict, B: Optional[int] = None, S: Optional[int] = None, n_layers: Optional[int] = None):
    """Expands an entry of synth.CONFIGS into Layer objects (optionally with fewer tokens/layers)."""
    out = []
    B = B or cfg["B"]
    for arch, count in cfg["stack"]:
        cnt = n_layers if (n_layers is not None and len(cfg["stack"]) == 1) else count
        for _ in range(cnt):
            if arch == "t5_enc":
                out.append(Layer(arch, cfg["dtype"], B, cfg["S_enc"], cfg["H"], cfg["A"], cfg["F"], cfg["act"],
                                 cfg["norm"], "none", cfg["has_bias"], cfg["eps"]))
            elif arch == "t5_dec":
                out.append(Layer(arch, cfg["dtype"], B, S or cfg["S"], cfg["H"], cfg["A"], cfg["F"], cfg["act"],
                                 cfg["norm"], "causal", cfg["has_bias"], cfg["eps"], S_kv=cfg["S_enc"]))
            else:
                out.append(Layer(arch, cfg["dtype"], B, S or cfg["S"], cfg["H"], cfg["A"], cfg["F"], cfg["act"],
                                 cfg["norm"], cfg["mask"], cfg["has_bias"], cfg["eps"]))
    return out


def saved_bytes_per_layer(l: Layer) -> int:
    """Upper bound of the arena bytes one layer's saved tensors and output take (for sizing)."""
    e = 4 if l.dtype == "f32" else 2
    T, H, F = l.T, l.H, l.F
    n = (10 * T * H + 2 * T * F) * e + 8 * T * 4 + 2 * l.B * l.A * l.S * 4
    if l.arch == "t5_dec":
        n += (4 * T * H + 3 * l.B * l.S_kv * H) * e
    return n + 64 * 256


def pool_bytes_needed(layers: List[Layer], keep_last: int = 1, min_offload_elems: int = 1 << 20) -> int:
    """Pinned-pool bytes that offloading every eligible tensor of every layer but the last
    `keep_last` takes (tensor sizes rounded to 256 bytes, one 4 KiB-rounded pack per layer)."""
    tot = 0
    for l in layers[:len(layers) - keep_last]:
        e = 4 if l.dtype == "f32" else 2
        T, H, F = l.T, l.H, l.F
        sizes = [(T * H, e)] * (5 if l.arch != "t5_dec" else 9) + [(T * 3 * H, e)] + [(T * F, e)] * 2
        sizes += [(l.B * l.A * l.S, 4)] * (2 if l.arch == "t5_dec" else 1) + [(T, 4)] * 6
        if l.arch == "t5_dec":
            sizes += [(l.B * l.S_kv * H, e), (l.B * l.S_kv * 2 * H, e)]
        pack = sum((n * b + 255) // 256 * 256 for n, b in sizes if n >= min_offload_elems)
        tot += (pack + 4095) // 4096 * 4096
    return tot + (1 << 20)
