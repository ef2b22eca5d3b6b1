"""Parity at the benchmark's full layer shapes, in the launch configuration bench.py times.

The CPU checker cannot run a whole micro-batch at these sizes, so the test uses what holds at
any size: sequences do not interact in a layer except through the sums over tokens in the weight
gradients.  The GPU runs the full micro-batch with a random input for every sequence and an
upstream gradient that is non-zero for one sequence only; the checker runs that one sequence
alone.  Then the layer output and input gradient of that sequence must match, the input gradient
of every other sequence must be exactly zero, and every weight gradient must match (the other
sequences contribute exact zeros through the full-size kernels).
"""
import numpy as np
import pytest
import torch

from oracle import layer_oracle as lo
from paper_2408_10013_amd import binding as sb
from paper_2408_10013_amd import runner, synth

import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("workload,seq", [("gpt_2048", 2), ("gpt_8192", 5)])
def test_full_shape_layer_against_one_sequence(workload, seq):
    cfg = synth.CONFIGS[workload]
    l = runner.layers_from_config(cfg, n_layers=1)[0]
    B, S, H = l.B, l.S, l.H
    dev = torch.device(DEV)
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + 100 + cfg["index"])
    w = {}
    for name, shp in l.shapes.items():
        if name.startswith("w_"):
            w[name] = (torch.randn(shp, generator=gen, device=dev) * 0.02).to(torch.bfloat16)
        elif name.endswith("_g"):
            w[name] = (1.0 + 0.1 * torch.randn(shp, generator=gen, device=dev)).to(torch.bfloat16)
        else:
            w[name] = (0.05 * torch.randn(shp, generator=gen, device=dev)).to(torch.bfloat16)
    l.set_weights(w)
    x = torch.randn(l.T, H, generator=gen, device=dev).to(torch.bfloat16)
    dy = torch.zeros(l.T, H, device=dev, dtype=torch.bfloat16)
    rows = slice(seq * S, (seq + 1) * S)
    dy[rows] = torch.randn(S, H, generator=gen, device=dev).to(torch.bfloat16)

    per = runner.saved_bytes_per_layer(l)
    st = runner.Stack([l], 2 * per + (64 << 20), per, DEV, keep_last=0, min_offload_elems=1 << 20)
    st.register_weights()
    yp = st.forward(x)
    y = st.view(yp, (l.T, H)).clone()
    dx, _ = st.backward(dy)
    torch.cuda.synchronize()
    stats = st.stats()
    reg = hp.registry_expectation([l], 0, 1 << 20, -1, per)                      # the big tensors went and came back
    assert stats["offloaded"] == reg.c.offloaded >= 8 and stats["bytes_offloaded"] == reg.c.bytes_offloaded
    assert stats["loads"] + stats["forwarded"] == reg.c.offloaded
    sb.ssdt_arena_free(st.ctx, yp, st.stream)

    # the checker on the one sequence, same bytes
    d = lo.LayerDesc(arch=l.arch, B=1, S=S, H=H, A=l.A, F=l.F, act=l.act, norm=l.norm, mask=l.mask,
                     has_bias=l.has_bias, eps=l.eps)
    wh = {k: runner.to_host(v) for k, v in w.items()}
    y_ref, sv = lo.layer_fwd(d, wh, runner.to_host(x[rows]))
    dx_ref, _, gr = lo.layer_bwd(d, wh, sv, runner.to_host(dy[rows]))
    errs = {"y": hp.rel_err(runner.to_host(y[rows]), y_ref), "dx": hp.rel_err(runner.to_host(dx[rows]), dx_ref)}
    other = torch.ones(l.T, dtype=torch.bool, device=dev)
    other[rows] = False
    assert torch.count_nonzero(dx[other]).item() == 0
    for k in gr:
        errs["grad." + k] = hp.rel_err(runner.to_host(l.g[k]), gr[k])
    st.close()
    print(workload, {k: round(v, 5) for k, v in errs.items()})
    bad = {k: v for k, v in errs.items() if not v <= hp.TOL["bf16"]}
    assert not bad, bad


@pytest.mark.parametrize("workload,which,seq", [("bert_1024", 0, 3), ("t5_2048", 0, 1), ("t5_2048", 2, 6)])
def test_full_shape_other_variants(workload, which, seq):
    """Same scheme for the post-norm encoder with key padding (BERT) and for the T5 encoder / decoder layers, element
    by element.  T5 uses ReLU, whose derivative is a 0/1 decision on the sign of a computed value: both sides take it
    from the activation values the GPU stored (helpers.layer_bwd_same_relu_decisions)."""
    cfg = synth.CONFIGS[workload]
    l = runner.layers_from_config(cfg)[which]
    B, S, H = l.B, l.S, l.H
    dev = torch.device(DEV)
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + 200 + cfg["index"] + which)
    w = {}
    for name, shp in l.shapes.items():
        if name.startswith("w_"):
            w[name] = (torch.randn(shp, generator=gen, device=dev) * 0.02).to(torch.bfloat16)
        elif name.endswith("_g"):
            w[name] = (1.0 + 0.1 * torch.randn(shp, generator=gen, device=dev)).to(torch.bfloat16)
        else:
            w[name] = (0.05 * torch.randn(shp, generator=gen, device=dev)).to(torch.bfloat16)
    l.set_weights(w)
    x = torch.randn(l.T, H, generator=gen, device=dev).to(torch.bfloat16)
    dy = torch.zeros(l.T, H, device=dev, dtype=torch.bfloat16)
    rows = slice(seq * S, (seq + 1) * S)
    dy[rows] = torch.randn(S, H, generator=gen, device=dev).to(torch.bfloat16)
    kv = None
    if l.mask == "keypad":
        lo_, hi_ = cfg["kv_len_range"]
        kv = torch.from_numpy(np.random.default_rng(7).integers(lo_, hi_ + 1, size=B).astype(np.int32)).to(dev)
    Se = l.S_kv
    enc = torch.randn(B * Se, H, generator=gen, device=dev).to(torch.bfloat16) if l.arch == "t5_dec" else None

    per = runner.saved_bytes_per_layer(l)
    st = runner.Stack([l], 3 * per + (64 << 20), 2 * per, DEV, keep_last=0, min_offload_elems=1 << 20)
    st.register_weights()
    sb.ssdt_step_begin(st.ctx, 1)
    st.kv_len, st.n_enc = kv, 0
    xp, xv = st.arena_tensor((l.T, H)); xv.copy_(x)
    ep = 0
    if enc is not None:
        ep, ev = st.arena_tensor((B * Se, H)); ev.copy_(enc)
    yp, l.saved = sb.ssdt_layer_fwd(st.ctx, l.desc, l.wstruct, 0, xp, ep, kv.data_ptr() if kv is not None else 0,
                                    st.ws_ptr, st.ws_bytes, st.stream)
    ge = l.saved.e[sb.SV_NAMES.index("g")]
    g_gpu = runner.to_host(st.view(ge.ptr, (l.T, l.F))[seq * S:(seq + 1) * S]) if l.act == "relu" else None
    sb.ssdt_offload(st.ctx, 0, st.stream)
    sb.ssdt_arena_free(st.ctx, xp, st.stream)
    if ep:
        sb.ssdt_arena_free(st.ctx, ep, st.stream)
    y = st.view(yp, (l.T, H)).clone()
    sb.ssdt_arena_free(st.ctx, yp, st.stream)
    d_enc = torch.zeros(B * Se, H, dtype=torch.bfloat16, device=dev) if enc is not None else None
    dx = torch.empty_like(dy)
    sb.ssdt_prefetch(st.ctx, 0)
    sb.ssdt_layer_bwd(st.ctx, l.desc, l.wstruct, l.saved, kv.data_ptr() if kv is not None else 0, dy.data_ptr(),
                      dx.data_ptr(), d_enc.data_ptr() if d_enc is not None else 0, l.gstruct, st.ws_ptr, st.ws_bytes,
                      st.stream)
    sb.ssdt_release(st.ctx, 0, st.stream)
    torch.cuda.synchronize()
    assert st.stats()["offloaded"] >= 7

    d = lo.LayerDesc(arch=l.arch, B=1, S=S, S_kv=Se, H=H, A=l.A, F=l.F, act=l.act, norm=l.norm, mask=l.mask,
                     has_bias=l.has_bias, eps=l.eps)
    wh = {k: runner.to_host(v) for k, v in w.items()}
    kv1 = kv[seq:seq + 1].cpu().numpy() if kv is not None else None
    enc1 = runner.to_host(enc[seq * Se:(seq + 1) * Se]) if enc is not None else None
    y_ref, sv = lo.layer_fwd(d, wh, runner.to_host(x[rows]), enc1, kv1)
    dx_ref, denc_ref, gr = hp.layer_bwd_same_relu_decisions(d, wh, sv, runner.to_host(dy[rows]), kv1, g_gpu)
    assert hp.rel_err(runner.to_host(y[rows]), y_ref) <= hp.TOL["bf16"]
    other = torch.ones(l.T, dtype=torch.bool, device=dev); other[rows] = False
    assert torch.count_nonzero(dx[other]).item() == 0
    f, bar = hp.rel_err, hp.TOL["bf16"]
    errs = {"dx": f(runner.to_host(dx[rows]), dx_ref)}
    if denc_ref is not None:
        errs["d_enc"] = f(runner.to_host(d_enc[seq * Se:(seq + 1) * Se]), denc_ref)
        oth = torch.ones(B * Se, dtype=torch.bool, device=dev); oth[seq * Se:(seq + 1) * Se] = False
        assert torch.count_nonzero(d_enc[oth]).item() == 0
    for k in gr:
        errs["grad." + k] = f(runner.to_host(l.g[k]), gr[k])
    st.close()
    print(workload, l.arch, {k: round(v, 5) for k, v in errs.items()})
    bad = {k: v for k, v in errs.items() if not v <= bar}
    assert not bad, bad
