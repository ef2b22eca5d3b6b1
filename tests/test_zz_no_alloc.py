"""ssdt_layer_bwd_static (the backward entry point that brings its own workspace and allocates nothing) against
ssdt_layer_bwd: two calls in a row through the C ABI, the second on a smaller layer, results bit-identical to the
ordinary entry point's and within the bf16 / fp32 bars of the CPU checker; a layer that needs more workspace than
the built-in one is refused."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle as lo
from paper_2408_10013_amd import binding as sb
from paper_2408_10013_amd import runner, synth

import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

FIRST = dict(arch="gpt_preln", B=2, S=256, H=256, A=2, F=1024, act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5)
SECOND = dict(arch="bert_postln", B=3, S=128, H=128, A=2, F=256, act="gelu", norm="layernorm", mask="keypad", has_bias=True, eps=1e-5)


def forward_both(variants, dtype, seed):
    """One context, one step, the given layers as its scopes 0, 1, ... (each with an input of its own); everything
    stays on the device."""
    layers = [runner.Layer(dtype=dtype, **v) for v in variants]
    per = sum(runner.saved_bytes_per_layer(l) for l in layers)
    st = runner.Stack(layers, 3 * per + (1 << 20), 0, DEV, keep_last=1, min_offload_elems=0, budget_bytes=0)
    sb.ssdt_step_begin(st.ctx, len(layers))
    out = []
    for i, (l, v) in enumerate(zip(layers, variants)):
        kvr = (1, v["S"]) if v["mask"] == "keypad" else None
        case = hp.make_layer_case(l, seed + i, bias_std=0.05, kv_len_range=kvr)
        hp.load_weights(l, case["w"], st.dev)
        xp, xv = st.arena_tensor((l.T, l.H))
        xv.copy_(runner.to_device(case["x"], dtype, st.dev))
        kv = torch.from_numpy(case["kv_len"]).to(st.dev) if "kv_len" in case else None
        yp, l.saved = sb.ssdt_layer_fwd(st.ctx, l.desc, l.wstruct, i, xp, 0, kv.data_ptr() if kv is not None else 0,
                                        st.ws_ptr, st.ws_bytes, st.stream)
        out.append(dict(l=l, st=st, case=case, kv=kv, dy=runner.to_device(case["dy"], dtype, st.dev), yp=yp, scope=i))
    return st, out


def finish(st, cs):
    for c in cs:
        sb.ssdt_release(st.ctx, c["scope"], st.stream)
        sb.ssdt_arena_free(st.ctx, c["yp"], st.stream)
    st.close()


def backward(c, static):
    l, st, kv, dy = c["l"], c["st"], c["kv"], c["dy"]
    g = {k: torch.full_like(v, float("nan")) for k, v in l.w.items()}
    gs = sb.make_weights({k: v.data_ptr() for k, v in g.items()})
    dx = torch.full_like(dy, float("nan"))
    kvp = kv.data_ptr() if kv is not None else 0
    if static:
        sb.ssdt_layer_bwd_static(st.ctx, l.desc, l.wstruct, l.saved, kvp, dy.data_ptr(), dx.data_ptr(), 0, gs, st.stream)
    else:
        sb.ssdt_layer_bwd(st.ctx, l.desc, l.wstruct, l.saved, kvp, dy.data_ptr(), dx.data_ptr(), 0, gs, st.ws_ptr,
                          st.ws_bytes, st.stream)
    return dx, g


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_workspace_backward_equals_ordinary_backward(dtype):
    st, (a, b) = forward_both([FIRST, SECOND], dtype, 7001)
    for c in (a, b):
        need = sb.ssdt_layer_workspace(c["l"].desc)[1]
        assert 0 < need <= sb.STATIC_WS_BYTES
    ref = [backward(a, False), backward(b, False)]
    torch.cuda.synchronize()
    # two calls in a row on one stream, the second one smaller: it runs over what the first one left behind
    got = [backward(a, True), backward(b, True)]
    torch.cuda.synchronize()
    for (dx_r, g_r), (dx_g, g_g), c in zip(ref, got, (a, b)):
        assert torch.isfinite(dx_g.float()).all()
        assert torch.equal(dx_r, dx_g)
        for k in g_r:
            assert torch.equal(g_r[k], g_g[k]), k
        # and against the CPU checker
        l, case = c["l"], c["case"]
        d = hp.oracle_desc(l)
        kvh = case.get("kv_len")
        _, sv = lo.layer_fwd(d, case["w"], case["x"], None, kvh)
        dx_ref, _, gr = lo.layer_bwd(d, case["w"], sv, case["dy"], kvh)
        errs = {"dx": hp.rel_err(runner.to_host(dx_g), dx_ref)}
        for k in gr:
            errs[k] = hp.rel_err(runner.to_host(g_g[k]), gr[k])
        bad = {k: v for k, v in errs.items() if not v <= hp.TOL[dtype]}
        assert not bad, bad
    finish(st, (a, b))


def test_static_workspace_refuses_a_layer_that_does_not_fit():
    st, (c,) = forward_both([SECOND], "bf16", 7003)
    big = runner.layers_from_config(synth.CONFIGS["gpt_2048"], n_layers=1)[0]
    assert sb.ssdt_layer_workspace(big.desc)[1] > sb.STATIC_WS_BYTES
    z = sb.make_weights({})
    with pytest.raises(sb.SsdtError) as ei:
        sb.ssdt_layer_bwd_static(st.ctx, big.desc, z, c["l"].saved, 0, c["dy"].data_ptr(), c["dy"].data_ptr(), 0, z, st.stream)
    assert ei.value.status == sb.E_NOMEM and "workspace" in str(ei.value)
    finish(st, (c,))
