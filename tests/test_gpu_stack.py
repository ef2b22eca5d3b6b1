"""Stacks of layers through the driver: parity of the chained forward/backward against the CPU
checker, bookkeeping against the bookkeeping checker, the shared encoder output stored once, and
bit-identical gradients with offload on / off / under arena pressure."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle as lo
from paper_2408_10013_amd import binding as sb
from paper_2408_10013_amd import runner, synth

import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def build(layers, cases, arena, pool, **kw):
    st = runner.Stack(layers, arena, pool, DEV, **kw)
    for l, c in zip(layers, cases):
        hp.load_weights(l, c["w"], st.dev)
    st.register_weights()
    return st


def oracle_stack(layers, cases, x, dy, enc_x=None, relu_g=None):
    """Chains the checker through the stack; returns y, dx, d(enc input), per-layer gradients.  relu_g: per layer,
    the activation outputs the GPU stored, from which both sides take ReLU's 0/1 derivative."""
    bwd = lambda i, sv, g: hp.layer_bwd_same_relu_decisions(hp.oracle_desc(layers[i]), cases[i]["w"], sv, g, None,
                                                            relu_g[i] if relu_g else np.maximum(sv["h1"], 0.0))
    n_enc = sum(1 for l in layers if l.arch == "t5_enc") if enc_x is not None else 0
    svs, cur = [], enc_x
    for i in range(n_enc):
        cur, sv = lo.layer_fwd(hp.oracle_desc(layers[i]), cases[i]["w"], cur)
        svs.append(sv)
    enc_out = cur if n_enc else None
    cur = x
    for i in range(n_enc, len(layers)):
        cur, sv = lo.layer_fwd(hp.oracle_desc(layers[i]), cases[i]["w"], cur, enc_out)
        svs.append(sv)
    y = cur
    grads = [None] * len(layers)
    g, d_enc = dy, 0
    for i in range(len(layers) - 1, n_enc - 1, -1):
        g, de, grads[i] = bwd(i, svs[i], g)
        if de is not None:
            d_enc = d_enc + de
    dx = g
    g = d_enc
    for i in range(n_enc - 1, -1, -1):
        g, _, grads[i] = bwd(i, svs[i], g)
    return y, dx, (g if n_enc else None), grads


def run_gpu(st, layers, x, dy, enc_x=None, capture=False):
    if capture:
        st.capture = {}
    yp = st.forward(x, enc_x=enc_x)
    y = st.view(yp, tuple(x.shape)).clone()
    stats_fwd, recs = st.stats(), st.records()
    dx, dxe = st.backward(dy)
    torch.cuda.synchronize()
    sb.ssdt_arena_free(st.ctx, yp, st.stream)
    grads = [{k: v.clone() for k, v in l.g.items()} for l in layers]
    return y, dx.clone(), None if dxe is None else dxe.clone(), grads, stats_fwd, recs, st.stats()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_gpt_stack_parity_bookkeeping_and_transparency(dtype):
    mk = lambda: [runner.Layer("gpt_preln", dtype, B=2, S=128, H=128, A=2, F=256, act="gelu", norm="layernorm",
                               mask="causal", has_bias=True, eps=1e-5) for _ in range(4)]
    layers = mk()
    cases = [hp.make_layer_case(l, 300 + i, bias_std=0.05) for i, l in enumerate(layers)]
    x = runner.to_device(cases[0]["x"], dtype, DEV)
    dy = runner.to_device(cases[0]["dy"], dtype, DEV)
    per = runner.saved_bytes_per_layer(layers[0])
    pool = 5 * per
    results = {}
    # roomy arena / offload off / arena that holds fewer layers than the stack (stores must be waited for)
    for name, kw, arena in (("on", dict(keep_last=1, min_offload_elems=0, budget_bytes=-1), 8 * per),
                            ("off", dict(keep_last=1, min_offload_elems=0, budget_bytes=0), 8 * per),
                            ("tight", dict(keep_last=0, min_offload_elems=0, budget_bytes=-1), 3 * per)):
        ls = mk()
        st = build(ls, cases, arena, pool, **kw)
        results[name] = run_gpu(st, ls, x, dy)
        if name == "on":
            reg = hp.registry_expectation(ls, 1, 0, -1, pool)
            for k, v in vars(reg.c).items():
                assert results[name][4][k] == v, (k, results[name][4][k], v)
            got = [(r["tid"], r["layer"], r["cls"], r["bytes"], r["pack_offset"], r["pool_offset"]) for r in results[name][5]]
            cls = {"small": sb.CLS_SMALL, "kept": sb.CLS_KEPT, "offloaded": sb.CLS_OFFLOADED}
            assert got == [(r.stamp, r.layer, cls[r.cls], r.bytes, r.pack_offset, r.pool_offset) for r in reg.records]
        st.close()
    y, dx, _, grads = results["on"][:4]
    y_ref, dx_ref, _, g_ref = oracle_stack(layers, cases, cases[0]["x"], cases[0]["dy"])
    errs = {"y": hp.rel_err(runner.to_host(y), y_ref), "dx": hp.rel_err(runner.to_host(dx), dx_ref)}
    for i, g in enumerate(g_ref):
        for k in g:
            errs["l%d.%s" % (i, k)] = hp.rel_err(runner.to_host(grads[i][k]), g[k])
    bad = {k: v for k, v in errs.items() if not v <= hp.TOL[dtype]}
    assert not bad, sorted(bad.items(), key=lambda kv: -kv[1])[:12]
    for other in ("off", "tight"):
        assert torch.equal(results["on"][0], results[other][0]) and torch.equal(results["on"][1], results[other][1])
        for ga, gb in zip(results["on"][3], results[other][3]):
            for k in ga:
                assert torch.equal(ga[k], gb[k]), (other, k)
    fin = results["tight"][6]
    assert fin["loads"] > 0 and fin["arena_peak_in_use"] <= 3 * per < results["off"][6]["arena_peak_in_use"]
    assert results["off"][6]["offloaded"] == 0 and results["on"][6]["released"] == 4 * 13


def test_spill_file_tier_is_transparent(tmp_path):
    """With a spill file every reloaded tensor comes from the file (its pool bytes are overwritten
    after the write): outputs and gradients must still equal those without one, bit for bit."""
    dtype = "bf16"
    mk = lambda: [runner.Layer("gpt_preln", dtype, B=2, S=128, H=128, A=2, F=256, act="gelu", norm="layernorm",
                               mask="causal", has_bias=True, eps=1e-5) for _ in range(4)]
    cases = [hp.make_layer_case(l, 300 + i, bias_std=0.05) for i, l in enumerate(mk())]
    x = runner.to_device(cases[0]["x"], dtype, DEV)
    dy = runner.to_device(cases[0]["dy"], dtype, DEV)
    per = runner.saved_bytes_per_layer(mk()[0])
    res = {}
    for name, path in (("pool", None), ("file", str(tmp_path / "spill.bin"))):
        ls = mk()
        st = build(ls, cases, 3 * per, 5 * per, keep_last=0, min_offload_elems=0, budget_bytes=-1, spill_path=path)
        res[name] = run_gpu(st, ls, x, dy)
        if path:
            sb.ssdt_sync_io(st.ctx)
            w, r = sb.ssdt_spill_stats(st.ctx)
            fin = res[name][6]
            assert fin["loads"] > 0 and 0 < r <= fin["bytes_loaded"] and w >= r
        st.close()
    assert torch.equal(res["pool"][0], res["file"][0]) and torch.equal(res["pool"][1], res["file"][1])
    for ga, gb in zip(res["pool"][3], res["file"][3]):
        for k in ga:
            assert torch.equal(ga[k], gb[k]), k


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layerwise_recomputation_is_transparent_and_saves_memory(dtype):
    """Recompute arm (Sec. 4.3): only layer inputs survive the forward pass (and are offloaded like any other
    tensor); each layer is re-run inside its backward scope.  Same kernels on the same inputs, so outputs and
    gradients equal the keep-everything run bit for bit, with a far lower activation peak."""
    mk = lambda: [runner.Layer("gpt_preln", dtype, B=2, S=128, H=128, A=2, F=256, act="gelu", norm="layernorm",
                               mask="causal", has_bias=True, eps=1e-5) for _ in range(4)]
    cases = [hp.make_layer_case(l, 300 + i, bias_std=0.05) for i, l in enumerate(mk())]
    x = runner.to_device(cases[0]["x"], dtype, DEV)
    dy = runner.to_device(cases[0]["dy"], dtype, DEV)
    per = runner.saved_bytes_per_layer(mk()[0])
    res = {}
    for name in ("keep", "recompute"):
        ls = mk()
        st = build(ls, cases, 8 * per, 5 * per, keep_last=1, min_offload_elems=0,
                   budget_bytes=0 if name == "keep" else -1)
        st.recompute = name == "recompute"
        res[name] = run_gpu(st, ls, x, dy)
        st.close()
    assert torch.equal(res["keep"][0], res["recompute"][0]) and torch.equal(res["keep"][1], res["recompute"][1])
    for ga, gb in zip(res["keep"][3], res["recompute"][3]):
        for k in ga:
            assert torch.equal(ga[k], gb[k]), k
    fwd, fin = res["recompute"][4], res["recompute"][6]
    xbytes = x.numel() * x.element_size()
    assert (fwd["save_calls"], fwd["unique"], fwd["offloaded"], fwd["kept"]) == (4, 4, 3, 1)
    assert fwd["bytes_offloaded"] == 3 * xbytes
    assert (fin["save_calls"], fin["unique"], fin["dedup_hits"]) == (4 + 4 * 16, 4 * 13, 4 * 4)
    assert fin["offloaded"] == 3 and fin["kept"] + fin["bypass_small"] == 1 + 4 * 12   # recomputed tensors stay put
    assert fin["arena_peak_in_use"] < 0.5 * res["keep"][6]["arena_peak_in_use"]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_t5_encoder_decoder_stack(dtype):
    B, S, Se, H, A, F = 2, 128, 256, 128, 2, 256
    def mk():
        enc = [runner.Layer("t5_enc", dtype, B, Se, H, A, F, "relu", "rmsnorm", "none", False, 1e-6) for _ in range(2)]
        dec = [runner.Layer("t5_dec", dtype, B, S, H, A, F, "relu", "rmsnorm", "causal", False, 1e-6, S_kv=Se) for _ in range(2)]
        return enc + dec
    layers = mk()
    cases = [hp.make_layer_case(l, 400 + i, bias_std=0.05) for i, l in enumerate(layers)]
    for c in cases:
        for k in c["w"]:
            if k.startswith("w_"):
                c["w"][k] = synth.bf16_round(c["w"][k] * 4) if dtype == "bf16" else c["w"][k] * 4
    enc_x_h = cases[0]["x"]
    x_h, dy_h = cases[2]["x"], cases[2]["dy"]
    x, dy, enc_x = (runner.to_device(a, dtype, DEV) for a in (x_h, dy_h, enc_x_h))
    per = max(runner.saved_bytes_per_layer(l) for l in layers)
    res = {}
    for name, budget in (("on", -1), ("off", 0)):
        ls = mk()
        st = build(ls, cases, 8 * per, 6 * per, keep_last=1, min_offload_elems=0, budget_bytes=budget)
        res[name] = run_gpu(st, ls, x, dy, enc_x=enc_x, capture=name == "on")
        if name == "on":
            relu_g = {i: runner.to_host(t) for i, t in st.capture["g"].items()}
        st.close()
    y, dx, dxe, grads, stats_fwd, recs, fin = res["on"]
    # the encoder output: saved by both decoder layers, one storage, stored once, owned by the first decoder layer
    Te = B * Se
    enc_bytes = Te * H * (4 if dtype == "f32" else 2)
    reg = hp.registry_expectation(layers, 1, 0, -1, 6 * per)
    for k, v in vars(reg.c).items():
        assert stats_fwd[k] == v, (k, stats_fwd[k], v)
    shared = [r for r in recs if r["bytes"] == enc_bytes and r["layer"] == 2 and r["n_scopes"] == 2]
    assert len(shared) == 1 and shared[0]["cls"] == sb.CLS_OFFLOADED
    assert fin["released"] == stats_fwd["unique"]
    for ga, gb in zip(res["on"][3], res["off"][3]):
        for k in ga:
            assert torch.equal(ga[k], gb[k]), k
    assert torch.equal(dx, res["off"][1]) and torch.equal(dxe, res["off"][2]) and torch.equal(y, res["off"][0])
    # ReLU's derivative is a 0/1 decision on the sign of a computed value; both sides take it from the activation
    # outputs the GPU stored, so that the chained backward can be compared element by element
    y_ref, dx_ref, dxe_ref, g_ref = oracle_stack(layers, cases, x_h, dy_h, enc_x=enc_x_h, relu_g=relu_g)
    errs = {"y": hp.rel_err(runner.to_host(y), y_ref), "dx": hp.rel_err(runner.to_host(dx), dx_ref),
            "dx_enc": hp.rel_err(runner.to_host(dxe), dxe_ref)}
    for i, g in enumerate(g_ref):
        for k in g:
            errs["l%d.%s" % (i, k)] = hp.rel_err(runner.to_host(grads[i][k]), g[k])
    bad = {k: v for k, v in errs.items() if not v <= hp.TOL[dtype]}
    assert not bad, sorted(bad.items(), key=lambda kv: -kv[1])[:12]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("in_flight", [1, 2])
def test_training_step_with_gradient_accumulation_and_sgd(dtype, in_flight):
    """A step over four micro-batches: gradients accumulate in place, weights take one SGD step at the end.  With
    two micro-batches between forward and backward at once the cache works from per-micro-batch records
    (Sec. 3.1).  Reference: the checker's per-micro-batch gradients summed in double, w - lr * sum."""
    mk = lambda: [runner.Layer("gpt_preln", dtype, B=2, S=128, H=128, A=2, F=256, act="gelu", norm="layernorm",
                               mask="causal", has_bias=True, eps=1e-5) for _ in range(2)]
    layers = mk()
    cases = [hp.make_layer_case(l, 500 + i, bias_std=0.05) for i, l in enumerate(layers)]
    mbs = [hp.make_layer_case(layers[0], 600 + i, bias_std=0.05) for i in range(4)]     # only x, dy are used
    per = runner.saved_bytes_per_layer(layers[0])
    st = build(layers, cases, 6 * per, 8 * per, keep_last=1, min_offload_elems=0, budget_bytes=-1)
    xs = [runner.to_device(m["x"], dtype, DEV) for m in mbs]
    dys = [runner.to_device(m["dy"], dtype, DEV) for m in mbs]
    lr = 0.05
    ys = st.train_step(xs, dys, lr, in_flight=in_flight)
    torch.cuda.synchronize()
    fin = st.stats()
    # reference
    gsum = [None] * len(layers)
    for j, m in enumerate(mbs):
        y_ref, _, _, g_ref = oracle_stack(layers, cases, m["x"], m["dy"])
        assert hp.rel_err(runner.to_host(ys[j]), y_ref) <= hp.TOL[dtype]
        for i, g in enumerate(g_ref):
            gsum[i] = g if gsum[i] is None else {k: gsum[i][k] + g[k] for k in g}
    errs = {}
    for i, l in enumerate(layers):
        for k in gsum[i]:
            errs["l%d.g.%s" % (i, k)] = hp.rel_err(runner.to_host(l.g[k]), gsum[i][k])
            errs["l%d.w.%s" % (i, k)] = hp.rel_err(runner.to_host(l.w[k]), cases[i]["w"][k] - lr * gsum[i][k])
    bad = {k: v for k, v in errs.items() if not v <= hp.TOL[dtype]}
    assert not bad, sorted(bad.items(), key=lambda kv: -kv[1])[:10]
    # bookkeeping: 4 micro-batches x 2 layers x 13 storages, all released; the kept last layer depends on the schedule
    assert fin["unique"] == 4 * 2 * 13 and fin["released"] == 4 * 2 * 13 and fin["arena_in_use"] == 0
    assert fin["kept"] == (4 if in_flight == 1 else 2) * 13
    recs = st.records()
    assert sorted(set(r["micro_batch"] for r in recs)) == [0, 1, 2, 3]
    st.close()
