"""The layer stacks of the benchmark configurations at their full shapes, driven as bench.py drives them.

(1) gpt_2048 x4, bert_1024 x8 (per-sequence key padding) and t5_2048 (2 encoder + 2 decoder layers): the whole stack
    runs with every layer offloaded under arena pressure (layer l's copies out overlap layer l+1's compute; the
    arena holds fewer layers than the stack, so blocks are reclaimed and reloaded) and again with offload off;
    outputs and every gradient must be bit-identical.  Parity with the CPU checker is then taken layer by layer
    inside the offloaded run: the checker gets the GPU's own input and upstream gradient of a layer (the full
    micro-batch, every sequence different, dense gradient) and must reproduce that layer's output, input gradient
    and parameter gradients element by element; that the layers are chained correctly is what the shared buffers
    and the on/off identity show.  For T5 the encoder output must be one record of B*S_enc*H*2 bytes with two
    scopes, stored once, and its gradient the sum of both decoder layers' contributions.
(2) gpt_8192 at micro-batch 16 (the benchmark workload, three layers): offload-all under arena pressure against
    offload off, bit for bit; no checker needed.
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


def device_weights(layers, seed):
    dev = torch.device(DEV)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    out = []
    for l in layers:
        w = {}
        for name, shp in l.shapes.items():
            if name.startswith("w_"):
                w[name] = (torch.randn(shp, generator=gen, device=dev) * 0.02).to(torch.bfloat16)
            elif name.endswith("_g"):
                w[name] = (1.0 + 0.1 * torch.randn(shp, generator=gen, device=dev)).to(torch.bfloat16)
            else:
                w[name] = (0.05 * torch.randn(shp, generator=gen, device=dev)).to(torch.bfloat16)
        out.append(w)
    return gen, out


def run_stack(cfg, weights, x, dy, enc_x, kv, *, offload, arena_layers, capture, spill_path=None, settle=False):
    layers = runner.layers_from_config(cfg)
    for l, w in zip(layers, weights):
        l.set_weights(w)
    per = max(runner.saved_bytes_per_layer(l) for l in layers)
    pool = runner.pool_bytes_needed(layers, keep_last=0) if offload else 0
    st = runner.Stack(layers, int(arena_layers * per) + (64 << 20), pool, DEV, keep_last=0, min_offload_elems=1 << 20,
                      budget_bytes=-1 if offload else 0, spill_path=spill_path)
    st.register_weights()
    if capture:
        st.capture = {}
    yp = st.forward(x, enc_x=enc_x, kv_len=kv)
    y = st.view(yp, tuple(x.shape)).clone()
    recs = st.records()
    if settle:          # let every store (and file write) finish before backward asks for anything back
        torch.cuda.synchronize()
        sb.ssdt_sync_io(st.ctx)
    dx, dxe = st.backward(dy)
    torch.cuda.synchronize()
    sb.ssdt_arena_free(st.ctx, yp, st.stream)
    out = dict(y=y, dx=dx.clone(), dxe=None if dxe is None else dxe.clone(), layers=layers, stats=st.stats(), recs=recs,
               grads=[{k: v.clone() for k, v in l.g.items()} for l in layers], cap=st.capture)
    if spill_path:
        sb.ssdt_sync_io(st.ctx)
        out["spill"] = sb.ssdt_spill_info(st.ctx)
    st.close()
    return out


def assert_identical(a, b):
    assert torch.equal(a["y"], b["y"]) and torch.equal(a["dx"], b["dx"])
    if a["dxe"] is not None:
        assert torch.equal(a["dxe"], b["dxe"])
    for i, (ga, gb) in enumerate(zip(a["grads"], b["grads"])):
        for k in ga:
            assert torch.equal(ga[k], gb[k]), (i, k)


@pytest.mark.parametrize("workload", ["gpt_2048", "bert_1024", "t5_2048"])
def test_full_stack_offloaded_under_pressure_and_checked_layer_by_layer(workload):
    cfg = synth.CONFIGS[workload]
    dev = torch.device(DEV)
    proto = runner.layers_from_config(cfg)
    L = len(proto)
    gen, weights = device_weights(proto, synth.BASE_SEED + 400 + cfg["index"])
    dec0 = next(l for l in proto if l.arch != "t5_enc")
    x = torch.randn(dec0.T, dec0.H, generator=gen, device=dev).to(torch.bfloat16)
    dy = torch.randn(dec0.T, dec0.H, generator=gen, device=dev).to(torch.bfloat16)
    enc_x = torch.randn(proto[0].T, proto[0].H, generator=gen, device=dev).to(torch.bfloat16) if proto[0].arch == "t5_enc" else None
    kv = None
    if cfg.get("kv_len_range"):
        lo_, hi_ = cfg["kv_len_range"]
        kv = torch.from_numpy(np.random.default_rng(synth.BASE_SEED + cfg["index"]).integers(lo_, hi_ + 1, size=cfg["B"]).astype(np.int32)).to(dev)
    # arena: three layers' worth of the 4 / 8 GPT / BERT layers; for T5 (two large encoder layers, two small decoder
    # layers) less than the two encoder layers together, so that the second one has to reclaim the first one's blocks
    on = run_stack(cfg, weights, x, dy, enc_x, kv, offload=True, arena_layers=1.8 if enc_x is not None else 3, capture=True)
    off = run_stack(cfg, weights, x, dy, enc_x, kv, offload=False, arena_layers=L + 1, capture=False)
    assert_identical(on, off)
    s = on["stats"]
    assert s["offloaded"] >= 7 * L and s["kept"] == 0 and s["loads"] > 0 and s["loads"] + s["forwarded"] == s["offloaded"]
    assert s["arena_peak_in_use"] < (1.0 if enc_x is not None else 0.9) * off["stats"]["arena_peak_in_use"]
    assert off["stats"]["offloaded"] == 0
    n_enc = sum(1 for l in proto if l.arch == "t5_enc")
    if n_enc:
        # the encoder output: saved by both decoder layers, one storage, stored once (Sec. 3.3.1)
        enc_bytes = proto[0].T * proto[0].H * 2
        assert enc_bytes == 16777216
        shared = [r for r in on["recs"] if r["bytes"] == enc_bytes and r["n_scopes"] == 2]
        assert len(shared) == 1 and shared[0]["cls"] == sb.CLS_OFFLOADED and shared[0]["layer"] == n_enc

    # ---- layer by layer against the checker, on the GPU's own layer inputs and upstream gradients ------------------
    cap = on["cap"]
    kv_h = kv.cpu().numpy() if kv is not None else None
    enc_out = runner.to_host(cap["y"][n_enc - 1]) if n_enc else None
    worst = {}
    d_enc_sum = 0.0
    for i, l in enumerate(on["layers"]):
        is_enc = i < n_enc
        xin = (enc_x if i == 0 else cap["y"][i - 1]) if is_enc else (x if i == n_enc else cap["y"][i - 1])
        if i == L - 1:
            dyin = dy
        elif i == n_enc - 1:
            dyin = cap["d_enc"]
        else:
            dyin = cap["dx"][i + 1]
        d = hp.oracle_desc(l)
        wh = {k: runner.to_host(v) for k, v in weights[i].items()}
        y_ref, sv = lo.layer_fwd(d, wh, runner.to_host(xin), enc_out if l.arch == "t5_dec" else None, kv_h)
        g_gpu = runner.to_host(cap["g"][i]) if l.act == "relu" else None
        dx_ref, de_ref, gr = hp.layer_bwd_same_relu_decisions(d, wh, sv, runner.to_host(dyin), kv_h, g_gpu)
        errs = {"y": hp.rel_err(runner.to_host(cap["y"][i]), y_ref), "dx": hp.rel_err(runner.to_host(cap["dx"][i]), dx_ref)}
        for k in gr:
            errs["grad." + k] = hp.rel_err(runner.to_host(on["grads"][i][k]), gr[k])
        if de_ref is not None:
            d_enc_sum = d_enc_sum + de_ref
        bad = {k: v for k, v in errs.items() if not v <= hp.TOL["bf16"]}
        assert not bad, (workload, i, l.arch, bad)
        k = max(errs, key=errs.get)
        worst[i] = (k, round(errs[k], 5))
    if n_enc:
        e = hp.rel_err(runner.to_host(cap["d_enc"]), d_enc_sum)     # accumulated over both decoder layers
        assert e <= hp.TOL["bf16"], ("d_enc", e)
        worst["d_enc"] = round(e, 5)
    print(workload, "worst per layer:", worst)


def test_benchmark_shape_offload_on_equals_off_bit_for_bit():
    """Three gpt_8192 layers at micro-batch 16: everything offloaded with an arena of two layers' worth (blocks are
    reclaimed while stores are in flight, tensors are forwarded or reloaded, loads are waited for) against offload
    off.  Outputs, input gradient and all parameter gradients must be the same bits (Sec. 3.2: the cache is
    transparent)."""
    cfg = dict(synth.CONFIGS["gpt_8192"], stack=[("gpt_preln", 3)])
    dev = torch.device(DEV)
    proto = runner.layers_from_config(cfg)
    gen, weights = device_weights(proto, synth.BASE_SEED + 450)
    x = torch.randn(proto[0].T, proto[0].H, generator=gen, device=dev).to(torch.bfloat16)
    dy = torch.randn(proto[0].T, proto[0].H, generator=gen, device=dev).to(torch.bfloat16)
    on = run_stack(cfg, weights, x, dy, None, None, offload=True, arena_layers=2.5, capture=False)
    off = run_stack(cfg, weights, x, dy, None, None, offload=False, arena_layers=4, capture=False)
    assert_identical(on, off)
    s = on["stats"]
    assert s["offloaded"] == 3 * 9 and s["loads"] > 0 and s["loads"] + s["forwarded"] == s["offloaded"]
    assert s["arena_peak_in_use"] < 0.9 * off["stats"]["arena_peak_in_use"]
    assert float(on["dx"].float().abs().max()) > 0 and all(float(g["w_1"].float().abs().max()) > 0 for g in on["grads"])
    print("gpt_8192 x3 B=16 on/off identical; loads %d forwarded %d arena peak %.1f vs %.1f GB" % (
        s["loads"], s["forwarded"], s["arena_peak_in_use"] / 1e9, off["stats"]["arena_peak_in_use"] / 1e9))


def test_file_tier_at_the_benchmark_layer_shape(tmp_path):
    """Three gpt_8192 layers (full width, micro-batch 4: 2.1 GB of saved tensors each) offloaded through the pinned pool
    into a spill file with an arena that cannot keep them: every tensor that is reloaded comes from the file (its pool
    bytes are overwritten once written), in several direct-I/O requests each.  Outputs and gradients must be the same
    bits as with the pool alone."""
    cfg = dict(synth.CONFIGS["gpt_8192"], stack=[("gpt_preln", 3)], B=4)
    dev = torch.device(DEV)
    proto = runner.layers_from_config(cfg)
    gen, weights = device_weights(proto, synth.BASE_SEED + 460)
    x = torch.randn(proto[0].T, proto[0].H, generator=gen, device=dev).to(torch.bfloat16)
    dy = torch.randn(proto[0].T, proto[0].H, generator=gen, device=dev).to(torch.bfloat16)
    # The host enqueues a whole pass ahead of the GPU, and a tensor whose copy out has not been seen finished when it
    # is asked back is served from the pool; so both runs wait for their stores between forward and backward, after
    # which the file run has nothing but the file to load from.
    pool = run_stack(cfg, weights, x, dy, None, None, offload=True, arena_layers=2.5, capture=False, settle=True)
    file = run_stack(cfg, weights, x, dy, None, None, offload=True, arena_layers=2.5, capture=False, settle=True,
                     spill_path=str(tmp_path / "spill.bin"))
    assert_identical(pool, file)
    s, si = file["stats"], file["spill"]
    assert s["loads"] > 0 and s["loads"] + s["forwarded"] == s["offloaded"] == 3 * 8
    assert s["forwarded"] == 0 and si["bytes_read"] == s["bytes_loaded"] == si["bytes_written"] == s["bytes_offloaded"]
    assert si["bytes_read"] >= 1 << 30                      # whole activations came back from the file
    print("file tier: direct I/O %d, %d threads, wrote %.2f GB at %.2f GB/s, read %.2f GB at %.2f GB/s" % (
        si["direct_io"], si["threads"], si["bytes_written"] / 1e9, si["bytes_written"] / max(1, si["write_busy_ns"]),
        si["bytes_read"] / 1e9, si["bytes_read"] / max(1, si["read_busy_ns"])))
