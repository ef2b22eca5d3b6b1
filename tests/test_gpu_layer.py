"""GPU parity of ssdt_layer_fwd / ssdt_layer_bwd against the CPU checker, element by element,
through the C ABI; offload transparency; bookkeeping."""
import numpy as np
import pytest
import torch

from oracle import layer_oracle as lo
from paper_2408_10013_amd import binding as sb
from paper_2408_10013_amd import runner, synth

import helpers as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_single_layer(l, case, offload, keep_last=0, min_elems=0, fetch=True):
    arena = 3 * runner.saved_bytes_per_layer(l) + (1 << 20)
    st = runner.Stack([l], arena, 2 * runner.saved_bytes_per_layer(l), DEV, keep_last=keep_last,
                      min_offload_elems=min_elems, budget_bytes=-1 if offload else 0)
    hp.load_weights(l, case["w"], st.dev)
    st.register_weights()
    x = runner.to_device(case["x"], l.dtype, st.dev)
    dy = runner.to_device(case["dy"], l.dtype, st.dev)
    kv = torch.from_numpy(case["kv_len"]).to(st.dev) if "kv_len" in case else None
    enc_ptr = 0
    res = {}
    if l.arch == "t5_dec":
        # drive the C ABI directly: the encoder output is an arena block held by the caller
        sb.ssdt_step_begin(st.ctx, 1)
        enc_ptr, ev = st.arena_tensor((l.B * l.S_kv, l.H)); ev.copy_(runner.to_device(case["enc"], l.dtype, st.dev))
        xp, xv = st.arena_tensor((l.T, l.H)); xv.copy_(x)
        y, l.saved = sb.ssdt_layer_fwd(st.ctx, l.desc, l.wstruct, 0, xp, enc_ptr, 0, st.ws_ptr, st.ws_bytes, st.stream)
        st.kv_len, st.n_enc = None, 0
    else:
        sb.ssdt_step_begin(st.ctx, 1)
        xp, xv = st.arena_tensor((l.T, l.H)); xv.copy_(x)
        y, l.saved = sb.ssdt_layer_fwd(st.ctx, l.desc, l.wstruct, 0, xp, 0, kv.data_ptr() if kv is not None else 0,
                                       st.ws_ptr, st.ws_bytes, st.stream)
        st.kv_len, st.n_enc = kv, 0
    torch.cuda.synchronize()
    if fetch:
        res["saved"] = hp.fetch_saved(st, l)
    res["y"] = runner.to_host(st.view(y, (l.T, l.H)))
    res["records_fwd"] = st.records()
    if offload:
        sb.ssdt_offload(st.ctx, 0, st.stream)
    sb.ssdt_arena_free(st.ctx, xp, st.stream)
    if enc_ptr:
        sb.ssdt_arena_free(st.ctx, enc_ptr, st.stream)
    sb.ssdt_arena_free(st.ctx, y, st.stream)
    if offload:
        sb.ssdt_sync_io(st.ctx)          # stores complete: device copies are dropped
        res["records_stored"] = st.records()
        res["pool"] = {r["tid"]: sb.ssdt_pool_read(st.ctx, r["pool_offset"], r["bytes"])
                       for r in res["records_stored"] if r["cls"] == sb.CLS_OFFLOADED}
        # poison the arena so that a backward reading a stale address fails parity loudly
        st.arena.fill_(0xFF)
        torch.cuda.synchronize()
    d_enc = torch.zeros(l.B * l.S_kv, l.H, dtype=dy.dtype, device=st.dev) if l.arch == "t5_dec" else None
    dx = torch.empty_like(dy)
    sb.ssdt_prefetch(st.ctx, 0)
    sb.ssdt_layer_bwd(st.ctx, l.desc, l.wstruct, l.saved, kv.data_ptr() if kv is not None else 0, dy.data_ptr(),
                      dx.data_ptr(), d_enc.data_ptr() if d_enc is not None else 0, l.gstruct, st.ws_ptr, st.ws_bytes,
                      st.stream)
    sb.ssdt_release(st.ctx, 0, st.stream)
    torch.cuda.synchronize()
    res["dx"] = dx.clone()
    res["d_enc"] = d_enc
    res["grads"] = {k: v.clone() for k, v in l.g.items()}
    res["stats"] = st.stats()
    st.close()
    return res


def check_against_oracle(l, case, res, tol, check_bwd=True):
    d = hp.oracle_desc(l)
    kv = case.get("kv_len")
    y, sv = lo.layer_fwd(d, case["w"], case["x"], case.get("enc"), kv)
    errs = {"y": hp.rel_err(res["y"], y)}
    for name, got in res.get("saved", {}).items():
        if name in ("mean1", "mean2", "meanx") and l.norm != "layernorm":
            continue
        errs["saved." + name] = hp.rel_err(got, sv[name])
    if not check_bwd:
        bad = {k: v for k, v in errs.items() if not v <= tol}
        assert not bad, bad
        return errs
    dx, denc, gr = lo.layer_bwd(d, case["w"], sv, case["dy"], kv)
    errs["dx"] = hp.rel_err(runner.to_host(res["dx"]), dx)
    if denc is not None:
        errs["d_enc"] = hp.rel_err(runner.to_host(res["d_enc"]), denc)
    assert set(res["grads"]) == set(gr)
    for k in gr:
        errs["grad." + k] = hp.rel_err(runner.to_host(res["grads"][k]), gr[k])
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, bad
    return errs


def test_config1_gpt_fp32_full_parity_offloaded_and_reloaded():
    cfg = synth.CONFIGS["gpt_small_f32"]
    l = runner.layers_from_config(cfg)[0]
    case = hp.make_layer_case(l, synth.BASE_SEED + 1, bias_std=0.0)
    on = run_single_layer(l, case, offload=True)
    errs = check_against_oracle(l, case, on, hp.TOL["f32"])
    print("config 1 max rel err:", max(errs.values()), max(errs, key=errs.get))
    # all 13 unique storages left the device and came back
    s = on["stats"]
    assert (s["save_calls"], s["unique"], s["dedup_hits"], s["offloaded"], s["kept"]) == (16, 13, 3, 13, 0)
    assert s["bytes_offloaded"] == 4202496 and s["loads"] == 13 and s["bytes_loaded"] == 4202496 and s["forwarded"] == 0
    assert all(r["state"] == sb.ST_OFFLOADED and r["device_ptr"] is None for r in on["records_stored"])
    reg = hp.registry_expectation([l], 0, 0, -1, 2 * runner.saved_bytes_per_layer(l))
    got = [(r["tid"], r["bytes"], r["pack_offset"], r["pool_offset"]) for r in on["records_stored"]]
    assert got == [(r.stamp, r.bytes, r.pack_offset, r.pool_offset) for r in reg.records]
    # offload off: same bits everywhere
    l2 = runner.layers_from_config(cfg)[0]
    off = run_single_layer(l2, case, offload=False)
    assert off["stats"]["offloaded"] == 0 and off["stats"]["kept"] == 13
    assert torch.equal(on["dx"], off["dx"])
    for k in on["grads"]:
        assert torch.equal(on["grads"][k], off["grads"][k]), k
    # the host copies are bit-identical to the activations that were kept
    names = {}
    for i, n in enumerate(sb.SV_NAMES):
        if l.saved.e[i].tid:
            names[l.saved.e[i].tid] = n
    for tid, blob in on["pool"].items():
        kept = off["saved"][names[tid]].astype(np.float32)
        assert blob == kept.tobytes(), names[tid]


VARIANTS = {
    "gpt_ragged": dict(arch="gpt_preln", B=2, S=37, H=96, A=3, F=200, act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
    "bert_keypad": dict(arch="bert_postln", B=3, S=70, H=128, A=4, F=260, act="gelu", norm="layernorm", mask="keypad", has_bias=True, eps=1e-5),
    "t5_enc": dict(arch="t5_enc", B=2, S=65, H=128, A=2, F=192, act="relu", norm="rmsnorm", mask="none", has_bias=False, eps=1e-6),
    "t5_dec": dict(arch="t5_dec", B=2, S=33, S_kv=75, H=128, A=2, F=192, act="relu", norm="rmsnorm", mask="causal", has_bias=False, eps=1e-6),
    "gpt_d128": dict(arch="gpt_preln", B=1, S=130, H=256, A=2, F=512, act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
    # shapes the matrix-core kernels take (multiples of 128; head size 64 / 128)
    "gpt_mfma": dict(arch="gpt_preln", B=2, S=256, H=256, A=2, F=1024, act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
    "bert_mfma": dict(arch="bert_postln", B=3, S=128, H=256, A=4, F=512, act="gelu", norm="layernorm", mask="keypad", has_bias=True, eps=1e-5),
    # head size 128 with key padding: the direct-load attention kernels with ragged valid lengths (a last tile that is
    # partly masked, sequences shorter than one tile)
    "bert_d128": dict(arch="bert_postln", B=3, S=256, H=256, A=2, F=512, act="gelu", norm="layernorm", mask="keypad", has_bias=True, eps=1e-5),
    "t5enc_mfma": dict(arch="t5_enc", B=2, S=128, H=128, A=2, F=384, act="relu", norm="rmsnorm", mask="none", has_bias=False, eps=1e-6),
    "t5dec_mfma": dict(arch="t5_dec", B=2, S=128, S_kv=256, H=128, A=2, F=256, act="relu", norm="rmsnorm", mask="causal", has_bias=False, eps=1e-6),
    # 4096 x 4096 outputs (256 tiles of 256 x 256: the large-tile GEMM kernel) over a contraction of only two
    # and three 64-wide stages: its prologue and its peeled last stages without the steady-state loop between
    "gpt_thin128": dict(arch="gpt_preln", B=2, S=2048, H=128, A=2, F=4096, act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
    "gpt_thin192": dict(arch="gpt_preln", B=2, S=2048, H=192, A=3, F=4096, act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
    # eight heads of size 128 over five query / key blocks: the attention kernels' re-ordered block indices (heads dealt
    # to the XCDs, an odd number of blocks per head) and the key-side backward's descending walk over 20 query tiles
    "gpt_heads8": dict(arch="gpt_preln", B=4, S=640, H=256, A=2, F=512, act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
}


@pytest.mark.parametrize("name", list(VARIANTS))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_variants_small(name, dtype):
    v = dict(VARIANTS[name])
    l = runner.Layer(dtype=dtype, **v)
    kvr = (1, v["S"]) if v["mask"] == "keypad" else None
    case = hp.make_layer_case(l, 1000 + len(name), bias_std=0.05, kv_len_range=kvr)
    for k in case["w"]:
        if k.startswith("w_"):          # larger weights than the workload's so that every path carries signal
            case["w"][k] = synth.bf16_round(case["w"][k] * 4) if dtype == "bf16" else case["w"][k] * 4
    on = run_single_layer(l, case, offload=True)
    # ReLU's derivative is a decision taken on the sign of a computed value: with bf16 storage the
    # two sides can decide differently for pre-activations within rounding distance of zero, so
    # for that combination the chained backward is checked in test_backward_from_checker_saved
    # (same stored activations on both sides) and only forward and bit-transparency here.
    errs = check_against_oracle(l, case, on, hp.TOL[dtype], check_bwd=not (dtype == "bf16" and v["act"] == "relu"))
    l2 = runner.Layer(dtype=dtype, **v)
    off = run_single_layer(l2, case, offload=False, fetch=False)
    assert torch.equal(on["dx"], off["dx"])
    for k in on["grads"]:
        assert torch.equal(on["grads"][k], off["grads"][k]), k
    if on["d_enc"] is not None:
        assert torch.equal(on["d_enc"], off["d_enc"])


@pytest.mark.parametrize("name", ["bert_keypad", "bert_mfma", "bert_d128"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sequence_without_any_admissible_key(name, dtype):
    """Degenerate case of the key-padding mask: one sequence of valid length 0.  Every one of its query rows has
    no key to attend to: probabilities and attention output are exactly 0 there, lse is -inf, and no gradient
    flows through its attention (the convention written in the checker's header); the other sequences are
    unaffected.  Covers both attention paths (generic and matrix-core)."""
    v = dict(VARIANTS[name])
    l = runner.Layer(dtype=dtype, **v)
    case = hp.make_layer_case(l, 3000 + len(name), bias_std=0.05, kv_len_range=(1, v["S"]))
    case["kv_len"] = case["kv_len"].copy()
    case["kv_len"][1] = 0
    for k in case["w"]:
        if k.startswith("w_"):
            case["w"][k] = synth.bf16_round(case["w"][k] * 4) if dtype == "bf16" else case["w"][k] * 4
    on = run_single_layer(l, case, offload=True)
    check_against_oracle(l, case, on, hp.TOL[dtype])
    S, H = v["S"], v["H"]
    lse = on["saved"]["lse"]
    assert np.all(np.isneginf(lse[1])) and np.all(np.isfinite(lse[0])) and np.all(np.isfinite(lse[2]))
    assert not np.any(on["saved"]["o"][S:2 * S])          # exact zeros


@pytest.mark.parametrize("name", list(VARIANTS))
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_from_checker_saved(name, dtype):
    """ssdt_layer_bwd as a function of (saved tensors, dy, weights): the saved tensors are the CPU
    checker's forward results rounded to the storage type, handed over as bypassed entries, so both
    sides differentiate exactly the same stored activations."""
    v = dict(VARIANTS[name])
    l = runner.Layer(dtype=dtype, **v)
    kvr = (1, v["S"]) if v["mask"] == "keypad" else None
    case = hp.make_layer_case(l, 2000 + len(name), bias_std=0.05, kv_len_range=kvr)
    for k in case["w"]:
        if k.startswith("w_"):
            case["w"][k] = synth.bf16_round(case["w"][k] * 4) if dtype == "bf16" else case["w"][k] * 4
    d = hp.oracle_desc(l)
    kv = case.get("kv_len")
    _, sv = lo.layer_fwd(d, case["w"], case["x"], case.get("enc"), kv)
    rnd = (lambda a: synth.bf16_round(a.astype(np.float32)).astype(np.float64)) if dtype == "bf16" else \
          (lambda a: a.astype(np.float32).astype(np.float64))
    stats = {"mean1", "rstd1", "meanx", "rstdx", "mean2", "rstd2", "lse", "lsex"}
    sv_r = {k: (a.astype(np.float32).astype(np.float64) if k in stats else rnd(a)) for k, a in sv.items()}
    dx, denc, gr = lo.layer_bwd(d, case["w"], sv_r, case["dy"], kv)

    st = runner.Stack([l], 1 << 20, 1 << 20, DEV, keep_last=0, min_offload_elems=0)
    hp.load_weights(l, case["w"], st.dev)
    sb.ssdt_step_begin(st.ctx, 1)
    saved = sb.ssdt_layer_saved()
    saved.scope = 0
    keep = []
    for i, n in enumerate(sb.SV_NAMES):
        if n not in sv_r or (n.startswith("mean") and l.norm != "layernorm"):
            continue
        if n in stats:
            t = torch.from_numpy(sv_r[n].astype(np.float32)).to(st.dev).contiguous()
        else:
            t = runner.to_device(sv_r[n].astype(np.float32), dtype, st.dev).contiguous()
        keep.append(t)
        saved.e[i].ptr, saved.e[i].bytes, saved.e[i].tid = t.data_ptr(), t.numel() * t.element_size(), 0
    dy = runner.to_device(case["dy"], dtype, st.dev)
    dxg = torch.empty_like(dy)
    kvt = torch.from_numpy(kv).to(st.dev) if kv is not None else None
    d_enc = torch.zeros(l.B * l.S_kv, l.H, dtype=dy.dtype, device=st.dev) if l.arch == "t5_dec" else None
    sb.ssdt_layer_bwd(st.ctx, l.desc, l.wstruct, saved, kvt.data_ptr() if kvt is not None else 0, dy.data_ptr(),
                      dxg.data_ptr(), d_enc.data_ptr() if d_enc is not None else 0, l.gstruct, st.ws_ptr, st.ws_bytes,
                      st.stream)
    torch.cuda.synchronize()
    errs = {"dx": hp.rel_err(runner.to_host(dxg), dx)}
    if denc is not None:
        errs["d_enc"] = hp.rel_err(runner.to_host(d_enc), denc)
    assert set(l.g) == set(gr)
    for k in gr:
        errs["grad." + k] = hp.rel_err(runner.to_host(l.g[k]), gr[k])
    st.close()
    bad = {k: e for k, e in errs.items() if not e <= hp.TOL[dtype]}
    assert not bad, bad
