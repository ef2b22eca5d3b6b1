"""Pins for the CPU checker of the layer (no GPU).  Each test ties the checker to
something outside itself: finite differences, closed forms, invariants, special cases
that reduce to a library routine (torch CPU ops, autograd), and stored values."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import layer_oracle as lo
from paper_2408_10013_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _case(desc, seed=7, bias_std=0.3, kv=None):
    shapes = lo.weight_shapes(desc)
    c = synth.make_case(shapes, desc.T, desc.H, seed, "f32", T_enc=desc.B * desc.S_kv, bias_std=bias_std,
                        B=desc.B, kv_len_range=kv)
    # larger weights than the workload's 0.02 so that every path carries signal
    for k in c["w"]:
        if k.startswith("w_"):
            c["w"][k] = c["w"][k] * 10.0
    return c


DESCS = {
    "gpt": lo.LayerDesc(arch="gpt_preln", B=2, S=5, H=8, A=2, F=12, mask="causal"),
    "bert": lo.LayerDesc(arch="bert_postln", B=2, S=6, H=8, A=2, F=12, mask="keypad"),
    "t5enc": lo.LayerDesc(arch="t5_enc", B=1, S=5, H=8, A=2, F=12, mask="none", norm="rmsnorm", act="relu",
                          has_bias=False, eps=1e-6),
    "t5dec": lo.LayerDesc(arch="t5_dec", B=2, S=3, S_kv=5, H=8, A=4, F=12, mask="causal", norm="rmsnorm",
                          act="relu", has_bias=False, eps=1e-6),
}


def _loss(desc, w, x, enc, kv_len, dy):
    y, _ = lo.layer_fwd(desc, w, x, enc, kv_len)
    return float((y * dy).sum())


@pytest.mark.parametrize("name", list(DESCS))
def test_backward_matches_central_differences(name):
    desc = DESCS[name]
    kv = (3, 6) if desc.mask == "keypad" else None
    c = _case(desc, kv=kv)
    x = c["x"].astype(np.float64)
    w = {k: v.astype(np.float64) for k, v in c["w"].items()}
    enc = c.get("enc")
    enc = None if enc is None else enc.astype(np.float64)
    kv_len = c.get("kv_len")
    dy = c["dy"].astype(np.float64)
    y, sv = lo.layer_fwd(desc, w, x, enc, kv_len)
    dx, denc, gr = lo.layer_bwd(desc, w, sv, dy, kv_len)
    assert set(gr) == set(w)
    h = 1e-5
    rng = np.random.default_rng(0)

    def check(arr, grad, setter, label):
        flat = arr.reshape(-1)
        idx = rng.choice(flat.size, size=min(flat.size, 24), replace=False)
        for i in idx:
            old = flat[i]
            flat[i] = old + h
            lp = _loss(desc, w, x, enc, kv_len, dy)
            flat[i] = old - h
            lm = _loss(desc, w, x, enc, kv_len, dy)
            flat[i] = old
            fd = (lp - lm) / (2 * h)
            an = grad.reshape(-1)[i]
            scale = max(1.0, abs(fd), float(np.abs(grad).max()))
            assert abs(fd - an) <= 2e-7 * scale, (label, i, fd, an)

    check(x, dx, None, "x")
    if enc is not None:
        check(enc, denc, None, "enc")
    for k in w:
        check(w[k], gr[k], None, k)


@pytest.mark.parametrize("name", list(DESCS))
def test_layer_matches_torch_autograd(name):
    """The same layer written with torch CPU ops in fp64; gradients by autograd."""
    desc = DESCS[name]
    kv = (3, 6) if desc.mask == "keypad" else None
    c = _case(desc, seed=11, kv=kv)
    tw = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in c["w"].items()}
    tx = torch.tensor(c["x"], dtype=torch.float64, requires_grad=True)
    tenc = torch.tensor(c["enc"], dtype=torch.float64, requires_grad=True) if "enc" in c else None
    kv_len = c.get("kv_len")
    B, S, H, A, d = desc.B, desc.S, desc.H, desc.A, desc.d

    def norm(v, p):
        if desc.norm == "layernorm":
            return torch.nn.functional.layer_norm(v, (H,), tw[p + "_g"], tw[p + "_b"], desc.eps)
        return v * torch.rsqrt((v * v).mean(-1, keepdim=True) + desc.eps) * tw[p + "_g"]

    def lin(v, wn, bn):
        out = v @ tw[wn]
        return out + tw[bn] if bn in tw else out

    def mha(q, k, v, Sq, Sk, mask):
        q = q.reshape(B, Sq, A, d).transpose(1, 2)
        k = k.reshape(B, Sk, A, d).transpose(1, 2)
        v = v.reshape(B, Sk, A, d).transpose(1, 2)
        allow = torch.ones(B, 1, Sq, Sk, dtype=torch.bool)
        if mask == "causal":
            allow &= torch.tril(torch.ones(Sq, Sk, dtype=torch.bool))
        if mask == "keypad":
            allow &= (torch.arange(Sk)[None, None, None, :] < torch.tensor(kv_len)[:, None, None, None])
        o = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=allow)
        return o.transpose(1, 2).reshape(B * Sq, H)

    act = torch.nn.functional.gelu if desc.act == "gelu" else torch.relu
    pre = desc.arch != "bert_postln"
    a = norm(tx, "ln1") if pre else tx
    qkv = lin(a, "w_qkv", "b_qkv")
    r1 = tx + lin(mha(qkv[:, :H], qkv[:, H:2 * H], qkv[:, 2 * H:], S, S, desc.mask), "w_o", "b_o")
    x1 = r1 if pre else norm(r1, "ln1")
    if desc.arch == "t5_dec":
        kvx = lin(tenc, "w_kvx", "b_kvx")
        x2 = x1 + lin(mha(lin(norm(x1, "lnx"), "w_qx", "b_qx"), kvx[:, :H], kvx[:, H:], S, desc.S_kv, "none"),
                      "w_ox", "b_ox")
    else:
        x2 = x1
    m = norm(x2, "ln2") if pre else x2
    r2 = x2 + lin(act(lin(m, "w_1", "b_1")), "w_2", "b_2")
    ty = r2 if pre else norm(r2, "ln2")
    tdy = torch.tensor(c["dy"], dtype=torch.float64)
    (ty * tdy).sum().backward()

    y, sv = lo.layer_fwd(desc, c["w"], c["x"], c.get("enc"), kv_len)
    dx, denc, gr = lo.layer_bwd(desc, c["w"], sv, c["dy"], kv_len)
    np.testing.assert_allclose(y, ty.detach().numpy(), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(dx, tx.grad.numpy(), rtol=1e-10, atol=1e-10)
    if tenc is not None:
        np.testing.assert_allclose(denc, tenc.grad.numpy(), rtol=1e-10, atol=1e-10)
    for k in tw:
        np.testing.assert_allclose(gr[k], tw[k].grad.numpy(), rtol=1e-10, atol=1e-10, err_msg=k)


def test_softmax_invariants():
    rng = np.random.default_rng(3)
    B, A, S, d = 2, 3, 9, 4
    q, k, v = (rng.standard_normal((B * S, A * d)) for _ in range(3))
    kv_len = np.array([9, 4], dtype=np.int32)
    for mask in ("none", "causal", "keypad"):
        o, lse, probs = lo.attention_fwd(q, k, v, B, A, 0.5, mask, kv_len)
        for (b, h), p in probs.items():
            np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-12)
            if mask == "causal":
                assert (p[np.triu_indices(S, 1)] == 0).all()
            if mask == "keypad":
                assert (p[:, kv_len[b]:] == 0).all()
            s = (q[b * S:(b + 1) * S, h * d:(h + 1) * d] @ k[b * S:(b + 1) * S, h * d:(h + 1) * d].T) * 0.5
            rebuilt = np.where(p > 0, np.exp(s - lse[b, h][:, None]), 0.0)
            np.testing.assert_allclose(rebuilt, p, atol=1e-12)


def test_attention_special_cases():
    rng = np.random.default_rng(4)
    # one key: output is that key's value
    q, k, v = rng.standard_normal((1, 4)), rng.standard_normal((1, 4)), rng.standard_normal((1, 4))
    o, lse, _ = lo.attention_fwd(q, k, v, 1, 1, 0.5, "none")
    np.testing.assert_allclose(o, v)
    np.testing.assert_allclose(lse[0, 0, 0], 0.5 * float((q @ k.T)[0, 0]))
    # identical keys: output is the mean of the admissible values
    S = 6
    q = rng.standard_normal((S, 4)); k = np.tile(rng.standard_normal((1, 4)), (S, 1)); v = rng.standard_normal((S, 4))
    o, _, _ = lo.attention_fwd(q, k, v, 1, 1, 0.3, "causal")
    for i in range(S):
        np.testing.assert_allclose(o[i], v[:i + 1].mean(axis=0), atol=1e-12)
    # constant values: output constant whatever the scores
    k = rng.standard_normal((S, 4)); v = np.tile(rng.standard_normal((1, 4)), (S, 1))
    o, _, _ = lo.attention_fwd(q, k, v, 1, 1, 0.3, "none")
    np.testing.assert_allclose(o, v, atol=1e-12)
    # no admissible key: p = 0, o = 0, lse = -inf
    o, lse, probs = lo.attention_fwd(q, k, v, 1, 1, 0.3, "keypad", np.array([0]))
    assert (o == 0).all() and np.isneginf(lse).all() and (probs[(0, 0)] == 0).all()
    dq, dk, dv = lo.attention_bwd(np.ones_like(o), q, k, v, o, lse, 1, 1, 0.3, "keypad", np.array([0]))
    assert (dq == 0).all() and (dk == 0).all() and (dv == 0).all()


def test_norm_invariants_and_library():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((7, 16)) * 3 + 1.5
    ones, zeros = np.ones(16), np.zeros(16)
    eps = 1e-5
    y, mu, r = lo.norm_fwd(x, ones, zeros, "layernorm", eps)
    var = x.var(axis=1)
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-12)
    np.testing.assert_allclose(y.var(axis=1), var / (var + eps), rtol=1e-12)
    np.testing.assert_allclose(mu, x.mean(axis=1)); np.testing.assert_allclose(r, 1 / np.sqrt(var + eps))
    g, b = rng.standard_normal(16), rng.standard_normal(16)
    y2, _, _ = lo.norm_fwd(x, g, b, "layernorm", eps)
    ref = torch.nn.functional.layer_norm(torch.tensor(x), (16,), torch.tensor(g), torch.tensor(b), eps).numpy()
    np.testing.assert_allclose(y2, ref, rtol=1e-12, atol=1e-12)
    yr, _, rr = lo.norm_fwd(x, ones, None, "rmsnorm", 1e-6)
    ms = (x * x).mean(axis=1)
    np.testing.assert_allclose((yr * yr).mean(axis=1), ms / (ms + 1e-6), rtol=1e-12)


def test_gelu_relu_pins():
    u = np.linspace(-6, 6, 97)
    assert lo.act_fwd(np.zeros(1), "gelu")[0] == 0.0
    assert lo.act_grad(np.zeros(1), "gelu")[0] == 0.5
    np.testing.assert_allclose(lo.act_fwd(u, "gelu") - lo.act_fwd(-u, "gelu"), u, atol=1e-14)
    np.testing.assert_allclose(lo.act_fwd(u, "gelu"), [0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in u], atol=1e-15)
    np.testing.assert_allclose(lo.act_fwd(u, "gelu"), torch.nn.functional.gelu(torch.tensor(u)).numpy(), atol=1e-14)
    h = 1e-6
    np.testing.assert_allclose(lo.act_grad(u, "gelu"), (lo.act_fwd(u + h, "gelu") - lo.act_fwd(u - h, "gelu")) / (2 * h), atol=1e-8)
    with open(os.path.join(GOLDEN, "gelu_values.json")) as f:
        gold = json.load(f)
    np.testing.assert_allclose(lo.act_fwd(np.array(gold["u"]), "gelu"), gold["gelu"], atol=5e-9)
    assert (lo.act_grad(np.array([-1.0, 0.0, 2.0]), "relu") == [0, 0, 1]).all()
    assert (lo.act_fwd(np.array([-1.0, 0.0, 2.0]), "relu") == [0, 0, 2]).all()


def test_identity_and_zero_weight_cases():
    desc = lo.LayerDesc(arch="gpt_preln", B=1, S=4, H=8, A=2, F=8)
    c = _case(desc, bias_std=0.0)
    w = c["w"]
    # zero output projections: the layer is the identity and passes gradients through
    w["w_o"][:] = 0; w["w_2"][:] = 0
    y, sv = lo.layer_fwd(desc, w, c["x"])
    np.testing.assert_array_equal(y, c["x"].astype(np.float64))
    dx, _, gr = lo.layer_bwd(desc, w, sv, c["dy"])
    np.testing.assert_array_equal(dx, c["dy"].astype(np.float64))
    # identity linear
    x = np.arange(12.0).reshape(3, 4)
    np.testing.assert_array_equal(lo.linear_fwd(x, np.eye(4), None), x)
    dx, dw, db = lo.linear_bwd(np.ones((3, 4)), x, np.eye(4))
    np.testing.assert_array_equal(dw, np.tile(x.sum(axis=0)[:, None], (1, 4)))
    np.testing.assert_array_equal(db, [3, 3, 3, 3])


def test_cross_attention_grad_is_sum_of_layer_contributions():
    desc = DESCS["t5dec"]
    c1, c2 = _case(desc, seed=21), _case(desc, seed=22)
    enc = c1["enc"]
    tot = 0
    for c in (c1, c2):
        _, sv = lo.layer_fwd(desc, c["w"], c["x"], enc)
        _, denc, _ = lo.layer_bwd(desc, c["w"], sv, c["dy"])
        tot = tot + denc

    def loss(e):
        return sum(float((lo.layer_fwd(desc, c["w"], c["x"], e)[0] * c["dy"]).sum()) for c in (c1, c2))
    e = enc.astype(np.float64).copy()
    h = 1e-5
    for i in (0, 7, 33):
        old = e.flat[i]
        e.flat[i] = old + h; lp = loss(e)
        e.flat[i] = old - h; lm = loss(e)
        e.flat[i] = old
        assert abs((lp - lm) / (2 * h) - tot.flat[i]) < 1e-6 * max(1, abs(tot.flat[i]))


def test_float32_instantiation_agrees_with_float64():
    desc = lo.LayerDesc(arch="gpt_preln", B=2, S=16, H=32, A=4, F=64)
    c = _case(desc, seed=9)
    y64, sv64 = lo.layer_fwd(desc, c["w"], c["x"])
    y32, sv32 = lo.layer_fwd(desc, c["w"], c["x"], dtype=np.float32)
    assert y32.dtype == np.float32
    dx64, _, g64 = lo.layer_bwd(desc, c["w"], sv64, c["dy"])
    dx32, _, g32 = lo.layer_bwd(desc, c["w"], sv32, c["dy"], dtype=np.float32)
    rel = lambda a, b: np.abs(a - b).max() / np.abs(b).max()
    assert rel(y32, y64) < 1e-5 and rel(dx32, dx64) < 1e-5
    for k in g64:
        assert rel(g32[k], g64[k]) < 1e-5, k


def test_flop_count_closed_form():
    # fwd+bwd of a causal GPT layer with F = 4H is 3 (24 T H^2 + 2 T S H)
    d = lo.LayerDesc(arch="gpt_preln", B=4, S=1024, H=2048, A=16, F=8192)
    assert lo.layer_flops(d) == 3 * (24 * d.T * d.H ** 2 + 2 * d.T * d.S * d.H)
    assert abs(4 * lo.layer_flops(d) / 5.15e12 - 1) < 0.01
    d = lo.LayerDesc(arch="gpt_preln", B=2, S=128, H=256, A=4, F=1024)
    assert abs(lo.layer_flops(d) / 1.26e9 - 1) < 0.01
