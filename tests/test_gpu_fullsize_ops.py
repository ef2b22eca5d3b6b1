"""Operator-by-operator parity at the benchmark layer shape (gpt_8192: H 8192, 64 heads, FFN 32768, S 2048) for every
micro-batch size of the sweep, in the launch configuration bench.py times, with a dense upstream gradient.

The CPU checker cannot run a whole layer at this size, but it can run every operator of the layer on a sample of
that operator's outputs.  The GPU runs one full layer forward and backward; then each operator is taken by itself:
its inputs are the tensors the GPU itself stored (saved activations, and the intermediate gradients the backward
leaves in its workspace), its reference output is the checker's function on those inputs, on

  * rows spread over every 256-row tile of the token dimension (at least 256 rows) for the eight forward /
    input-gradient matrix products, the norms and the elementwise parts,
  * 64 rows of each weight gradient, and all (or 64 / 512) columns of each bias / gain / shift gradient, summed over
    the full token dimension with every token contributing,
  * whole (sequence, head) pairs, spread over the sequences and over the heads' residues modulo 8, for attention
    forward and backward.

Each comparison is element-wise: the tensor-scaled bar of the other bf16 tests (2e-2), and a per-element bound of a
few bf16 roundings of the reference value plus a small share of the tensor's r.m.s. (the operators are checked one at
a time from identical inputs, so nothing but one output rounding and the fp32 accumulation separates the two sides).
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
CFG = synth.CONFIGS["gpt_8192"]


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


@pytest.fixture(scope="module")
def weights():
    """Seeded weights of one gpt_8192 layer on the device, and the same values widened to fp64 on the host."""
    dev = torch.device(DEV)
    l = runner.layers_from_config(CFG, B=1, n_layers=1)[0]
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + 300)
    w = {}
    for name, shp in l.shapes.items():
        if name.startswith("w_"):
            w[name] = (torch.randn(shp, generator=gen, device=dev) * 0.02).to(torch.bfloat16)
        elif name.endswith("_g"):
            w[name] = (1.0 + 0.1 * torch.randn(shp, generator=gen, device=dev)).to(torch.bfloat16)
        else:
            w[name] = (0.05 * torch.randn(shp, generator=gen, device=dev)).to(torch.bfloat16)
    wh = {k: host(v) for k, v in w.items()}
    yield w, wh
    del w, wh
    torch.cuda.empty_cache()


class Checker:
    def __init__(self):
        self.worst = {}

    def cmp(self, name, got, ref, k_rel=2.0 ** -7, k_rms=8e-3):
        got = np.asarray(got, dtype=np.float64)
        ref = np.asarray(ref, dtype=np.float64)
        assert got.shape == ref.shape, (name, got.shape, ref.shape)
        assert np.isfinite(got).all() and np.isfinite(ref).all(), name
        scaled = hp.rel_err(got, ref)
        rms = float(np.sqrt(np.mean(ref * ref)))
        assert rms > 0, name                                   # a check on zeros would prove nothing
        ex = np.abs(got - ref) - k_rel * np.abs(ref)
        at = np.unravel_index(int(np.argmax(ex)), ex.shape)
        excess = float(ex[at] / rms)
        self.worst[name] = (round(scaled, 5), round(excess, 5))
        assert scaled <= hp.TOL["bf16"], (name, scaled)
        assert excess <= k_rms, (name, "element-wise", excess, k_rms, "at", at, float(got[at]), float(ref[at]), rms)


def sample_rows(T, rng):
    """At least 256 rows, the same number from every 256-row tile, at random places inside the tile."""
    tiles = T // 256
    per = max(2, 256 // tiles)
    return np.sort(np.concatenate([t * 256 + rng.choice(256, per, replace=False) for t in range(tiles)]))


@pytest.mark.parametrize("B", [16, 1, 2, 4, 8])
def test_every_operator_of_the_layer_at_full_shape(B, weights):
    w, wh = weights
    dev = torch.device(DEV)
    l = runner.layers_from_config(CFG, B=B, n_layers=1)[0]
    T, S, H, F, A = l.T, l.S, l.H, l.F, l.A
    d = H // A
    l.set_weights(w)
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.BASE_SEED + 310 + B)
    x = torch.randn(T, H, generator=gen, device=dev).to(torch.bfloat16)
    dy = torch.randn(T, H, generator=gen, device=dev).to(torch.bfloat16)
    rng = np.random.default_rng(synth.BASE_SEED + 320 + B)

    per = runner.saved_bytes_per_layer(l)
    st = runner.Stack([l], 2 * per + (64 << 20), 0, DEV, keep_last=1, min_offload_elems=1 << 20, budget_bytes=0)
    st.register_weights()
    sb.ssdt_step_begin(st.ctx, 1)
    xp, xv = st.arena_tensor((T, H))
    xv.copy_(x)
    yp, l.saved = sb.ssdt_layer_fwd(st.ctx, l.desc, l.wstruct, 0, xp, 0, 0, st.ws_ptr, st.ws_bytes, st.stream)
    torch.cuda.synchronize()

    def sv(name, shape, dtype=torch.bfloat16):
        e = l.saved.e[sb.SV_NAMES.index(name)]
        assert e.ptr and e.bytes, name
        return st.view(e.ptr, shape, dtype)

    a, qkv, o, x1, m = sv("a", (T, H)), sv("qkv", (T, 3 * H)), sv("o", (T, H)), sv("x1", (T, H)), sv("m", (T, H))
    h1, g = sv("h1", (T, F)), sv("g", (T, F))
    mean1, rstd1 = sv("mean1", (T,), torch.float32), sv("rstd1", (T,), torch.float32)
    mean2, rstd2 = sv("mean2", (T,), torch.float32), sv("rstd2", (T,), torch.float32)
    lse = sv("lse", (B, A, S), torch.float32)
    y = st.view(yp, (T, H))
    ck = Checker()
    R = sample_rows(T, rng)
    Rt = torch.from_numpy(R).to(dev)
    rows = lambda t: host(t[Rt])
    scale = 1.0 / np.sqrt(d)
    # (sequence, head) pairs: first / last / middle sequences, heads of different residues modulo 8 (the XCD a
    # head's blocks run on)
    pairs = sorted({(0, 0), (B - 1, A - 1), (B // 2, 9), ((B * 3) // 4, 34), (B // 3, 21), (B - 1, 6)})

    # ---- forward ----------------------------------------------------------------------------------------------
    a_ref, mu_ref, rs_ref = lo.norm_fwd(rows(xv), wh["ln1_g"], wh["ln1_b"], "layernorm", l.eps)
    ck.cmp("a", rows(a), a_ref)
    ck.cmp("mean1", host(mean1[Rt]), mu_ref, 2.0 ** -18, 1e-4)
    ck.cmp("rstd1", host(rstd1[Rt]), rs_ref, 2.0 ** -18, 1e-4)
    ck.cmp("qkv", rows(qkv), lo.linear_fwd(rows(a), wh["w_qkv"], wh["b_qkv"]))
    for (b, h) in pairs:
        rs, cs = slice(b * S, (b + 1) * S), slice(h * d, (h + 1) * d)
        q_, k_, v_ = host(qkv[rs, cs]), host(qkv[rs, H + h * d:H + (h + 1) * d]), host(qkv[rs, 2 * H + h * d:2 * H + (h + 1) * d])
        o_ref, lse_ref, _ = lo.attention_fwd(q_, k_, v_, 1, 1, scale, "causal")
        ck.cmp("o[%d,%d]" % (b, h), host(o[rs, cs]), o_ref, 2.0 ** -6, 1e-2)
        ck.cmp("lse[%d,%d]" % (b, h), host(lse[b, h]), lse_ref[0, 0], 2.0 ** -18, 1e-4)
    ck.cmp("x1", rows(x1), rows(xv) + lo.linear_fwd(rows(o), wh["w_o"], wh["b_o"]))
    m_ref, mu_ref, rs_ref = lo.norm_fwd(rows(x1), wh["ln2_g"], wh["ln2_b"], "layernorm", l.eps)
    ck.cmp("m", rows(m), m_ref)
    ck.cmp("mean2", host(mean2[Rt]), mu_ref, 2.0 ** -18, 1e-4)
    ck.cmp("rstd2", host(rstd2[Rt]), rs_ref, 2.0 ** -18, 1e-4)
    h1_ref = lo.linear_fwd(rows(m), wh["w_1"], wh["b_1"])
    ck.cmp("h1", rows(h1), h1_ref)
    ck.cmp("g", rows(g), lo.act_fwd(h1_ref, "gelu"))
    ck.cmp("y", rows(y), rows(x1) + lo.linear_fwd(rows(g), wh["w_2"], wh["b_2"]))

    # ---- backward ---------------------------------------------------------------------------------------------
    dx = torch.empty_like(dy)
    sb.ssdt_layer_bwd(st.ctx, l.desc, l.wstruct, l.saved, 0, dy.data_ptr(), dx.data_ptr(), 0, l.gstruct, st.ws_ptr,
                      st.ws_bytes, st.stream)
    torch.cuda.synchronize()
    off = sb.ssdt_layer_bwd_temporaries(l.desc)
    ws0 = st.ws_ptr - st.ws.data_ptr()

    def tmp(name, width):
        n = T * width * 2
        return st.ws[ws0 + off[name]:ws0 + off[name] + n].view(torch.bfloat16).reshape(T, width)

    dh1, t0, t1, t2, dqkv = tmp("d_h1", F), tmp("t0", H), tmp("t1", H), tmp("t2", H), tmp("d_qkv", 3 * H)
    none = lambda n: np.zeros((n, 0))                      # "no input": linear_bwd's weight gradient is then empty

    def dgrad(dyr, wname):
        return lo.linear_bwd(dyr, none(dyr.shape[0]), wh[wname])[0]

    def wgrad(inp, dY, krows, extra=None, chunk=4096):
        """Rows `krows` of in^T dY and the column sums of dY over all tokens, accumulated chunk by chunk in fp64;
        `extra(dY_chunk)` lets the caller reuse the converted chunk."""
        kt = torch.from_numpy(krows).to(dev)
        dW, db, ex = 0.0, 0.0, []
        for c0 in range(0, T, chunk):
            dyc = host(dY[c0:c0 + chunk])
            _, dw_c, db_c = lo.linear_bwd(dyc, host(inp[c0:c0 + chunk][:, kt]), np.zeros((0, dyc.shape[1])))
            dW, db = dW + dw_c, db + db_c
            if extra is not None:
                ex.append(extra(dyc))
        return dW, db, ex

    def grads_of(wname, bname, inp, dY, n_in, extra=None):
        krows = np.sort(rng.choice(n_in, 64, replace=False))
        dW, db, ex = wgrad(inp, dY, krows, extra)
        ck.cmp("grad." + wname, host(l.g[wname][torch.from_numpy(krows).to(dev)]), dW)
        ck.cmp("grad." + bname, host(l.g[bname]), db)
        return ex

    # FC2: dh1 = (dy W2^T) * gelu'(h1);  dW2 = g^T dy
    ck.cmp("d_h1", rows(dh1), dgrad(rows(dy), "w_2") * lo.act_grad(rows(h1), "gelu"))
    grads_of("w_2", "b_2", g, dy, F)
    # FC1 and the second norm: dm = dh1 W1^T;  t1 = dy + norm2-backward(dm);  dW1 = m^T dh1
    dm_R = dgrad(rows(dh1), "w_1")
    dn, _, _ = lo.norm_bwd(dm_R, rows(x1), host(mean2[Rt]), host(rstd2[Rt]), wh["ln2_g"], "layernorm")
    ck.cmp("d_x1", rows(t1), rows(dy) + dn, 2.0 ** -7, 1.5e-2)   # two operators: one more rounding in between
    C2 = np.sort(rng.choice(H, 64, replace=False))
    ex = grads_of("w_1", "b_1", m, dh1, H, extra=lambda dyc: dyc @ wh["w_1"][C2, :].T)
    C2t = torch.from_numpy(C2).to(dev)
    _, dg2, db2 = lo.norm_bwd(np.concatenate(ex, axis=0), host(x1[:, C2t]), host(mean2), host(rstd2), wh["ln2_g"][C2], "layernorm")
    ck.cmp("grad.ln2_g", host(l.g["ln2_g"][C2t]), dg2)
    ck.cmp("grad.ln2_b", host(l.g["ln2_b"][C2t]), db2)
    # out-projection: do = t1 Wo^T;  dWo = o^T t1
    ck.cmp("d_o", rows(t0), dgrad(rows(t1), "w_o"))
    grads_of("w_o", "b_o", o, t1, H)
    # attention backward on whole (sequence, head) pairs
    for (b, h) in pairs:
        rs, cs = slice(b * S, (b + 1) * S), slice(h * d, (h + 1) * d)
        ck_, cv_ = slice(H + h * d, H + (h + 1) * d), slice(2 * H + h * d, 2 * H + (h + 1) * d)
        dq_ref, dk_ref, dv_ref = lo.attention_bwd(host(t0[rs, cs]), host(qkv[rs, cs]), host(qkv[rs, ck_]), host(qkv[rs, cv_]),
                                                  host(o[rs, cs]), host(lse[b:b + 1, h:h + 1]), 1, 1, scale, "causal")
        # The fused backward takes delta_i = sum_j p_ij dp_ij as o_i . do_i from the stored (bf16) o, the checker from
        # p and dp themselves; where a row's softmax is concentrated, dp_ij - delta_i is a small difference of large
        # numbers and the 2^-9 rounding of o shows in single rows at several per cent of the tensor's r.m.s.: the
        # per-element bound is accordingly wide here, the tensor-scaled bar is the same 2e-2.
        ck.cmp("dq[%d,%d]" % (b, h), host(dqkv[rs, cs]), dq_ref, 2.0 ** -5, 0.15)
        ck.cmp("dk[%d,%d]" % (b, h), host(dqkv[rs, ck_]), dk_ref, 2.0 ** -5, 0.15)
        ck.cmp("dv[%d,%d]" % (b, h), host(dqkv[rs, cv_]), dv_ref, 2.0 ** -5, 0.15)
    # QKV projection and the first norm: da = dqkv Wqkv^T;  dx = t1 + norm1-backward(da);  dWqkv = a^T dqkv
    ck.cmp("d_a", rows(t2), dgrad(rows(dqkv), "w_qkv"))
    grads_of("w_qkv", "b_qkv", a, dqkv, H)
    dn, _, _ = lo.norm_bwd(rows(t2), rows(xv), host(mean1[Rt]), host(rstd1[Rt]), wh["ln1_g"], "layernorm")
    ck.cmp("dx", rows(dx), rows(t1) + dn, 2.0 ** -7, 1.5e-2)
    C1 = np.sort(rng.choice(H, 512, replace=False))
    C1t = torch.from_numpy(C1).to(dev)
    _, dg1, db1 = lo.norm_bwd(host(t2[:, C1t]), host(xv[:, C1t]), host(mean1), host(rstd1), wh["ln1_g"][C1], "layernorm")
    ck.cmp("grad.ln1_g", host(l.g["ln1_g"][C1t]), dg1)
    ck.cmp("grad.ln1_b", host(l.g["ln1_b"][C1t]), db1)

    sb.ssdt_release(st.ctx, 0, st.stream)
    sb.ssdt_arena_free(st.ctx, yp, st.stream)
    st.close()
    print("B=%d sampled rows %d; worst (tensor-scaled, element-wise excess / rms):" % (B, len(R)),
          sorted(ck.worst.items(), key=lambda kv: -kv[1][0])[:6])
