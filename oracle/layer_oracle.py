"""Reference (test-only) CPU implementation of one transformer layer, forward and backward.

THIS IS TEST INFRASTRUCTURE.  It exists to check the GPU library; nothing in the
product path may import it.  It shares no code with the HIP kernels.

What it follows.  The paper (Sec. 2.1, "Transformer-Based LLM") only says that a layer
is an attention block followed by an MLP block, that a decoder layer is an encoder
layer with a causal mask, and that an encoder-decoder's decoder layer carries a second,
cross-attention block over the encoder output.  It gives no formulas, so every function
below is the textbook definition written out step by step, one numpy statement per
mathematical step, with a library matmul / erf as the only primitives.  No blocking,
fusion or reordering is applied.

Precision.  Every function takes `dtype`; the default float64 is what parity tests and
finite-difference checks use, float32 is the "plain fp32" instantiation (its agreement
with float64 is itself a test).

Conventions (all tensors row-major):
  x        [T, H]     T = B*S tokens, sequence b owns rows b*S .. (b+1)*S-1
  w_*      [in, out]  y = x @ w + b
  qkv      [T, 3H]    Q | K | V thirds; head h = columns h*d .. (h+1)*d-1 of a third
  lse      [B, A, S]  log-sum-exp of the scaled, masked scores of each query row
  kv_len   [B]        number of valid keys of sequence b (key-padding mask)

Layer variants:
  gpt_preln   x1 = x + MHA(N1(x));             y = x1 + FFN(N2(x1))
  bert_postln x1 = N1(x + MHA(x));             y = N2(x1 + FFN(x1))
  t5_enc      gpt_preln with RMSNorm, ReLU, no bias, no mask
  t5_dec      x1 = x + MHA_causal(N1(x)); x2 = x1 + MHA_cross(Nx(x1), E); y = x2 + FFN(N2(x2))
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np
from scipy.special import erf as _erf


@dataclass
class LayerDesc:
    arch: str = "gpt_preln"        # gpt_preln | bert_postln | t5_enc | t5_dec
    B: int = 1
    S: int = 4
    S_kv: int = 0                  # encoder length for t5_dec cross-attention
    H: int = 8
    A: int = 2
    F: int = 16
    act: str = "gelu"              # gelu (erf form) | relu
    norm: str = "layernorm"        # layernorm | rmsnorm
    mask: str = "causal"           # none | causal | keypad   (self-attention)
    has_bias: bool = True
    eps: float = 1e-5
    scale: Optional[float] = None  # default 1/sqrt(d)

    @property
    def d(self) -> int:
        return self.H // self.A

    @property
    def T(self) -> int:
        return self.B * self.S

    @property
    def softmax_scale(self) -> float:
        return self.scale if self.scale is not None else 1.0 / float(np.sqrt(self.d))


# --------------------------------------------------------------------------------------
# elementary operators
# --------------------------------------------------------------------------------------

def norm_fwd(x, gamma, beta, kind, eps):
    """LayerNorm: mu = mean_H(x), var = mean_H((x-mu)^2) (biased), r = 1/sqrt(var+eps),
    xhat = (x-mu) r, y = xhat*gamma + beta.  RMSNorm: r = 1/sqrt(mean_H(x^2)+eps),
    xhat = x r, y = xhat*gamma.  Returns y, mean (zeros for RMSNorm), rstd."""
    if kind == "layernorm":
        mu = x.mean(axis=1, keepdims=True)
        var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
        r = 1.0 / np.sqrt(var + eps)
        xhat = (x - mu) * r
        y = xhat * gamma[None, :]
        if beta is not None:
            y = y + beta[None, :]
        return y, mu[:, 0], r[:, 0]
    ms = (x ** 2).mean(axis=1, keepdims=True)
    r = 1.0 / np.sqrt(ms + eps)
    y = (x * r) * gamma[None, :]
    return y, np.zeros(x.shape[0], dtype=x.dtype), r[:, 0]


def norm_bwd(dy, x, mean, rstd, gamma, kind):
    """Gradient of norm_fwd.  With dhat = dy*gamma and xhat as in the forward:
    LayerNorm dx = r (dhat - mean_H(dhat) - xhat mean_H(dhat*xhat));
    RMSNorm   dx = r (dhat - xhat mean_H(dhat*xhat));
    dgamma = sum_t dy*xhat, dbeta = sum_t dy."""
    r = rstd[:, None]
    if kind == "layernorm":
        xhat = (x - mean[:, None]) * r
    else:
        xhat = x * r
    dhat = dy * gamma[None, :]
    c2 = (dhat * xhat).mean(axis=1, keepdims=True)
    if kind == "layernorm":
        c1 = dhat.mean(axis=1, keepdims=True)
        dx = r * (dhat - c1 - xhat * c2)
    else:
        dx = r * (dhat - xhat * c2)
    dgamma = (dy * xhat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    return dx, dgamma, dbeta


def act_fwd(u, kind):
    """GELU in its erf form, 0.5 u (1 + erf(u / sqrt 2)); or ReLU."""
    if kind == "gelu":
        return 0.5 * u * (1.0 + _erf(u / math.sqrt(2.0)))
    return np.maximum(u, 0.0)


def act_grad(u, kind):
    """d act / du: GELU' = Phi(u) + u phi(u) with Phi, phi the standard normal cdf/pdf;
    ReLU' = [u > 0]."""
    if kind == "gelu":
        cdf = 0.5 * (1.0 + _erf(u / math.sqrt(2.0)))
        pdf = np.exp(-0.5 * u * u) / math.sqrt(2.0 * math.pi)
        return cdf + u * pdf
    return (u > 0).astype(u.dtype)


def linear_fwd(x, w, b):
    y = x @ w
    if b is not None:
        y = y + b[None, :]
    return y


def linear_bwd(dy, x, w):
    """dx = dy w^T, dw = x^T dy, db = sum_t dy."""
    return dy @ w.T, x.T @ dy, dy.sum(axis=0)


def _mask_matrix(Sq, Sk, mask, klen):
    """Boolean [Sq, Sk]: True where key j may be attended by query i."""
    allow = np.ones((Sq, Sk), dtype=bool)
    if mask == "causal":
        allow &= np.tril(np.ones((Sq, Sk), dtype=bool))
    if klen is not None:
        allow &= (np.arange(Sk)[None, :] < klen)
    return allow


def attention_fwd(q, k, v, B, A, scale, mask, kv_len=None):
    """Scaled dot-product attention, one (sequence, head) at a time.
    q [B*Sq, A*d]; k, v [B*Sk, A*d].  s_ij = scale q_i.k_j, masked entries are -inf
    (probability exactly 0); p = softmax_j(s); o_i = sum_j p_ij v_j;
    lse_i = max_j s_ij + log sum_j exp(s_ij - max).  A row with no admissible key
    gets p = 0, o = 0, lse = -inf.  Returns o [B*Sq, A*d], lse [B, A, Sq], and the
    list of probability matrices (for tests only)."""
    Tq, Hd = q.shape
    Sq = Tq // B
    Sk = k.shape[0] // B
    d = Hd // A
    o = np.zeros_like(q)
    lse = np.zeros((B, A, Sq), dtype=q.dtype)
    probs = {}
    for b in range(B):
        klen = None if (kv_len is None or mask not in ("keypad",)) else int(kv_len[b])
        allow = _mask_matrix(Sq, Sk, mask, klen)
        for h in range(A):
            qs = q[b * Sq:(b + 1) * Sq, h * d:(h + 1) * d]
            ks = k[b * Sk:(b + 1) * Sk, h * d:(h + 1) * d]
            vs = v[b * Sk:(b + 1) * Sk, h * d:(h + 1) * d]
            s = (qs @ ks.T) * scale
            s = np.where(allow, s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            m_safe = np.where(np.isfinite(m), m, 0.0)
            e = np.exp(s - m_safe)                      # exp(-inf) = 0 exactly
            z = e.sum(axis=1, keepdims=True)
            p = np.divide(e, z, out=np.zeros_like(e), where=z > 0)
            o[b * Sq:(b + 1) * Sq, h * d:(h + 1) * d] = p @ vs
            with np.errstate(divide="ignore"):
                lse[b, h, :] = (m_safe + np.log(z))[:, 0]
            lse[b, h, z[:, 0] == 0] = -np.inf
            probs[(b, h)] = p
    return o, lse, probs


def attention_bwd(do, q, k, v, o, lse, B, A, scale, mask, kv_len=None):
    """Gradient of attention_fwd.  p_ij = exp(scale q_i.k_j - lse_i) on admissible
    entries; dv_j = sum_i p_ij do_i; dp_ij = do_i.v_j; ds_ij = p_ij (dp_ij - sum_j p_ij dp_ij);
    dq_i = scale sum_j ds_ij k_j; dk_j = scale sum_i ds_ij q_i."""
    Tq, Hd = q.shape
    Sq = Tq // B
    Sk = k.shape[0] // B
    d = Hd // A
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    dv = np.zeros_like(v)
    for b in range(B):
        klen = None if (kv_len is None or mask not in ("keypad",)) else int(kv_len[b])
        allow = _mask_matrix(Sq, Sk, mask, klen)
        for h in range(A):
            rq = slice(b * Sq, (b + 1) * Sq)
            rk = slice(b * Sk, (b + 1) * Sk)
            c = slice(h * d, (h + 1) * d)
            s = (q[rq, c] @ k[rk, c].T) * scale
            l = lse[b, h, :][:, None]
            l_safe = np.where(np.isfinite(l), l, 0.0)
            p = np.where(allow & np.isfinite(l), np.exp(np.where(allow, s, 0.0) - l_safe), 0.0)
            dv[rk, c] = p.T @ do[rq, c]
            dp = do[rq, c] @ v[rk, c].T
            delta = (p * dp).sum(axis=1, keepdims=True)
            ds = p * (dp - delta)
            dq[rq, c] = (ds @ k[rk, c]) * scale
            dk[rk, c] = (ds.T @ q[rq, c]) * scale
    return dq, dk, dv


# --------------------------------------------------------------------------------------
# the layer
# --------------------------------------------------------------------------------------

def _g(w, name):
    v = w.get(name)
    return v


def _cast(w: Dict[str, np.ndarray], dtype):
    return {k: (None if v is None else np.asarray(v, dtype=dtype)) for k, v in w.items()}


def layer_fwd(desc: LayerDesc, w: Dict[str, np.ndarray], x, enc_out=None, kv_len=None,
              dtype=np.float64):
    """Forward of one layer.  Returns (y, saved) where `saved` holds every tensor the
    backward needs, under the names used in the saved-tensor trace."""
    w = _cast(w, dtype)
    x = np.asarray(x, dtype=dtype)
    H, A, B = desc.H, desc.A, desc.B
    sc = desc.softmax_scale
    sv: Dict[str, np.ndarray] = {}
    pre = desc.arch != "bert_postln"
    nk = desc.norm

    # ---- self-attention block ----
    sv["x"] = x
    if pre:
        a, sv["mean1"], sv["rstd1"] = norm_fwd(x, w["ln1_g"], _g(w, "ln1_b"), nk, desc.eps)
        sv["a"] = a
    else:
        a = x
    qkv = linear_fwd(a, w["w_qkv"], _g(w, "b_qkv"))
    sv["qkv"] = qkv
    q, k, v = qkv[:, :H], qkv[:, H:2 * H], qkv[:, 2 * H:]
    o, lse, _ = attention_fwd(q, k, v, B, A, sc, desc.mask, kv_len)
    sv["o"], sv["lse"] = o, lse
    r1 = x + linear_fwd(o, w["w_o"], _g(w, "b_o"))
    if pre:
        x1 = r1
    else:
        sv["r1"] = r1
        x1, sv["mean1"], sv["rstd1"] = norm_fwd(r1, w["ln1_g"], _g(w, "ln1_b"), nk, desc.eps)
    sv["x1"] = x1

    # ---- cross-attention block (t5_dec only) ----
    if desc.arch == "t5_dec":
        E = np.asarray(enc_out, dtype=dtype)
        sv["enc"] = E
        ax, sv["meanx"], sv["rstdx"] = norm_fwd(x1, w["lnx_g"], _g(w, "lnx_b"), nk, desc.eps)
        sv["ax"] = ax
        qx = linear_fwd(ax, w["w_qx"], _g(w, "b_qx"))
        kvx = linear_fwd(E, w["w_kvx"], _g(w, "b_kvx"))
        sv["qx"], sv["kvx"] = qx, kvx
        ox, lsex, _ = attention_fwd(qx, kvx[:, :H], kvx[:, H:], B, A, sc, "none", None)
        sv["ox"], sv["lsex"] = ox, lsex
        x2 = x1 + linear_fwd(ox, w["w_ox"], _g(w, "b_ox"))
        sv["x2"] = x2
    else:
        x2 = x1

    # ---- feed-forward block ----
    if pre:
        m, sv["mean2"], sv["rstd2"] = norm_fwd(x2, w["ln2_g"], _g(w, "ln2_b"), nk, desc.eps)
        sv["m"] = m
    else:
        m = x2
    h1 = linear_fwd(m, w["w_1"], _g(w, "b_1"))
    g = act_fwd(h1, desc.act)
    sv["h1"], sv["g"] = h1, g
    r2 = x2 + linear_fwd(g, w["w_2"], _g(w, "b_2"))
    if pre:
        y = r2
    else:
        sv["r2"] = r2
        y, sv["mean2"], sv["rstd2"] = norm_fwd(r2, w["ln2_g"], _g(w, "ln2_b"), nk, desc.eps)
    return y, sv


def layer_bwd(desc: LayerDesc, w: Dict[str, np.ndarray], sv: Dict[str, np.ndarray], dy,
              kv_len=None, dtype=np.float64):
    """Backward of one layer.  Returns (dx, d_enc_out or None, grads) with `grads`
    keyed like the weights."""
    w = _cast(w, dtype)
    dy = np.asarray(dy, dtype=dtype)
    H, A, B = desc.H, desc.A, desc.B
    sc = desc.softmax_scale
    pre = desc.arch != "bert_postln"
    nk = desc.norm
    gr: Dict[str, np.ndarray] = {}
    d_enc = None

    # ---- feed-forward block ----
    x2 = sv["x2"] if desc.arch == "t5_dec" else sv["x1"]
    if pre:
        dr2 = dy
        m = sv["m"]
    else:
        dr2, gr["ln2_g"], gr["ln2_b"] = norm_bwd(dy, sv["r2"], sv["mean2"], sv["rstd2"], w["ln2_g"], nk)
        m = x2
    dg, gr["w_2"], gr["b_2"] = linear_bwd(dr2, sv["g"], w["w_2"])
    dh1 = dg * act_grad(sv["h1"], desc.act)
    dm, gr["w_1"], gr["b_1"] = linear_bwd(dh1, m, w["w_1"])
    if pre:
        dn, gr["ln2_g"], gr["ln2_b"] = norm_bwd(dm, x2, sv["mean2"], sv["rstd2"], w["ln2_g"], nk)
        dx2 = dr2 + dn
    else:
        dx2 = dr2 + dm

    # ---- cross-attention block ----
    if desc.arch == "t5_dec":
        dox, gr["w_ox"], gr["b_ox"] = linear_bwd(dx2, sv["ox"], w["w_ox"])
        kvx = sv["kvx"]
        dqx, dkx, dvx = attention_bwd(dox, sv["qx"], kvx[:, :H], kvx[:, H:], sv["ox"], sv["lsex"],
                                      B, A, sc, "none", None)
        dax, gr["w_qx"], gr["b_qx"] = linear_bwd(dqx, sv["ax"], w["w_qx"])
        dkvx = np.concatenate([dkx, dvx], axis=1)
        d_enc, gr["w_kvx"], gr["b_kvx"] = linear_bwd(dkvx, sv["enc"], w["w_kvx"])
        dn, gr["lnx_g"], gr["lnx_b"] = norm_bwd(dax, sv["x1"], sv["meanx"], sv["rstdx"], w["lnx_g"], nk)
        dx1 = dx2 + dn
    else:
        dx1 = dx2

    # ---- self-attention block ----
    if pre:
        dr1 = dx1
        a = sv["a"]
    else:
        dr1, gr["ln1_g"], gr["ln1_b"] = norm_bwd(dx1, sv["r1"], sv["mean1"], sv["rstd1"], w["ln1_g"], nk)
        a = sv["x"]
    do, gr["w_o"], gr["b_o"] = linear_bwd(dr1, sv["o"], w["w_o"])
    qkv = sv["qkv"]
    dq, dk, dv = attention_bwd(do, qkv[:, :H], qkv[:, H:2 * H], qkv[:, 2 * H:], sv["o"], sv["lse"],
                               B, A, sc, desc.mask, kv_len)
    dqkv = np.concatenate([dq, dk, dv], axis=1)
    da, gr["w_qkv"], gr["b_qkv"] = linear_bwd(dqkv, a, w["w_qkv"])
    if pre:
        dn, gr["ln1_g"], gr["ln1_b"] = norm_bwd(da, sv["x"], sv["mean1"], sv["rstd1"], w["ln1_g"], nk)
        dx = dr1 + dn
    else:
        dx = dr1 + da
    gr = {k: v for k, v in gr.items() if w.get(k) is not None}   # absent biases / shifts have no gradient
    return dx, d_enc, gr


def weight_shapes(desc: LayerDesc):
    """Name -> shape of every parameter of a layer, in the order the C struct lists them.
    Biases and LayerNorm shifts are absent when has_bias is false / RMSNorm is used."""
    H, F = desc.H, desc.F
    out = {}
    def norm(prefix):
        out[prefix + "_g"] = (H,)
        if desc.norm == "layernorm":
            out[prefix + "_b"] = (H,)
    def lin(wn, bn, i, o):
        out[wn] = (i, o)
        if desc.has_bias:
            out[bn] = (o,)
    norm("ln1")
    lin("w_qkv", "b_qkv", H, 3 * H)
    lin("w_o", "b_o", H, H)
    if desc.arch == "t5_dec":
        norm("lnx")
        lin("w_qx", "b_qx", H, H)
        lin("w_kvx", "b_kvx", H, 2 * H)
        lin("w_ox", "b_ox", H, H)
    norm("ln2")
    lin("w_1", "b_1", H, F)
    lin("w_2", "b_2", F, H)
    return out


def layer_flops(desc: LayerDesc, kv_len=None, fwd_bwd=True):
    """Algorithmic FLOPs of one layer: 2 m n k per matmul; attention 4 Sq Sk H per
    sequence, halved under a causal mask, Sk replaced by the valid length under key
    padding; backward = 2x forward (recomputation inside a fused attention backward is
    not counted, in line with the paper's definition of model throughput, Sec. 4.3)."""
    T, H, F, B, S = desc.T, desc.H, desc.F, desc.B, desc.S
    f = 2 * T * H * 3 * H + 2 * T * H * H + 4 * T * H * F
    if desc.mask == "causal":
        f += 2 * B * S * S * H
    elif desc.mask == "keypad" and kv_len is not None:
        f += sum(4 * S * int(l) * H for l in kv_len)
    else:
        f += 4 * B * S * S * H
    if desc.arch == "t5_dec":
        Te = B * desc.S_kv
        f += 2 * T * H * H + 2 * Te * H * 2 * H + 2 * T * H * H + 4 * B * S * desc.S_kv * H
    return 3 * f if fwd_bwd else f
