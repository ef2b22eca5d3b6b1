"""Seeded synthetic workloads (shapes and value distributions only -- no layer arithmetic).

The paper trains BERT, T5 and GPT on a text corpus (Sec. 4.1); layer throughput,
activation bytes and offload traffic depend only on shapes and dtypes, so Gaussian
tensors of the same shapes stand in for it.  Both the GPU tests and the CPU checker take
their inputs from here, as the same bytes.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20240810 * 10

# name -> layer stack description.  `stack` lists (arch, count); sizes follow the five
# benchmark configurations (GPT small fp32, GPT 2048, BERT 1024, T5 2048, GPT 8192).
CONFIGS = {
    "gpt_small_f32": dict(index=1, dtype="f32", stack=[("gpt_preln", 1)], B=2, S=128, H=256, A=4, F=1024,
                          act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
    "gpt_2048": dict(index=2, dtype="bf16", stack=[("gpt_preln", 4)], B=4, S=1024, H=2048, A=16, F=8192,
                     act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
    "bert_1024": dict(index=3, dtype="bf16", stack=[("bert_postln", 8)], B=16, S=512, H=1024, A=16, F=4096,
                      act="gelu", norm="layernorm", mask="keypad", has_bias=True, eps=1e-5,
                      kv_len_range=(256, 512)),
    "t5_2048": dict(index=4, dtype="bf16", stack=[("t5_enc", 2), ("t5_dec", 2)], B=8, S=128, S_enc=512,
                    H=2048, A=32, F=5120, act="relu", norm="rmsnorm", mask="causal", has_bias=False, eps=1e-6),
    "gpt_8192": dict(index=5, dtype="bf16", stack=[("gpt_preln", 8)], B=16, S=2048, H=8192, A=64, F=32768,
                     act="gelu", norm="layernorm", mask="causal", has_bias=True, eps=1e-5),
}


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even) and return them widened to fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(a.shape)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 values that are exactly representable in bf16 -> their 16-bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def _streams(seed: int, n: int):
    return [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(n)]


def gaussian(rng, shape, std=1.0, dtype="f32"):
    v = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
    return bf16_round(v) if dtype == "bf16" else v


def layer_weights(rng, shapes: dict, dtype="f32", bias_std=0.0):
    """Weights N(0, 0.02^2); biases 0 (or N(0, bias_std^2) so that tests exercise the bias
    path); norm gains 1 and shifts 0 (perturbed by bias_std likewise)."""
    w = {}
    for name, shp in shapes.items():
        if name.startswith("w_"):
            w[name] = gaussian(rng, shp, 0.02, dtype)
        elif name.endswith("_g"):
            v = np.ones(shp, dtype=np.float32)
            if bias_std:
                v = v + gaussian(rng, shp, bias_std, "f32")
            w[name] = bf16_round(v) if dtype == "bf16" else v
        else:
            v = gaussian(rng, shp, bias_std, "f32") if bias_std else np.zeros(shp, dtype=np.float32)
            w[name] = bf16_round(v) if dtype == "bf16" else v
    return w


def make_case(shapes: dict, T: int, H: int, seed: int, dtype="f32", T_enc: int = 0, bias_std=0.0,
              B: int = 0, kv_len_range=None):
    """One layer's worth of inputs: x ~ N(0,1), weights, upstream gradient dy ~ N(0,1),
    optional encoder output and per-sequence valid key lengths (uniform, inclusive)."""
    r_x, r_w, r_dy, r_len, r_enc = _streams(seed, 5)
    case = dict(x=gaussian(r_x, (T, H), 1.0, dtype), w=layer_weights(r_w, shapes, dtype, bias_std),
                dy=gaussian(r_dy, (T, H), 1.0, dtype))
    if kv_len_range is not None:
        lo, hi = kv_len_range
        case["kv_len"] = r_len.integers(lo, hi + 1, size=B).astype(np.int32)
    if T_enc:
        case["enc"] = gaussian(r_enc, (T_enc, H), 1.0, dtype)
    return case
