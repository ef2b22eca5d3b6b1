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
