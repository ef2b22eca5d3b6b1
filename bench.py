#!/usr/bin/env python3
"""Benchmark of the layer forward+backward with activation offloading on one MI355X.

A step = forward then backward of the whole layer stack over one micro-batch of seeded
synthetic tensors (inputs resident in HBM), including every offload, prefetch and release.
Three modes are timed back to back with the same context and arena:
  off     offload amount 0: every saved tensor stays on the device
  all     every saved tensor of every layer but the last is offloaded and prefetched back
  recompute  nothing offloaded, every layer re-run inside its backward (only with --modes ...,recompute)
  budget  the offload amount is set from the measured link rate so that the I/O hides
          behind compute (the paper's adaptive offload amount, Sec. 3.1); the headline value
  file    (only with --modes ...,file) the file tier: two layers' worth offloaded through the pinned pool into a
          file opened for direct I/O under --spill-dir and read back from it, timed against the same amount
          served from the pool alone ("pool2"); reports the file's write / read rate as the offload path drives it
The JSON line printed at the end carries the headline (budget mode), the other two modes,
the roofline of the dominant kernel (timed with HIP events on its launch stream inside the
timed region) and the CPU checker timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

KERNEL_SOURCE = {"gemm_nt256_k": "kernels_mfma.hip", "gemm_km256_k": "kernels_mfma_km.hip"}


def recorded_traffic(kernel, workload, B):
    """HBM bytes per launch of the dominant kernel from the committed counter summary
    (profiles/traffic_<kernel>__<workload>_b<B>.md); None when there is no summary for this kernel / workload or
    when the kernel's source has changed since the counters were taken."""
    import hashlib
    import re
    rec = os.path.join(ROOT, "profiles", "traffic_%s__%s_b%d.md" % (kernel, workload, B))
    if kernel not in KERNEL_SOURCE or not os.path.exists(rec):
        return None
    txt = open(rec).read()
    m = {k: re.search(r"^%s:\s*(\S+)" % k, txt, re.M) for k in ("traffic_bytes_per_launch", "kernel_source_sha256")}
    if not all(m.values()):
        return None
    src = os.path.join(ROOT, "paper_2408_10013_amd", "csrc", KERNEL_SOURCE[kernel])
    if hashlib.sha256(open(src, "rb").read()).hexdigest() != m["kernel_source_sha256"].group(1):
        return None
    return float(m["traffic_bytes_per_launch"].group(1))


MFMA_BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16
HOST_LINK_PEAK_GBPS = 64.0          # PCIe 5.0 x16, per direction
HBM_PEAK_TBPS = 8.0                 # MI355X HBM3E


def stack_flops(layers, kv_len=None):
    tot = 0
    for l in layers:
        T, H, F, B, S = l.T, l.H, l.F, l.B, l.S
        f = 2 * T * H * 3 * H + 2 * T * H * H + 4 * T * H * F
        if l.mask == "causal":
            f += 2 * B * S * S * H
        elif l.mask == "keypad" and kv_len is not None:
            f += sum(4 * S * int(v) * H for v in kv_len)
        else:
            f += 4 * B * S * S * H
        if l.arch == "t5_dec":
            Te = B * l.S_kv
            f += 4 * T * H * H + 4 * Te * H * H + 4 * B * S * l.S_kv * H
        tot += 3 * f
    return tot


def cpu_baseline(cfg):
    """Times the CPU checker (as it stands) on bounded samples of the workload, forward + backward: (a) one layer at
    the workload's real widths with few tokens, all host threads (the headline figure); (b) the small fp32
    configuration in full, all threads and one thread; (c) a still smaller token sample of (a) on one thread."""
    import numpy as np
    from oracle import layer_oracle as lo
    from paper_2408_10013_amd import synth
    try:
        from threadpoolctl import threadpool_limits
    except Exception:      # no way to pin the BLAS thread count: single-thread figures are left out
        threadpool_limits = None
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))

    def run(d, dtype, limit=None):
        shapes = lo.weight_shapes(d)
        case = synth.make_case(shapes, d.T, d.H, synth.BASE_SEED + 99, dtype)

        def go():
            t0 = time.perf_counter()
            y, sv = lo.layer_fwd(d, case["w"], case["x"])
            lo.layer_bwd(d, case["w"], sv, case["dy"])
            return time.perf_counter() - t0
        if limit is None:
            dt = go()
        else:
            with threadpool_limits(limits=limit):
                dt = go()
        return dt, lo.layer_flops(d) / dt / 1e12

    arch = cfg["stack"][0][0]
    mask = "causal" if cfg["mask"] == "causal" else "none"
    big = lambda S: lo.LayerDesc(arch=arch, B=1, S=S, H=cfg["H"], A=cfg["A"], F=cfg["F"], act=cfg["act"], norm=cfg["norm"],
                                 mask=mask, has_bias=cfg["has_bias"], eps=cfg["eps"])
    dt, tf = run(big(2048), "bf16")            # about 10-20 s of host work at the headline widths
    out = {"value": tf, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
           "sample": "1 %s layer fwd+bwd at H=%d F=%d A=%d with B=1 S=2048 tokens, numpy fp64, %.1f s"
                     % (arch, cfg["H"], cfg["F"], cfg["A"], dt)}
    c1 = synth.CONFIGS["gpt_small_f32"]
    d1 = lo.LayerDesc(arch="gpt_preln", B=c1["B"], S=c1["S"], H=c1["H"], A=c1["A"], F=c1["F"])
    run(d1, "f32")                              # warm the BLAS threads
    dt1, tf1 = run(d1, "f32")
    out["config1_full"] = {"seconds": dt1, "TFLOPs": tf1, "threads": threads,
                           "sample": "gpt_small_f32 in full (B=2 S=128 H=256 F=1024), fwd+bwd"}
    if threadpool_limits is not None:
        dt1s, tf1s = run(d1, "f32", 1)
        out["config1_full_1thread"] = {"seconds": dt1s, "TFLOPs": tf1s, "threads": 1}
        dts, tfs = run(big(64), "bf16", 1)
        out["one_thread"] = {"seconds": dts, "TFLOPs": tfs, "threads": 1,
                             "sample": "the same layer with B=1 S=64 tokens"}
    return out


def link_rate(torch, dev, nbytes=1 << 28):
    """Measured ceiling of one pinned hipMemcpyAsync each way, GB/s."""
    h = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    d = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    out = {}
    for name, (dst, src) in {"d2h": (h, d), "h2d": (d, h)}.items():
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        dst.copy_(src, non_blocking=True)
        e1.record()
        torch.cuda.synchronize()
        out[name] = nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del h, d
    return out


def hbm_copy_rate(torch, dev, nbytes=1 << 30):
    """Measured ceiling of a plain 1 GiB device-to-device copy: bytes read + written per second, TB/s."""
    a = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    a.zero_()
    b.copy_(a)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 5
    del a, b
    torch.cuda.empty_cache()
    return 2 * nbytes / (ms * 1e-3) / 1e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="gpt_8192")
    ap.add_argument("--micro-batch", type=int, default=0, help="0 = the configuration's own")
    ap.add_argument("--layers", type=int, default=0, help="0 = the configuration's own")
    ap.add_argument("--modes", default="off,all,budget")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--spill-dir", default="", help="directory for the spill file of the file mode (default: the "
                                                    "system's temporary directory)")
    ap.add_argument("--no-sweep", action="store_true",
                    help="leave the micro-batch sweep (sizes below the configuration's own, off / adaptive offload, "
                         "2 timed steps each) out of the default line")
    ap.add_argument("--sweep", default="", help="comma-separated micro-batch sizes: one off/budget measurement per size "
                                                "(throughput and activation memory vs micro-batch), printed as one JSON line")
    ap.add_argument("--accumulate-sweep", default="",
                    help="comma-separated micro-batch sizes: a training step of --global-batch sequences split into "
                         "micro-batches of each size, gradients accumulated, one SGD update at the end (no offload)")
    ap.add_argument("--global-batch", type=int, default=16)
    ap.add_argument("--copy-probe", action="store_true",
                    help="run one 1 GiB device-to-device copy and exit: the kernel of known size that calibrates the "
                         "HBM byte counters of a profiler run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one process, one MI355X, no collectives); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2408_10013_amd import binding as sb
    from paper_2408_10013_amd import runner, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    if args.copy_probe:
        a = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read": a.numel() * 4, "copy_probe_bytes_written": a.numel() * 4}))
        return
    cfg = synth.CONFIGS[args.workload]
    dtype = cfg["dtype"]
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    weights_cache = {}

    def init_weights(layers):
        """Seeded synthetic weights, generated on the device (the same for every micro-batch size)."""
        gen = torch.Generator(device=dev)
        gen.manual_seed(synth.BASE_SEED + cfg["index"])
        for li, l in enumerate(layers):
            if li not in weights_cache:
                w = {}
                for name, shp in l.shapes.items():
                    if name.startswith("w_"):
                        w[name] = (torch.randn(shp, generator=gen, device=dev, dtype=torch.float32) * 0.02).to(tdt)
                    elif name.endswith("_g"):
                        w[name] = torch.ones(shp, device=dev, dtype=tdt)
                    else:
                        w[name] = torch.zeros(shp, device=dev, dtype=tdt)
                weights_cache[li] = w
            l.set_weights(weights_cache[li])
        return gen

    def measure(B, want):
        layers = runner.layers_from_config(cfg, B=B, n_layers=args.layers or None)
        L = len(layers)
        gen = init_weights(layers)
        first_dec = next((l for l in layers if l.arch != "t5_enc"), layers[0])
        x = torch.randn(first_dec.T, first_dec.H, generator=gen, device=dev, dtype=torch.float32).to(tdt)
        dy = torch.randn(first_dec.T, first_dec.H, generator=gen, device=dev, dtype=torch.float32).to(tdt)
        enc_x = None
        if layers[0].arch == "t5_enc":
            enc_x = torch.randn(layers[0].T, layers[0].H, generator=gen, device=dev, dtype=torch.float32).to(tdt)
        kv_len = None
        if cfg.get("kv_len_range"):
            lo_, hi_ = cfg["kv_len_range"]
            kv_len = torch.from_numpy(np.random.default_rng(synth.BASE_SEED).integers(lo_, hi_ + 1, size=B).astype(np.int32)).to(dev)

        per_layer = [runner.saved_bytes_per_layer(l) for l in layers]
        full = sum(per_layer) + max(per_layer) + (64 << 20)   # every layer resident, plus slack
        flops = stack_flops(layers, kv_len.cpu().numpy() if kv_len is not None else None)
        setup = {}

        def run_mode(name, budget, arena_bytes, pool_bytes, profile=False, distance=1, recompute=False, spill_path=None,
                     settle=False):
            """One context per mode: the arena size is what bounds the activation memory of that mode."""
            t0 = time.perf_counter()
            st = runner.Stack(layers, arena_bytes, pool_bytes, "cuda:0", keep_last=1, min_offload_elems=1 << 20,
                              budget_bytes=budget, measure_waits=1, spill_path=spill_path)
            st.prefetch_distance = distance
            st.recompute = recompute
            st.register_weights()
            setup[name] = time.perf_counter() - t0

            def step():
                y = st.forward(x, enc_x=enc_x, kv_len=kv_len)
                if settle:      # file mode and its pool-only twin: stores (and file writes) finish before backward
                    torch.cuda.synchronize()
                    sb.ssdt_sync_io(st.ctx)
                st.backward(dy)
                sb.ssdt_arena_free(st.ctx, y, st.stream)

            for _ in range(args.warmup):
                step()
            torch.cuda.synchronize()
            sb.ssdt_sync_io(st.ctx)
            if profile:
                sb.ssdt_profile(st.ctx, True)
            marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
            t0 = time.perf_counter()
            marks[0].record()
            for i in range(args.steps):
                step()
                marks[i + 1].record()      # on the compute stream, no synchronisation between steps
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / args.steps
            per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
            prof = None
            if profile:
                prof = sb.ssdt_profile_read(st.ctx)
                sb.ssdt_profile(st.ctx, False)
            s = st.stats()
            spill = None
            if spill_path:
                sb.ssdt_sync_io(st.ctx)
                si = sb.ssdt_spill_info(st.ctx)
                spill = {"direct_io": bool(si["direct_io"]), "threads": si["threads"],
                         "bytes_written": si["bytes_written"], "bytes_read": si["bytes_read"],
                         "write_GBps": si["bytes_written"] / max(1, si["write_busy_ns"]),
                         "read_GBps": si["bytes_read"] / max(1, si["read_busy_ns"])}
            st.close()
            del st
            torch.cuda.empty_cache()
            return dict(spill=spill, ms_per_step=dt * 1e3, tflops=flops / dt / 1e12,
                        ms_per_step_median=per_step[len(per_step) // 2], ms_per_step_min=per_step[0],
                        tflops_median=flops / (per_step[len(per_step) // 2] * 1e-3) / 1e12,
                        tflops_best=flops / (per_step[0] * 1e-3) / 1e12, arena_bytes=arena_bytes,
                        bytes_offloaded=s["bytes_offloaded"], bytes_kept=s["bytes_kept"], bytes_loaded=s["bytes_loaded"],
                        forwarded=s["forwarded"], loads=s["loads"], arena_peak_bytes=s["arena_peak_in_use"],
                        exposed_load_wait_ms=s["exposed_load_wait_ns"] / 1e6,      # of the last timed step
                        exposed_store_wait_ms=s["exposed_store_wait_ns"] / 1e6,
                        link_GBps=(s["bytes_offloaded"] + s["bytes_loaded"]) / dt / 1e9), prof

        modes = {}
        prof = None
        modes["off"], prof = run_mode("off", 0, full, 0, profile=("budget" not in want))
        if "all" in want:
            # three layers' worth of arena: the layer computing, the one being stored / loaded, and slack
            modes["all"], _ = run_mode("all", -1, 3 * max(per_layer) + (64 << 20), runner.pool_bytes_needed(layers))
        if "budget" in want:
            # The offload amount comes from the planner (Sec. 3.1: it is set from the amount of computation, the
            # activation sizes, the GPU throughput and the I/O bandwidth): per-layer times are the layers' FLOP
            # shares of the measured step without offload, the rates are the measured link rates.  The arena
            # shrinks by what is expected to have left the device by the end of the forward pass.
            t_off = modes["off"]["ms_per_step"] * 1e-3
            lf = [stack_flops([l], kv_len.cpu().numpy() if kv_len is not None else None) for l in layers]
            fwd_s = [t_off * f / sum(lf) / 3.0 for f in lf]
            plan = sb.ssdt_plan(per_layer, fwd_s, [2.0 * t for t in fwd_s], link["d2h"] * 1e9, link["h2d"] * 1e9,
                                safety=0.85, keep_last=1)
            budget = plan["budget_bytes"]
            arena = modes["off"]["arena_peak_bytes"] + (256 << 20) + max(per_layer) // 4 - int(0.75 * budget)
            modes["budget"], prof = run_mode("budget", budget, arena, budget + (256 << 20), profile=True,
                                             distance=max(1, plan["prefetch_distance"]))
            modes["budget"]["plan"] = plan
            modes["budget"]["budget_bytes"] = budget
        if "file" in want:
            # The file tier (Sec. 3.1: the SSD offloader next to the CPU offloader): the first two layers' worth of
            # saved tensors leave through the pinned pool into a file and come back from it, with an arena that has
            # no room to keep them; "pool2" is the same amount served from the pool alone.
            import tempfile
            amount = sum(per_layer[:min(2, L - 1)])
            arena = modes["off"]["arena_peak_bytes"] + (256 << 20) + max(per_layer) // 4 - amount
            path = os.path.join(args.spill_dir or tempfile.gettempdir(), "ssdt_bench_spill_%d.bin" % os.getpid())
            # The host enqueues a whole pass ahead of the GPU, and a tensor whose copy out has not been seen finished
            # when backward asks for it is served from the pool.  To time the file itself both runs let the stores
            # (and the file writes) finish between forward and backward, so their step times include that wait.
            modes["pool2"], _ = run_mode("pool2", amount, arena, amount + (256 << 20), distance=2, settle=True)
            try:
                modes["file"], _ = run_mode("file", amount, arena, amount + (256 << 20), distance=2, spill_path=path,
                                            settle=True)
            finally:
                if os.path.exists(path):
                    os.remove(path)
        if "recompute" in want:
            # layerwise full recomputation, nothing offloaded: the third arm of the comparison in Sec. 4.3.  Its
            # rate counts the algorithmic FLOPs only (the repeated forward is overhead, as in the paper's "model
            # throughput").
            modes["recompute"], _ = run_mode("recompute", 0, sum(l.T * l.H * (4 if l.dtype == "f32" else 2) for l in layers) + 2 * max(per_layer)
                                             + (256 << 20), 0, recompute=True)
        for k, m in modes.items():
            m["exposed_io_pct"] = max(0.0, (m["ms_per_step"] - modes["off"]["ms_per_step"]) / m["ms_per_step"] * 100.0)
            m["arena_peak_vs_off"] = m["arena_peak_bytes"] / max(1, modes["off"]["arena_peak_bytes"])
        return layers, modes, prof, setup

    def measure_accumulate(B, n_mb):
        """Training step of n_mb micro-batches of size B with gradient accumulation and one SGD update; everything
        stays on the device (budget 0).  Returns time per step, algorithmic rate, time in the SGD kernel."""
        layers = runner.layers_from_config(cfg, B=B, n_layers=args.layers or None)
        gen = init_weights(layers)
        T, H = layers[0].T, layers[0].H
        xs = [torch.randn(T, H, generator=gen, device=dev, dtype=torch.float32).to(tdt) for _ in range(min(n_mb, 2))]
        dys = [torch.randn(T, H, generator=gen, device=dev, dtype=torch.float32).to(tdt) * 1e-3 for _ in range(min(n_mb, 2))]
        xs = [xs[i % len(xs)] for i in range(n_mb)]
        dys = [dys[i % len(dys)] for i in range(n_mb)]
        per_layer = [runner.saved_bytes_per_layer(l) for l in layers]
        st = runner.Stack(layers, sum(per_layer) + max(per_layer) + (64 << 20), 0, "cuda:0", keep_last=1,
                          min_offload_elems=1 << 20, budget_bytes=0)
        st.register_weights()
        for _ in range(args.warmup):
            st.train_step(xs, dys, 1e-6)
        torch.cuda.synchronize()
        sb.ssdt_profile(st.ctx, True)
        t0 = time.perf_counter()
        for _ in range(args.steps):
            st.train_step(xs, dys, 1e-6)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        prof = {p["name"]: p for p in sb.ssdt_profile_read(st.ctx)}
        sb.ssdt_profile(st.ctx, False)
        peak = st.stats()["arena_peak_in_use"]
        st.close()
        del st, layers
        torch.cuda.empty_cache()
        fl = n_mb * stack_flops(runner.layers_from_config(cfg, B=B, n_layers=args.layers or None))
        upd = next((v["ms"] for k, v in prof.items() if "add" in k or "sgd" in k), 0.0) / args.steps
        gemm = next((v for k, v in prof.items() if k.startswith("gemm_nt256")), None)
        return {"micro_batch": B, "micro_batches": n_mb, "ms_per_step": dt * 1e3, "tflops": fl / dt / 1e12,
                "sgd_update_ms": upd, "activation_peak_bytes": peak,
                "gemm_tflops": gemm["flops"] / (gemm["ms"] * 1e-3) / 1e12 if gemm else None}

    if args.accumulate_sweep:
        rows = [measure_accumulate(B, max(1, args.global_batch // B)) for B in [int(v) for v in args.accumulate_sweep.split(",")]]
        print(json.dumps({"metric": "training-step TFLOP/s vs micro-batch size at a fixed global batch "
                                    "(gradient accumulation + SGD update, no offload)", "unit": "TFLOP/s",
                          "workload": args.workload, "global_batch": args.global_batch, "steps": args.steps,
                          "warmup": args.warmup, "dtype": dtype, "data": "synthetic", "sweep": rows}))
        return

    link = link_rate(torch, dev)

    def sweep_rows(sizes):
        rows = []
        for Bs in sizes:
            _, modes, _, _ = measure(Bs, ["off", "budget"])
            rows.append({"micro_batch": Bs, "off_tflops": modes["off"]["tflops"], "off_ms": modes["off"]["ms_per_step"],
                         "off_activation_bytes": modes["off"]["arena_peak_bytes"],
                         "budget_tflops": modes["budget"]["tflops"], "budget_ms": modes["budget"]["ms_per_step"],
                         "budget_activation_bytes": modes["budget"]["arena_peak_bytes"],
                         "budget_offloaded_bytes": modes["budget"]["bytes_offloaded"],
                         "budget_exposed_io_pct": modes["budget"]["exposed_io_pct"]})
        return rows

    if args.sweep:
        rows = sweep_rows([int(v) for v in args.sweep.split(",")])
        print(json.dumps({"metric": "layer fwd+bwd TFLOP/s vs micro-batch (off / adaptive offload)", "unit": "TFLOP/s",
                          "workload": args.workload, "steps": args.steps, "warmup": args.warmup, "dtype": dtype,
                          "data": "synthetic", "link_measured_GBps": link, "sweep": rows}))
        return
    B = args.micro_batch or cfg["B"]
    layers, modes, prof, setup = measure(B, args.modes.split(","))
    L = len(layers)
    head = modes.get("budget") or modes["off"]

    copy_TBps = hbm_copy_rate(torch, dev)
    roof = None
    if prof:
        for k in prof:    # each class against its own bound: matrix-core peak, or the measured device-copy rate
            if k["flops"] > 0:
                k["TFLOPs"] = k["flops"] / (k["ms"] * 1e-3) / 1e12
                k["frac_of_mfma_peak"] = k["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
            elif k["bytes"] > 0:
                k["TBps"] = k["bytes"] / (k["ms"] * 1e-3) / 1e12
                k["frac_of_hbm_peak"] = k["TBps"] / HBM_PEAK_TBPS
                k["frac_of_measured_copy"] = k["TBps"] / copy_TBps
            k["ms_per_step"] = k["ms"] / args.steps
        dom = max((p for p in prof if p["flops"] > 0), key=lambda p: p["ms"], default=None)
        if dom:
            ach = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
            gemms = [p for p in prof if p["name"].startswith("gemm_")]
            roof = {"kernel": dom["name"], "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": recorded_traffic(dom["name"], args.workload, B),
                    "launches": dom["launches"], "avg_launch_ms": dom["ms"] / dom["launches"],
                    "all_gemm_kernels_TFLOPs": sum(p["flops"] for p in gemms) / (sum(p["ms"] for p in gemms) * 1e-3) / 1e12}
    sweep = None
    if not args.no_sweep and args.workload == "gpt_8192" and not args.micro_batch and not args.layers:
        keep = args.steps, args.warmup
        args.steps, args.warmup = 2, 1
        sweep = sweep_rows([b for b in (1, 2, 4, 8) if b < B])
        args.steps, args.warmup = keep
        sweep.append({"micro_batch": B, "off_tflops": modes["off"]["tflops"], "off_ms": modes["off"]["ms_per_step"],
                      "off_activation_bytes": modes["off"]["arena_peak_bytes"],
                      **({"budget_tflops": modes["budget"]["tflops"], "budget_ms": modes["budget"]["ms_per_step"],
                          "budget_activation_bytes": modes["budget"]["arena_peak_bytes"],
                          "budget_offloaded_bytes": modes["budget"]["bytes_offloaded"],
                          "budget_exposed_io_pct": modes["budget"]["exposed_io_pct"]} if "budget" in modes else {})})
    cpu = None if args.no_cpu_baseline else cpu_baseline(cfg)
    out = {
        "metric": "layer fwd+bwd TFLOP/s (whole stack; offload on with the planner's amount: the exposed-I/O figure "
                  "holds for that amount, the offload-everything mode is reported beside it under modes.all)",
        "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "ms_per_step_median": head["ms_per_step_median"],
        "ms_per_step_min": head["ms_per_step_min"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s: %s x%d, H=%d A=%d F=%d S=%d micro-batch %d" % (
            args.workload, "+".join(a for a, _ in cfg["stack"]), L, cfg["H"], cfg["A"], cfg["F"], layers[-1].S, B)},
        "mfma_peak_frac": head["tflops"] / MFMA_BF16_PEAK_TFLOPS,
        "exposed_io_pct": head.get("exposed_io_pct"),
        "exposed_io_ms_per_step_by_events": head["exposed_load_wait_ms"] + head["exposed_store_wait_ms"],
        "activation_peak_vs_no_offload": head.get("arena_peak_vs_off"),
        "offload_GBps": modes["all"]["link_GBps"] if "all" in modes else head["link_GBps"],
        "offload_link_frac": (modes["all"]["link_GBps"] if "all" in modes else head["link_GBps"]) / (2 * HOST_LINK_PEAK_GBPS),
        "link_measured_GBps": link, "hbm_copy_measured_TBps": copy_TBps, "modes": modes, "kernels": prof,
        "roofline": roof, "micro_batch_sweep": sweep, "cpu_baseline": cpu, "setup_s": setup,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
