#!/usr/bin/env python3
"""Benchmark: ResNet-50-shaped inference forward, batch 64, bf16 storage / fp32 accumulate, one MI355X.

A "step" is one pass of the whole hot path (every fused conv, the stem pool, the global average
pool and the linear layer: 56 layers, fewer launches where the plan fuses layers -- the JSON line
says how many) over one resident batch of synthetic images.  Prints ONE JSON line with images/s, the
roofline of the dominant kernel (the fused convolution launches) from durations measured inside whole
passes, the machine's measured ceilings, the CPU checker timed on a bounded sample of the same workload,
and the error of the timed network's output against that checker run.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "conv_resnet50_bs64_hbm_traffic.md")


def measured_traffic():
    """HBM bytes per convolution launch of the ResNet-50-shaped batch-64 pass, read from the committed summary of the
    FETCH_SIZE / WRITE_SIZE counter runs (its line "per launch <x> MB"); None when the summary is not there."""
    import re
    try:
        with open(TRAFFIC_SUMMARY) as f:
            m = re.search(r"convolution launches of one pass:.*?per launch ([0-9.]+) MB", f.read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def layer_shapes(layers, in_shape, out_size):
    """Logical NCHW input/output shape of every layer (bookkeeping for the algorithmic work counts)."""
    shapes, ins = [], []
    for i, l in enumerate(layers):
        s = l.get("src", -1)
        x = in_shape if (i == 0 and s == -1) else shapes[i - 1 if s == -1 else s]
        if l["kind"] == "conv":
            o = (x[0], l["cout"], out_size(x[2], l["kh"], l["sh"], l["ph"]), out_size(x[3], l["kw"], l["sw"], l["pw"]))
            if l.get("pool"):      # a pool fused behind the convolution: the stored tensor is the pooled one
                p = l["pool"]
                o = (o[0], o[1], out_size(o[2], p["kh"], p["sh"], p["ph"]), out_size(o[3], p["kw"], p["sw"], p["pw"]))
        elif l["kind"] == "pool":
            p = l["pool"]
            o = (x[0], x[1], out_size(x[2], p["kh"], p["sh"], p["ph"]), out_size(x[3], p["kw"], p["sw"], p["pw"]))
        elif l["kind"] == "gap":
            o = (x[0], x[1], 1, 1)
        elif l["kind"] == "concat":
            o = (x[0], x[1] + shapes[l["res"]][1], x[2], x[3])
        else:
            o = (x[0], l["out"], 1, 1)
        ins.append(x)
        shapes.append(o)
    return ins, shapes


def algorithmic_work(l, x, y, esize):
    """(flops, bytes) the layer must perform/move: read input, weights and residual once, write output once."""
    numel = lambda s: s[0] * s[1] * s[2] * s[3]  # noqa: E731
    if l["kind"] == "conv" and l.get("dw"):     # one filter per channel: no reduction over channels
        taps = l["kh"] * l["kw"]
        return 2.0 * numel(y) * taps, esize * (numel(x) + taps * y[1] + numel(y) * (2 if l["res"] >= 0 else 1)) + 8 * y[1]
    if l["kind"] == "conv":
        k = l["kh"] * l["kw"] * x[1]
        ho, wo = (x[2] + 2 * l["ph"] - l["kh"]) // l["sh"] + 1, (x[3] + 2 * l["pw"] - l["kw"]) // l["sw"] + 1    # before any fused pool
        flops = 2.0 * y[0] * ho * wo * y[1] * k
        byts = esize * (numel(x) + k * y[1] + numel(y) * (2 if l["res"] >= 0 else 1)) + 8 * y[1]
        return flops, byts
    if l["kind"] == "linear":
        return 2.0 * x[0] * x[1] * y[1], esize * (numel(x) + x[1] * y[1] + numel(y)) + 4 * y[1]
    return 0.0, esize * (numel(x) + numel(y))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload: 3 = ResNet-50-shaped bs64 (default), 2 = ResNet-18-shaped bs32, 5 = 3-layer MLP with 8192 features bs64, 6 = depthwise-separable chain bs64, 7 = SqueezeNet-shaped bs64 (channel concatenations), 8 = DenseNet-121-shaped bs64 (pre-activation convolutions on dense chains)")
    ap.add_argument("--batch", type=int, default=None)
    ap.add_argument("--layer-reps", type=int, default=20, help="event-timed repetitions per layer for the roofline")
    ap.add_argument("--pass-reps", type=int, default=20, help="whole passes with an event in front of every launch (in-pass durations for the roofline)")
    ap.add_argument("--cpu-sample", type=int, default=32, help="images the CPU checker is timed on (0 = skip); 32 is 10-15 s of CPU work")
    ap.add_argument("--layers", action="store_true", help="also print a per-layer table to stderr")
    ap.add_argument("--graph", action="store_true", help="time HIP-graph replays of the pass instead of plain launches")
    ap.add_argument("--tune-reps", type=int, default=10,
                    help="launches per candidate in the plan-time per-layer kernel/tile auto-tune (0 = shape heuristic only)")
    ap.add_argument("--save-plan", default=None, help="write the auto-tuned per-layer tile ids to this JSON file")
    ap.add_argument("--load-plan", default=None, help="use the per-layer tile ids of an earlier --save-plan run instead of tuning "
                                                      "(profiler runs, whose timing would mislead the tuner)")
    ap.add_argument("--train-steps", type=int, default=10,
                    help="timed steps of the ResNet-18-shaped bs32 training step reported beside the headline (0 = skip)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no multi-GPU sharding or collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2003_10688_amd import sol
    from paper_2003_10688_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    sol.lib()
    wk = wl.config(a.config, batch=a.batch)
    dt = sol.BF16 if wk.bf16 else sol.F32
    esize = 2 if wk.bf16 else 4
    net = sol.Network(wk.layers, wk.in_shape, dt)
    net.set_params(wk.params)
    x = sol.to_device_nhwc(wk.x, dt)
    stream = torch.cuda.current_stream()
    torch.cuda.synchronize()
    # plan time (not timed): per-layer kernel / tile selection by a short timed sweep, the "very short auto-tuning" of
    # the paper's optimize step (Sec. III-A); the plan is then fixed for every timed pass
    t0 = time.perf_counter()
    if a.load_plan:
        with open(a.load_plan) as f:
            tuned = {(k if k[-1] in "bx" else int(k)): v for k, v in json.load(f).items()}
        net.set_tiles(tuned)
    else:
        tuned = net.autotune(x, reps=a.tune_reps, stream=stream) if a.tune_reps > 0 else {}
    tune_s = time.perf_counter() - t0
    if a.save_plan:
        with open(a.save_plan, "w") as f:
            json.dump(tuned, f)

    # ---- whole-step throughput -------------------------------------------------------------------
    # One step = one forward pass: plain launches on one stream.  --graph replays the same pass from a HIP
    # graph recorded through the library instead (sol_network_graph_create); measured, it makes no difference
    # here -- the step is bound by the kernels and the drain between dependent launches, not by submission.
    def timed(step_fn, st):
        for _ in range(a.warmup):
            step_fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(st)
        for _ in range(a.steps):
            step_fn()
        e1.record(st)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / a.steps, e0.elapsed_time(e1) / a.steps

    eager_ms, eager_ev_ms = timed(lambda: net.forward(x, stream), stream)
    if not a.graph:
        wall_ms, ev_ms = eager_ms, eager_ev_ms
    else:
        side = torch.cuda.Stream()
        wall_ms, ev_ms = timed(net.graph(x, side), side)
    batch = wk.in_shape[0]
    imgs_per_s = batch / (wall_ms * 1e-3)

    # ---- per-layer event timing (same stream) for the roofline of the dominant kernel ---------------
    ins, outs = layer_shapes(wk.layers, wk.in_shape, sol.sol_out_size)
    rows = []
    into = [net.fused_into(i) for i in range(len(wk.layers))]   # the plan runs a stem convolution and the max pool behind it as one launch
    for i, l in enumerate(wk.layers):
        if into[i] != i or (l["kind"] == "concat" and net.concat_in_place(i) == 2):   # nothing is launched for this layer
            rows.append({"i": i, "kind": "fused", "us": 0.0, "flops": 0, "bytes": 0})
            continue
        net.run_layer(i, x, stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(a.layer_reps):
            net.run_layer(i, x, stream)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / a.layer_reps
        absorbs = i + 1 < len(into) and into[i + 1] == i and wk.layers[i + 1]["kind"] == "pool"
        fl, by = algorithmic_work(l, ins[i], outs[i], esize)
        numel = lambda t: t[0] * t[1] * t[2] * t[3]  # noqa: E731
        if absorbs:   # a fused stem pair stores only the pooled tensor
            by += esize * (numel(outs[i + 1]) - numel(outs[i]))
        if i + 1 < len(into) and into[i + 1] == i and wk.layers[i + 1]["kind"] == "conv":   # an expand-reduce pair: the second
            fj, bj = algorithmic_work(wk.layers[i + 1], ins[i + 1], outs[i + 1], esize)         # convolution's work, minus the read of its input
            fl += fj
            by += bj - esize * numel(ins[i + 1])
        for j in range(i):   # layers computed inside this launch (a projection shortcut, the first two convolutions of a
            if into[j] == i:  # bottleneck): their work, minus the write and the re-read of their outputs
                fj, bj = algorithmic_work(wk.layers[j], ins[j], outs[j], esize)
                fl += fj
                by += bj - 2 * esize * numel(outs[j])
                sj = wk.layers[j].get("src", -1)
                if l.get("res", -1) >= 0 and (j - 1 if sj == -1 else sj) == l["res"]:
                    by -= esize * numel(outs[l["res"]])      # ... and the shortcut is the block input, which is read once
        rows.append({"i": i, "kind": "dwconv" if l.get("dw") else l["kind"], "us": us, "flops": fl, "bytes": by})
    # ---- the same launches timed inside whole passes (cold weights, inputs as the producer left them): an event in
    # front of every launch of a pass.  A long register-only kernel goes first so that the host has queued the whole
    # pass before its first launch starts (an event otherwise also measures the wait for the next submission).
    launched = [r for r in rows if r["kind"] != "fused"]
    sink = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    acc_us = [0.0] * len(launched)
    for _ in range(a.pass_reps):
        sol.sol_debug_probe_mfma(40000, 256, sink, stream)           # about 3 ms
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(launched) + 1)]
        for k, r in enumerate(launched):
            evs[k].record(stream)
            net.run_layer(r["i"], x, stream)
        evs[-1].record(stream)
        torch.cuda.synchronize()
        for k in range(len(launched)):
            acc_us[k] += evs[k].elapsed_time(evs[k + 1]) * 1e3
    for k, r in enumerate(launched):
        r["us_pass"] = acc_us[k] / max(a.pass_reps, 1) if a.pass_reps > 0 else r["us"]
    # An event between two launches costs about 3 us that the timed passes do not pay (it keeps the next launch from
    # being set up under the tail of the previous one), so the instrumented pass is longer than the timed one.  The
    # per-launch durations are scaled by one common factor so that they add up to the timed pass: the timed region
    # itself is what the roofline figures divide by.
    marker_scale = (eager_ev_ms * 1e3) / max(sum(r["us_pass"] for r in launched), 1e-9) if a.pass_reps > 0 else 1.0
    marker_scale = min(marker_scale, 1.0)
    for r in launched:
        r["us_pass_raw"] = r["us_pass"]
        r["us_pass"] *= marker_scale
    for r in rows:
        r.setdefault("us_pass", 0.0)

    # ---- measured ceilings of this machine: a plain 100 MB copy and a register-resident MFMA loop
    cbuf = torch.empty(2 * 100 * (1 << 20), dtype=torch.uint8, device="cuda:0")
    src_b, dst_b = cbuf[:100 << 20], cbuf[100 << 20:]

    def ev_time(fn, reps):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / reps
    copy_s = ev_time(lambda: sol.sol_debug_probe_copy(dst_b, src_b, stream), 20)
    flop_box = [0.0]

    def mfma_once():
        flop_box[0] = sol.sol_debug_probe_mfma(4000, 1024, sink, stream)
    mfma_s = ev_time(mfma_once, 5)
    measured_peak = {"hbm_copy_gbs": round(2 * (100 << 20) / copy_s / 1e9, 1), "hbm_copy_mb": 104.9,
                     "mfma_bf16_tflops": round(flop_box[0] / mfma_s / 1e12, 1),
                     "source": "sol_debug_probe_copy / sol_debug_probe_mfma, this run"}
    del cbuf

    conv = [r for r in rows if r["kind"] == "conv"]
    mem = [r for r in rows if r["kind"] in ("pool", "gap")]
    dwr = [r for r in rows if r["kind"] == "dwconv"]
    if conv:
        conv_us = sum(r["us_pass"] for r in conv)           # durations inside whole passes
        conv_us_hot = sum(r["us"] for r in conv)            # the same launches repeated back to back on hot buffers
        conv_fl = sum(r["flops"] for r in conv)
        conv_by = sum(r["bytes"] for r in conv)
        ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
        mf = [r for r in conv if r["flops"] / r["bytes"] >= ridge]
        hb = [r for r in conv if r["flops"] / r["bytes"] < ridge]
        tfl = conv_fl / (conv_us * 1e-6) / 1e12
        grp = lambda rs, key, peak, scale: {"n": len(rs),  # noqa: E731
                                            key: round(sum(r["flops" if key == "tflops" else "bytes"] for r in rs) / max(sum(r["us_pass"] for r in rs), 1e-9) / scale, 2),
                                            "frac": round(sum(r["flops" if key == "tflops" else "bytes"] for r in rs) / max(sum(r["us_pass"] for r in rs), 1e-9) / scale / peak, 4)}
        traffic_mb = measured_traffic() if a.config == 3 and wk.in_shape[0] == 64 else None
        roofline = {
            "bound": "mfma", "kernel": "fused convolution kernels (conv_dma / conv_halo / conv_gemm8 / conv_stem_pool / conv_pair / conv_block / conv_xr)", "launches_per_step": len(conv),
            "achieved": round(tfl, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(tfl / PEAK_BF16_TFLOPS, 4),
            "avg_launch_us": round(conv_us / len(conv), 2), "algorithmic_gflop_per_launch": round(conv_fl / len(conv) / 1e9, 3),
            "timing": f"HIP events around every launch inside {a.pass_reps} whole passes, scaled by {marker_scale:.3f} so that the launches add up to the timed pass (the events between launches cost time the timed passes do not pay)",
            "frac_hot_repeats": round(conv_fl / (conv_us_hot * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "measured_peak": measured_peak,
            "traffic": ({"hbm_mb_per_launch": traffic_mb, "algorithmic_mb_per_launch": round(conv_by / len(conv) / 1e6, 1),
                         "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary read from profiles/conv_resnet50_bs64_hbm_traffic.md (a run of its own, same workload)"}
                        if traffic_mb is not None else None),
            "mfma_bound_layers": grp(mf, "tflops", PEAK_BF16_TFLOPS, 1e6),
            "hbm_bound_layers": grp(hb, "gbs", PEAK_HBM_GBS, 1e3),
            "pool_gap_kernels": grp(mem, "gbs", PEAK_HBM_GBS, 1e3),
            "depthwise_kernels": grp(dwr, "gbs", PEAK_HBM_GBS, 1e3) if dwr else None,
            "conv_algorithmic_gb_per_step": round(conv_by / 1e9, 3),
            "sum_layer_us": round(sum(r["us_pass"] for r in rows), 1),
        }
    else:   # no convolution (the MLP workload): the linear kernel streams its weights once, bound by HBM
        lin = [r for r in rows if r["kind"] == "linear"]
        lin_us, lin_by = sum(r["us_pass"] for r in lin), sum(r["bytes"] for r in lin)
        gbs = lin_by / max(lin_us, 1e-9) / 1e3
        roofline = {"bound": "hbm", "kernel": "linear layers (linear_kernel, or the conv_gemm8 weight-streaming tile for large weight matrices)", "launches_per_step": len(lin), "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(gbs / PEAK_HBM_GBS, 4), "avg_launch_us": round(lin_us / max(len(lin), 1), 2),
                    "algorithmic_mb_per_launch": round(lin_by / max(len(lin), 1) / 1e6, 2), "traffic": None, "measured_peak": measured_peak,
                    "tflops": round(sum(r["flops"] for r in lin) / max(lin_us, 1e-9) / 1e6, 2), "sum_layer_us": round(sum(r["us_pass"] for r in rows), 1)}
    if a.layers:
        for r, xi, yo in zip(rows, ins, outs):
            if r["kind"] == "fused":
                print(f"L{r['i']:02d} " + ("(both inputs written in place by their producers)" if wk.layers[r['i']]["kind"] == "concat"
                                           else f"(computed by the launch of L{into[r['i']]:02d})"), file=sys.stderr)
                continue
            ai = r["flops"] / r["bytes"]
            up = max(r["us_pass"], 1e-9)
            t_roof = max(r["flops"] / (PEAK_BF16_TFLOPS * 1e6), r["bytes"] / (PEAK_HBM_GBS * 1e3))      # us at min(MFMA, HBM) roof
            print(f"L{r['i']:02d} {r['kind']:6s} in{xi} out{yo} in-pass {up:7.1f} us (hot {r['us']:6.1f})  {r['flops'] / up / 1e6:7.1f} TFLOP/s"
                  f"  {r['bytes'] / up / 1e3:7.1f} GB/s  AI {ai:5.0f}  {'mfma' if r['flops'] / r['bytes'] >= PEAK_BF16_TFLOPS / PEAK_HBM_GBS * 1e3 else 'hbm '}"
                  f" roof {t_roof:5.1f} us = {100 * t_roof / up:4.1f} %", file=sys.stderr)

    # ---- CPU checker on a bounded sample of the same workload ------------------------------------------
    cpu, parity = None, None
    if a.cpu_sample > 0:
        import oracle

        import numpy as np

        n = min(a.cpu_sample, batch)
        t0 = time.perf_counter()
        ref = oracle.network_forward(wk.layers, wk.params, wk.x[:n], bf16=wk.bf16)
        dt_s = time.perf_counter() - t0
        cpu = {"value": round(n / dt_s, 3), "unit": "images/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": f"first {n} images of the batch, full network, one pass, {dt_s:.1f} s"}
        # the timed plan (tuned tiles, fused pairs, reused buffers) against that run: images of a batch are independent
        got = sol.to_host_nchw(net.forward(x, stream))[:n].astype(np.float64).reshape(ref.shape)
        torch.cuda.synchronize()
        floor = max(float(np.sqrt(np.mean(ref * ref))), 1e-30)
        tol = 2e-2 if wk.bf16 else 1e-4
        parity = {"n_images": n, "normwise": float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30)),
                  "elementwise_max": float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor))), "tolerance": tol,
                  "gate": "normwise" if wk.bf16 else "elementwise_max",
                  "what": "output of the timed network (free running, tuned plan) vs the CPU checker on the same images"}
        parity["ok"] = bool(parity[parity["gate"]] <= tol)
        parity["normwise"], parity["elementwise_max"] = float(f"{parity['normwise']:.3e}"), float(f"{parity['elementwise_max']:.3e}")

    # ---- training step (second workload, reported beside the headline number) -------------------------
    training = None
    if a.train_steps > 0:
        del net
        tw = wl.config(4)
        tnet = sol.Network(tw.layers, tw.in_shape, sol.BF16, flags=sol.NET_TRAINING)
        tnet.set_params(tw.params)
        tx = sol.to_device_nhwc(tw.x, sol.BF16)
        lab = torch.from_numpy(tw.labels).to("cuda:0")
        if a.tune_reps > 0:      # plan time, not timed: per-layer tiles for the forward and data-gradient convolutions
            tnet.autotune(tx, reps=a.tune_reps, stream=stream)

        def train_step():
            tnet.forward(tx, stream)
            tnet.backward(tx, lab, stream)
            tnet.sgd_step(0.1, 0.9, stream)                      # the workload's optimiser setting

        for _ in range(3):
            train_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.train_steps):
            train_step()
        torch.cuda.synchronize()
        tms = (time.perf_counter() - t0) * 1e3 / a.train_steps
        # algorithmic contraction work of a step: forward + weight gradient of every convolution / linear layer, data
        # gradient of all but the first (its input needs none)
        tin, tout = layer_shapes(tw.layers, tw.in_shape, sol.sol_out_size)
        tfl, first = 0.0, True
        for l, xi, yo in zip(tw.layers, tin, tout):
            f, _ = algorithmic_work(l, xi, yo, 2)
            if f > 0:
                tfl += f * (2 if first else 3)
                first = False
        training = {"workload": f"{tw.name} batch {tw.in_shape[0]} input 3x224x224: forward (batch-stat BN) + loss + backward + SGD lr 0.1 momentum 0.9",
                    "images_per_s": round(tw.in_shape[0] / (tms * 1e-3), 1), "ms_per_step": round(tms, 3), "steps": a.train_steps,
                    "loss_after": round(float(tnet.loss[0].cpu()), 4),
                    "roofline": {"bound": "mfma", "achieved": round(tfl / (tms * 1e-3) / 1e12, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                 "frac": round(tfl / (tms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4), "algorithmic_gflop_per_step": round(tfl / 1e9, 1),
                                 "what": "contraction FLOPs of the step (forward, data and weight gradients) over the whole step time, BN / loss / update launches included"}}

    out = {
        "metric": "images/sec ResNet-50-shaped fwd bs64 on 1 GPU" if a.config == 3 and batch == 64 else f"images/sec {wk.name} fwd bs{batch} on 1 GPU",
        "value": round(imgs_per_s, 1), "unit": "images/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(wall_ms, 4), "event_ms_per_step": round(ev_ms, 4),
        "submission": "HIP graph replay" if a.graph else "eager launches", "eager_ms_per_step": round(eager_ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if wk.bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{wk.name} batch {batch} input {wk.in_shape[1]}x{wk.in_shape[2]}x{wk.in_shape[3]} (seeded synthetic, He-normal weights)",
                   "launches_per_step": sum(1 for r in rows if r["kind"] != "fused"), "autotuned_layers": sum(1 for k in tuned if str(k)[-1] not in "bx"), "fused_bottlenecks": sum(1 for k, v in tuned.items() if str(k).endswith("b") and v),
                   "fused_expand_reduce_pairs": sum(1 for k, v in tuned.items() if str(k).endswith("x") and v), "autotune_seconds": round(tune_s, 2)},
        "roofline": roofline, "cpu_baseline": cpu, "parity": parity, "training_step": training,
    }
    print(json.dumps(out))
    if parity is not None and not parity["ok"]:
        print(f"bench.py: the timed network's output is outside the tolerance: {parity}", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
