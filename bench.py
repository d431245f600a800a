#!/usr/bin/env python3
"""Benchmark of the streaming-rollout hot path on one MI355X.

A step is one sr_rollout: T frame updates of the whole batch, inputs already resident in HBM,
every frame's output-node state recorded.  Prints ONE JSON line: rollout frames/s
(= batch * T * steps / time), per-frame latency, the roofline position of the dominant kernel
(the MFMA convolution tiles: algorithmic FLOP of one launch / its average duration, from HIP events on
the library's stream around the timed rollouts) and the CPU oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload gtsrb_sr|cifar_sr|hires_sr|tiny_sr]
                    [--pattern streaming|sequential|hybrid] [--no-cpu-baseline]

Further workloads: the paper's own network shapes (App. A2) mnist_ff, mnist_s, mnist_sr, dsr0 .. dsr6,
gtsrb_dsr4.  Extra fields of the line: frame_latency_us (p50 / p99 over single sr_frame_step calls,
HIP events), response_frames (frame updates between an input frame and the first output that depends
on it: the smallest number of bridging edges on a path from an input to the output node, at least 1 --
Sec. 4: the streaming rollout responds after the shortest path) and response_us = response_frames *
the median latency of a single frame (frame_latency_us.p50: a frame that is not overlapped with its
neighbours, as the frames of a dependency-driven rollout are).
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

KERNEL_SOURCES = ["sr_kernels.hip", "sr_host.cpp", "sr_internal.h", "sr_graph.h"]


def recorded_traffic(workload, pattern):
    """HBM bytes per launch of the dominant kernel from the committed counter record (FETCH_SIZE and
    WRITE_SIZE, scaled by a plain copy of known size); None if the record is for another workload or
    the kernel sources have changed since the counters were taken."""
    import hashlib
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", f"hbm_traffic_sr_mfma_kernel_{workload}.json")))
        h = hashlib.sha256()
        for f in KERNEL_SOURCES:
            h.update(open(os.path.join(ROOT, "paper_1806_04965_amd", "csrc", f), "rb").read())
        if h.hexdigest() != rec["source_sha256"] or not rec["workload"].startswith(f"{workload} ({pattern}"):
            return None
        return rec["hbm_bytes_per_launch"]
    except Exception:
        return None


def response_frames(g):
    """Frame updates until the output node first depends on a new input frame: 0-1 shortest path over
    the bridging bits from any input node to the output node, at least one update."""
    n = len(g.nodes)
    INF = 1 << 30
    dist = [INF] * n
    for v in g.input_nodes():
        dist[v] = 0
    for _ in range(n):
        for e in g.edges:
            if dist[e.src] + int(e.bridge) < dist[e.dst]:
                dist[e.dst] = dist[e.src] + int(e.bridge)
    return max(1, dist[g.out_node])


PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
PEAK_FP32_VALU_TFLOPS = 157.3  # fp32 vector peak (the fp32 graph runs on plain ALUs)


def train_window_bench(args, g):
    """One step = one training window (Sec. 3 rollout window of size W; loss of App. A2): forward over
    W frames, loss, gradients of every weight and bias, through sr_window_gradients on the fp32 graph.
    The roofline is the fp32 vector one; the algorithmic work of a window is, per edge and frame, the
    forward contraction, the weight gradient and, where one is kept (not into an input node, not into
    frame 0), the state gradient."""
    import dataclasses
    import numpy as np
    import torch
    import workloads as W
    import paper_1806_04965_amd as sr
    Wn = args.train_window
    g = dataclasses.replace(g, dtype="f32", frames=Wn)
    B = g.batch
    w, b, x = W.make_case(g, seed=0, frames=Wn, bias_scale=0.1)
    labels_h = np.random.default_rng(1).integers(0, g.nodes[g.out_node].channels, B).astype(np.int32)
    opts = {0: 0} if args.no_hipgraph else {}
    for kv in args.option:
        k, v = kv.split("=")
        opts[int(k)] = int(v)
    dev = sr.SrGraph(g, options=opts or None)
    dev.set_parameters(w, b)
    ins = g.input_nodes()
    xin = [torch.from_numpy(x[v][:Wn + 1]).to("cuda").float().contiguous() for v in ins]
    labels = torch.from_numpy(labels_h).to("cuda")
    work = dev.work()
    res = None   # every step writes the same output tensors, as a training loop does
    for _ in range(max(1, args.warmup)):
        res = dev.window_gradients(xin, labels, Wn, into=res)
    dev.synchronize()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(dev.stream)
    for _ in range(args.steps):
        res = dev.window_gradients(xin, labels, Wn, into=res)
    ev1.record(dev.stream)
    dev.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    # algorithmic work of the window: per edge and frame the forward contraction and the weight gradient, and the
    # state gradient where one is kept (not into input nodes, not into frame 0)
    inputs_set = set(ins)
    flop = 0.0
    for e in g.edges:
        sn, dn = g.nodes[e.src], g.nodes[e.dst]
        if e.kind == "conv":
            macs = B * (dn.height // e.up) * (dn.width // e.up) * dn.channels * sn.channels * e.kh * e.kw
        elif e.kind == "dense":
            macs = B * dn.channels * sn.channels * sn.height * sn.width
        else:
            macs = B * dn.channels * sn.channels
        for i in range(1, Wn + 1):
            flop += 2.0 * macs * (2 + (1 if e.src not in inputs_set and i - int(e.bridge) >= 1 else 0))
    achieved = flop / (ev0.elapsed_time(ev1) / args.steps * 1e-3) / 1e12
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import training as otr
        Bs = min(B, 4)          # bounded sample: the same window on a few samples of the batch
        gs = dataclasses.replace(g, batch=Bs)
        c0 = time.perf_counter()
        otr.window_gradients(gs, w, b, {v: x[v][:Wn + 1, :Bs] for v in x}, labels_h[:Bs], Wn)
        cdt = time.perf_counter() - c0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
        except Exception:
            cores = os.cpu_count()
        cpu = {"value": round(Bs * Wn / cdt, 3), "unit": "frames/s", "cores": int(cores), "kind": "oracle",
               "sample": f"one window of {Wn} frames on {Bs} of the {B} samples (float64), {cdt:.1f} s"}
    line = {
        "metric": "training-window frames/sec (batch x window frames / s; forward + loss + all gradients)",
        "value": round(B * Wn * args.steps / dt, 1), "unit": "frames/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload} ({args.pattern} rollout), training window W={Wn}", "batch": B,
                   "nodes": len(g.nodes), "edges": len(g.edges)},
        "loss": round(float(res[0].cpu()[0]), 6),
        "roofline": {"bound": "alu", "achieved": round(achieved, 4), "peak": PEAK_FP32_VALU_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / PEAK_FP32_VALU_TFLOPS, 5), "traffic": None,
                     "kernel": "sr_window_gradients (all kernels of a window)", "flop_per_step": flop},
        "cpu_baseline": cpu,
    }
    dev.close()
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gtsrb_sr")
    ap.add_argument("--pattern", default="streaming")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-hipgraph", action="store_true")
    ap.add_argument("--tile-kernel", type=int, default=0, help="1: 4-wave tile kernel, 2: 8-wave tile kernel, 0: library default")
    ap.add_argument("--option", action="append", default=[], metavar="KEY=VALUE",
                    help="sr_graph_configure option by number, e.g. 5=0 (dependency-driven execution off)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 512 MiB device copy (a kernel of known HBM traffic, for scaling "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--train-window", type=int, default=0, metavar="W",
                    help="time sr_window_gradients on a rollout window of W frames of the workload (as an fp32 "
                         "graph) instead of the rollout; a step is then one window: forward, loss, all gradients")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path would shard by batch or by node partition)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as W
    import paper_1806_04965_amd as sr

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    g = {**W.BENCH_CONFIGS, **W.PAPER_CONFIGS}[args.workload]()
    bits = {"streaming": W.streaming_pattern, "sequential": W.sequential_pattern,
            "hybrid": W.hybrid_pattern}[args.pattern](g)
    g = g.with_pattern(bits)
    if args.train_window > 0:
        return train_window_bench(args, g)
    T, B = g.frames, g.batch
    w, b, x = W.make_case(g, seed=0)

    opts = {}
    if args.no_hipgraph:
        opts[0] = 0
    if args.tile_kernel:
        opts[4] = args.tile_kernel
    for kv in args.option:
        k, v = kv.split("=")
        opts[int(k)] = int(v)
    dev = sr.SrGraph(g, options=opts or None)
    dev.set_parameters(w, b)
    tdt = torch.bfloat16 if g.dtype == "bf16" else torch.float32
    ins = g.input_nodes()
    xin = [torch.from_numpy(x[v]).to("cuda").to(tdt).contiguous() for v in ins]
    n_out = g.nodes[g.out_node]
    out = torch.empty((T, B, n_out.height, n_out.width, n_out.channels), dtype=tdt, device="cuda")
    info = dev.info()
    work = dev.work()

    if args.copy_calibration:
        a = torch.empty(128 * 1024 * 1024, dtype=torch.float32, device="cuda").normal_()
        c = torch.empty_like(a)
        c.copy_(a)            # reads 512 MiB, writes 512 MiB
        torch.cuda.synchronize()
        del a, c
    for _ in range(args.warmup):
        dev.rollout(xin, T, g.out_node, out)
    dev.synchronize()
    torch.cuda.synchronize()
    # the timed region, also bracketed by HIP events on the stream the kernels are launched on
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(dev.stream)
    for _ in range(args.steps):
        dev.rollout(xin, T, g.out_node, out)
    ev1.record(dev.stream)
    dev.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    frames_per_s = B * T * args.steps / dt
    event_ms_per_step = ev0.elapsed_time(ev1) / args.steps

    # dominant kernel, timed live with HIP events on the library's stream (plain launches)
    dev.reset([xi[0] for xi in xin])
    for t in range(1, min(T, 4) + 1):
        dev.frame_step([xi[t] for xi in xin])
    dev.synchronize()
    kind_ms = {}
    frame_ms = []
    reps = max(min(T, 12), 32)
    for r in range(reps):
        launches = dev.frame_step_timed([xi[1 + (r % T)] for xi in xin])
        frame_ms.append(sum(ms for _, ms in launches))
        for kind, ms in launches:
            kind_ms.setdefault(kind, []).append(ms)
    conv_flops = 0
    for e in g.edges:
        if e.kind == "conv":
            s, d = g.nodes[e.src], g.nodes[e.dst]
            conv_flops += 2 * B * (d.height // e.up) * (d.width // e.up) * d.channels * s.channels * e.kh * e.kw
    ideal_bytes = 0
    for n in g.nodes:
        ideal_bytes += 2 * B * n.height * n.width * n.channels * (2 if g.dtype == "bf16" else 4)
    for wi in w:
        ideal_bytes += wi.size * (2 if g.dtype == "bf16" else 4)
    if g.dtype == "bf16" and 1 in kind_ms:
        # Dominant kernel: the convolution tiles.  Its average launch duration is taken from the timed
        # region itself: HIP events on the library's stream around the replayed rollouts, divided by the
        # tile launches they contain (one per update step of a frame; the whole frame's time is charged to
        # them, so launches x duration = the timed time by construction).  The duration of the same
        # launches issued one by one between events is reported next to it (launch_ms_single).
        tile_launches_per_frame = len(kind_ms[1]) / reps
        launch_ms = event_ms_per_step / (T * tile_launches_per_frame)
        flop_per_launch = conv_flops / tile_launches_per_frame
        achieved = flop_per_launch / (launch_ms * 1e-3) / 1e12
        traffic = recorded_traffic(args.workload, args.pattern)
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                    "traffic": traffic,
                    "traffic_ratio": round(traffic / (ideal_bytes / tile_launches_per_frame), 2) if traffic else None,
                    "ideal_bytes_per_launch": int(ideal_bytes / tile_launches_per_frame),
                    "kernel": "sr_mfma8_kernel" if dev.tile_kernel() == 2 else "sr_mfma_kernel",
                    "launch_ms": round(launch_ms, 4),
                    "launch_ms_single": round(float(np.mean(kind_ms[1])), 4),
                    "launches_per_frame": tile_launches_per_frame, "flop_per_launch": flop_per_launch,
                    # bytes per frame by class as the planner counts them (no cache modelled)
                    "traffic_model": {k: int(v) for k, v in dev.traffic_model().items()}}
    else:
        d_ms = float(np.mean(kind_ms.get(2, [float("nan")])))
        achieved = work["flops_per_frame"] / (d_ms * 1e-3) / 1e12
        roofline = {"bound": "alu", "achieved": round(achieved, 5), "peak": PEAK_FP32_VALU_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_FP32_VALU_TFLOPS, 6), "traffic": None,
                    "kernel": "sr_direct_kernel", "launch_ms": round(d_ms, 4)}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import rollout as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
        except Exception:
            cores = os.cpu_count()
        mode = "bf16" if g.dtype == "bf16" else "f64"
        r = orc.Rollout(g, w, b, mode)
        r.reset({v: x[v][0] for v in ins})
        c0 = time.perf_counter()
        sample_frames = 0
        while sample_frames < 2 or (time.perf_counter() - c0 < 10.0 and sample_frames < 64):
            r.step({v: x[v][1 + sample_frames % T] for v in ins})   # bounded sample: about 10 s of CPU work
            sample_frames += 1
        cdt = time.perf_counter() - c0
        cpu = {"value": round(B * sample_frames / cdt, 3), "unit": "frames/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{sample_frames} frame updates of the full batch ({mode} mode), {cdt:.1f} s",
               "ms_per_frame": round(cdt / sample_frames * 1e3, 1)}

    line = {
        "metric": "rollout frames/sec (batch x frames / s)",
        "value": round(frames_per_s, 1),
        "unit": "frames/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": g.dtype,
        "data": "synthetic",
        "config": {"workload": f"{args.workload} ({args.pattern} rollout)", "batch": B, "frames_per_step": T,
                   "nodes": len(g.nodes), "edges": len(g.edges), "inference_factor": info["inference_factor"],
                   "launches_per_frame": info["launches_per_frame"], "hipgraph": not args.no_hipgraph},
        "us_per_frame": round(ms_per_step * 1e3 / T, 2),
        "frame_latency_us": {"p50": round(float(np.percentile(frame_ms, 50)) * 1e3, 2),
                             "p99": round(float(np.percentile(frame_ms, 99)) * 1e3, 2), "frames": len(frame_ms),
                             "how": "single sr_frame_step calls, plain launches, HIP events around every launch"},
        "response_frames": response_frames(g),
        "response_us": round(response_frames(g) * float(np.percentile(frame_ms, 50)) * 1e3, 2),
        "gflop_per_frame": round(work["flops_per_frame"] / 1e9, 3),
        "frame_tflops": round(work["flops_per_frame"] * T / (ms_per_step * 1e-3) / 1e12, 2),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    dev.close()
    print(json.dumps(line))


if __name__ == "__main__":
    main()
