"""Benchmark of the fused-operator hot path on one MI355X.

Default workload (the headline metric): one step = one pass of the whole path
(stem frame copy, 20 fused conv2d groups, max-pool, global average pool, dense
head) over one batch of the ResNet-18-shaped graph: batch 64, bf16 activations
and weights, fp32 accumulation, seeded synthetic data, random-init weights with
batch-norm folded in.  Prints ONE JSON line.  Paper figures for this metric:
none (the paper reports no measurement).

Other workloads (`--workload`), same JSON shape, for the remaining
configurations and the HBM-bound groups:
  eltwise   relu(bias_add(x) + r) on 256x64x112x112 bf16 (1.2 GB moved per step)
  eltwise32 the same in f32 on 128x64x112x112
  gates     stand-alone LSTM gate group on z 16384x4096 f32
  lstm      unrolled LSTM, batch 64, 1024 -> 1024, 128 steps, bf16 weights
  mlp       MLP 784 -> 128 -> 10, f32, batch 32
  lenet     the LeNet-shaped example graph (conv5x5, tanh, maxpool2, conv5x5, tanh, maxpool2, dense 500, tanh, dense 10), f32, batch 64
  conv      single fused conv2d group 64 -> 64, 56x56, f32, batch 1
  resnet18_f32_b1  the ResNet-18-shaped graph in f32 at batch 1
  copy      y = -x on 24 Mi f32 elements: a plain copy kernel of known size
            (100.7 MB read, 100.7 MB written, ordinary loads and stores), the
            yardstick for the HBM byte counters
  grads     the gradient operators of dense / conv2d at the benchmark graph's shapes
  mfma_peak a chain of bf16 MFMAs on register operands on every SIMD: what the
            matrix pipes deliver here, next to the quoted 2.5 PFLOP/s
The default line also carries that calibration ("peaks") and the HBM-bound groups
on tensors far larger than the last-level cache ("hbm_bound_groups").
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3        # MI355X fp32 (MFMA and vector)
PEAK_HBM_GBS = 8000.0


def cpu_baseline_resnet(n_images: int):
    """The oracle, as it stands, on `n_images` images of the same workload."""
    import workloads as W
    import oracle as O
    from oracle import graph as OG
    from helpers import fold_resnet_oracle
    spec, raw, bn = W.resnet18(batch=n_images, dtype="bf16")
    data = fold_resnet_oracle(raw, bn, "bf16")
    t0 = time.perf_counter()
    OG.run(spec, data)
    dt = time.perf_counter() - t0
    return {"value": n_images / dt, "unit": "images/s", "cores": O.num_threads(), "kind": "oracle",
            "sample": f"{n_images} images of the batch-64 bf16 ResNet-18-shaped graph, one oracle run, {dt:.1f} s"}


def cpu_baseline_graph(spec, data, unit_count: float, unit: str, what: str):
    import oracle as O
    from oracle import graph as OG
    t0 = time.perf_counter()
    OG.run(spec, data)
    dt = time.perf_counter() - t0
    return {"value": unit_count / dt, "unit": unit, "cores": O.num_threads(), "kind": "oracle", "sample": f"{what}, one oracle run, {dt:.1f} s"}


GRAPH = False     # --graph: time replays of a HIP graph holding one step instead of eager launches


TIMING = {}       # distribution of the last time_steps call (per-step milliseconds over chunks of the timed region)


def time_steps(run, steps, warmup, graph=None):
    """W untimed steps, then exactly `steps` steps between two events on the launch stream, bracketed by device
    synchronisation on both sides.  Returns the mean milliseconds per step of that region.  Events every few steps
    inside the region (at most 20 chunks, so that their own cost stays far below a percent) give median, minimum
    and 90th percentile of the per-step time over the chunks, left in TIMING."""
    import torch
    if GRAPH if graph is None else graph:
        run()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run()
        run = g.replay
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    chunk = max(1, -(-steps // 20))
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(-(-steps // chunk) + 1)]
    t0 = time.perf_counter()
    marks[0].record(stream)
    for i in range(steps):
        run()
        if (i + 1) % chunk == 0 or i + 1 == steps:
            marks[(i + chunk) // chunk].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = marks[0].elapsed_time(marks[-1]) / steps
    per = []
    for j in range(len(marks) - 1):
        n = min(chunk, steps - j * chunk)
        per.append(marks[j].elapsed_time(marks[j + 1]) / n)
    per.sort()
    TIMING.clear()
    TIMING.update({"ms_per_step_median": per[len(per) // 2], "ms_per_step_min": per[0], "ms_per_step_p90": per[min(len(per) - 1, int(0.9 * len(per)))],
                   "chunks": len(per), "steps_per_chunk": chunk})
    return max(ms, wall * 1e3 / steps)          # never report less than the host saw


def kernel_table(session, reps, whole_ms=None):
    """Per-kernel durations from HIP events recorded on the launch stream around every step of the plan.
    An event between two kernels costs time of its own (about 3 us here), which the intervals include: with
    whole_ms, the duration of one pass timed without those events, the excess of the intervals' sum over it is
    taken off the intervals that hold a launch, in equal parts (an interval without a launch counts as nothing)."""
    from paper_1810_00952_amd import harness
    desc = session.plan.describe()
    step_ms = session.plan.profile({vid: t.data_ptr() for vid, t in session.tensors.items()}, session.workspace.data_ptr(),
                                   session.workspace.numel(), harness.stream_handle(), reps)
    step_ms = list(step_ms)
    if whole_ms is not None:
        live = [i for i, st in enumerate(desc["steps"]) if not st["kernel"].startswith("(")]
        for i in range(len(step_ms)):
            if i not in live:
                step_ms[i] = 0.0
        excess = (sum(step_ms[i] for i in live) - whole_ms) / max(1, len(live))
        if excess > 0:
            floor = 0.25 * min(step_ms[i] for i in live)
            step_ms = [max(t - excess, floor) if i in live else t for i, t in enumerate(step_ms)]
        EVENT_OVERHEAD_US.append(max(excess, 0.0) * 1e3)
    by_kernel = {}
    for st, t in zip(desc["steps"], step_ms):
        k = by_kernel.setdefault(st["kernel"], {"ms": 0.0, "flops": 0.0, "bytes": 0.0, "launches": 0})
        k["ms"] += t; k["flops"] += st["flops"]; k["bytes"] += st["bytes"]; k["launches"] += 1
    return desc, by_kernel


def measured_traffic(kernel_name, profile_file):
    """HBM bytes per step of one kernel from the committed rocprofv3 counter summary, or None when the
    summary is missing, lacks the kernel, or was taken on other kernel sources than the ones in the tree."""
    import glob
    import hashlib
    path = os.path.join(ROOT, "profiles", profile_file)
    if not os.path.exists(path):
        return None
    h = hashlib.sha256()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_1810_00952_amd", "csrc", "*"))):
        with open(f, "rb") as fh:
            h.update(fh.read())
    sha, found = h.hexdigest()[:16], None
    sha_ok = False
    for line in open(path):
        if line.startswith("# source_sha"):
            sha_ok = line.split()[2] == sha
        elif not line.startswith("#") and line.split() and line.split()[0] == kernel_name:
            _, _, fb, wb = line.split()
            found = float(fb) + float(wb)
    return found if sha_ok else None


EVENT_OVERHEAD_US = []


def roofline_of(name, k, peak_tflops):
    """Roofline entry of one kernel (all its launches in a step): MFMA-bound when its algorithmic
    intensity is above the ridge of the peaks used, else HBM-bound."""
    tflops = k["flops"] / (k["ms"] * 1e-3) / 1e12
    gbs = k["bytes"] / (k["ms"] * 1e-3) / 1e9
    ridge = peak_tflops * 1e12 / (PEAK_HBM_GBS * 1e9)
    if name.startswith("igemm") and k["flops"] / max(k["bytes"], 1.0) >= ridge:
        roof = {"bound": "mfma", "achieved": tflops, "peak": peak_tflops, "unit": "TFLOP/s", "frac": tflops / peak_tflops}
    else:
        roof = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS}
    roof.update({"traffic": None, "kernel": name, "launches_per_step": k["launches"], "avg_launch_us": k["ms"] * 1e3 / k["launches"],
                 "event_overhead_us_removed_per_launch": EVENT_OVERHEAD_US[-1] if EVENT_OVERHEAD_US else 0.0,
                 "algorithmic_flops_per_step": k["flops"], "algorithmic_bytes_per_step": k["bytes"],
                 "algorithmic_bytes_per_launch": k["bytes"] / max(1, k["launches"])})
    return roof


def kernels_json(by_kernel, peak_tflops=None):
    """Per kernel: time, launches, algorithmic TFLOP/s and GB/s, and both as fractions of the quoted peaks (a contraction
    is held against the MFMA peak of its dtype whatever its arithmetic intensity says)."""
    rate = lambda amount, ms, unit: amount / (ms * 1e-3) / unit if ms > 0 else 0.0
    out = {}
    for k, v in sorted(by_kernel.items(), key=lambda kv: -kv[1]["ms"]):
        e = {"ms_per_step": v["ms"], "launches": v["launches"], "tflops": rate(v["flops"], v["ms"], 1e12), "gbs": rate(v["bytes"], v["ms"], 1e9)}
        e["hbm_frac"] = e["gbs"] / PEAK_HBM_GBS
        if peak_tflops and k.startswith("igemm"):
            e["mfma_frac"] = e["tflops"] / peak_tflops
        out[k] = e
    return out


def measure_peaks():
    """What this machine delivers next to the quoted peaks: a register-only bf16 MFMA chain on every SIMD, and the
    fused bias + residual + ReLU group streaming 1.2 GB (two reads and a write per element)."""
    import torch
    from paper_1810_00952_amd import binding, harness
    ctx = binding.Context()
    wg, iters = 512, 4096
    scratch = torch.empty(wg * 512, dtype=torch.float32, device="cuda:0")
    stream = harness.stream_handle()
    ctx.calibrate_mfma_bf16(scratch.data_ptr(), wg, 64, stream)
    torch.cuda.synchronize()
    best = None
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(torch.cuda.current_stream())
        flops = ctx.calibrate_mfma_bf16(scratch.data_ptr(), wg, iters, stream)
        e1.record(torch.cuda.current_stream())
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    return {"mfma_bf16_tflops_quoted": PEAK_BF16_TFLOPS, "mfma_bf16_tflops_measured": flops / (best * 1e-3) / 1e12,
            "mfma_measure": f"{wg} workgroups x 8 waves x {16 * iters} MFMAs 32x32x16 bf16 on register operands, best of 3",
            "hbm_gbs_quoted": PEAK_HBM_GBS}


def hbm_groups(args):
    """The HBM-bound groups on tensors far larger than the last-level cache, each as a plan of its own: algorithmic
    bytes per launch / mean launch duration (events on the launch stream) against the quoted 8 TB/s."""
    import workloads as W
    from paper_1810_00952_amd import harness
    import torch
    res = []

    def one(label, spec, data, nbytes):
        s = harness.Session(spec)
        s.load(data)
        s.alloc()
        ms = time_steps(s.run, 30, 5, graph=False)
        res.append({"group": label, "kernel": "+".join(st["kernel"] for st in s.plan.describe()["steps"]), "us": ms * 1e3,
                    "algorithmic_bytes": nbytes, "gbs": nbytes / (ms * 1e-3) / 1e9, "hbm_frac": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS})
        del s
        torch.cuda.empty_cache()
    for dtype, shape in (("bf16", (256, 64, 112, 112)), ("f32", (128, 64, 112, 112))):
        spec, make = W.eltwise_bias_res_relu(shape, dtype)
        n = shape[0] * shape[1] * shape[2] * shape[3]
        one(f"relu(bias_add(x) + r) {dtype} {'x'.join(map(str, shape))}", spec, make(), 3 * n * (2 if dtype == "bf16" else 4))
    B, H = 16384, 1024
    g = W.GraphSpec("gates")
    z = g.input("z", "f32", (B, 4 * H)); c = g.input("c", "f32", (B, H))
    o, (c2, h2) = g.op("lstm_gates", [z, c], [("f32", (B, H)), ("bf16", (B, H))])
    g.output(c2); g.output(h2)
    rng = W.rng_for(6, salt=2)
    one(f"lstm_gates z {B}x{4 * H} f32", g, {"z": W.as_dtype(W.normal(rng, (B, 4 * H)), "f32"), "c": W.as_dtype(W.normal(rng, (B, H)), "f32")},
        B * H * (16 + 4 + 4 + 2))
    spec, data = W.channel_last_maxpool(64, 64, 112, 112, 3, 2, 1, "bf16")
    one("maxpool2d 3x3/2 bf16 64x64x112x112 (channel-last)", spec, data, 64 * 64 * (112 * 112 + 56 * 56) * 2)
    return res


def time_steps_on_streams(sessions, steps, warmup):
    """The same K steps dealt round-robin to one stream per session (each session has its own activations and
    workspace; every step is still one whole pass over one batch).  Independent steps then overlap on the GPU: one
    stream's kernels run in the few microseconds between two dependent launches of the other, and on the CUs its
    196-200 workgroups leave free.  Host clock around the region, device synchronisation on both sides."""
    import time
    import torch
    streams = [torch.cuda.Stream() for _ in sessions]          # default priority

    def go(n):
        for i in range(n):
            k = i % len(sessions)
            with torch.cuda.stream(streams[k]):
                sessions[k].run()
    torch.cuda.synchronize()
    go(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    go(steps)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def base_json(metric, value, unit, args, ms, dtype, workload, extra_cfg=None):
    cfg = {"workload": workload, "launch": "hip graph replay" if GRAPH else "eager"}
    cfg.update(extra_cfg or {})
    out = {"metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic", "config": cfg,
           "paper_figures": "none"}
    out.update(TIMING)
    return out


def bench_resnet(args, batch, dtype):
    import torch
    import workloads as W
    from paper_1810_00952_amd import harness
    from helpers import fold_resnet_hip
    spec, raw, bn = W.resnet18(batch=batch, dtype=dtype)
    s = harness.Session(spec)
    fold_resnet_hip(s, raw, bn, dtype)
    s.alloc()
    ms = time_steps(s.run, args.steps, args.warmup)
    desc, by_kernel = kernel_table(s, args.profile_reps, ms)
    peak = PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_F32_TFLOPS
    dom_name, dom = max(by_kernel.items(), key=lambda kv: kv[1]["ms"])
    total_flops = sum(st["flops"] for st in desc["steps"] if st["kernel"].startswith("igemm"))
    name = "bf16 in / fp32 accumulate" if dtype == "bf16" else "f32"
    out = base_json(f"images/sec ResNet-18-shape bs{batch} {dtype}", batch / (ms * 1e-3), "images/s", args, ms, dtype,
                    f"ResNet-18-shaped inference graph, batch {batch}, {name}, folded batch-norm, 23 fused groups, 3x224x224 N(0,1) input",
                    {"global_batch": batch})
    out["tflops_whole_graph"] = total_flops / (ms * 1e-3) / 1e12
    out["roofline"] = roofline_of(dom_name, dom, peak)
    if dtype == "bf16" and batch == 64:
        per_step = measured_traffic(dom_name, "resnet18_b64_bf16_hbm_traffic.txt")
        out["roofline"]["traffic"] = per_step / dom["launches"] if per_step is not None else None      # bytes per launch
        out["roofline"]["traffic_per_step"] = per_step
    out["kernels"] = kernels_json(by_kernel, peak)
    if dtype == "bf16" and batch == 64:
        # the two targets of this path side by side: contractions against the bf16 MFMA peak, HBM-bound groups against 8 TB/s
        mf = sum(v["flops"] for k, v in by_kernel.items() if k.startswith("igemm"))
        mt = sum(v["ms"] for k, v in by_kernel.items() if k.startswith("igemm"))
        out["contractions_mfma_frac"] = mf / (mt * 1e-3) / 1e12 / peak if mt > 0 else None
        saved = dict(TIMING)
        if not args.no_extras:
            # reported beside the headline, never as it: `value` above is one step after the other on one stream
            s2 = harness.Session(spec)
            fold_resnet_hip(s2, raw, bn, dtype)
            s2.alloc()
            ms2 = time_steps_on_streams([s, s2], args.steps, args.warmup)
            out["two_streams"] = {"value": batch / (ms2 * 1e-3), "unit": "images/s", "ms_per_step": ms2, "streams": 2,
                                  "note": "the same K steps dealt alternately to two streams, each with its own session "
                                          "(activations, workspace); host clock, device synchronisation on both sides"}
            del s2
        del s
        torch.cuda.empty_cache()
        if not args.no_extras:
            out["peaks"] = measure_peaks()
            out["hbm_bound_groups"] = hbm_groups(args)
        TIMING.clear(); TIMING.update(saved)
    if not args.no_cpu and dtype == "bf16" and batch == 64:
        out["cpu_baseline"] = cpu_baseline_resnet(args.cpu_images)
    return out


def harness_session_run(spec, data):
    from paper_1810_00952_amd import harness
    s = harness.Session(spec)
    s.load(data)
    s.alloc()
    return s.run


def bench_graph(args, spec, data, metric, unit, units_per_step, dtype, workload, peak_tflops, cpu=None):
    from paper_1810_00952_amd import harness
    s = harness.Session(spec)
    s.load(data)
    s.alloc()
    ms = time_steps(s.run, args.steps, args.warmup)
    desc, by_kernel = kernel_table(s, args.profile_reps, ms)
    dom_name, dom = max(by_kernel.items(), key=lambda kv: kv[1]["ms"])
    out = base_json(metric, units_per_step / (ms * 1e-3), unit, args, ms, dtype, workload)
    out["roofline"] = roofline_of(dom_name, dom, peak_tflops)
    out["kernels"] = kernels_json(by_kernel, peak_tflops)
    if cpu is not None and not args.no_cpu:
        out["cpu_baseline"] = cpu()
    return out


def bench_lstm(args):
    import numpy as np
    import torch
    import workloads as W
    from paper_1810_00952_amd import harness
    T, B, I, H = 128, 64, 1024, 1024
    d = W.lstm_data(T, B, I, H, "bf16")
    spec = W.lstm_cell_graph(B, I, H, "bf16", fused=not args.unfused)
    s = harness.Session(spec)
    s.load({"w": d["w"], "b": d["b"]})
    x = harness.to_device(d["x"], "bf16")
    h0 = torch.zeros((B, H), dtype=torch.bfloat16, device="cuda:0")
    c = torch.zeros((B, H), dtype=torch.float32, device="cuda:0")
    hs = torch.empty((T, B, H), dtype=torch.bfloat16, device="cuda:0")
    ws = torch.empty(max(256, s.plan.recurrent_workspace_bytes(T)), dtype=torch.uint8, device="cuda:0")
    n = s.by_name
    roles = {"x": n["x"], "h_in": n["h"], "c_in": n["c"], "c_out": spec.outputs[0], "h_out": spec.outputs[1]}
    params = {n["w"]: s.tensors[n["w"]].data_ptr(), n["b"]: s.tensors[n["b"]].data_ptr()}

    def run():
        c.zero_()
        s.plan.run_recurrent(T, roles, x.data_ptr(), B * I * 2, h0.data_ptr(), c.data_ptr(), hs.data_ptr(), B * H * 2, params,
                             ws.data_ptr(), ws.numel(), harness.stream_handle())
    ms = time_steps(run, args.steps, args.warmup)
    timing = dict(TIMING)
    ms_two = None
    if not args.no_extras:
        # two independent batches of sequences on two streams (second cell state, outputs and workspace; x, h_0 and
        # the weights are only read): one stream's step kernel runs between two dependent launches of the other
        c2, hs2, ws2 = torch.zeros_like(c), torch.empty_like(hs), torch.empty_like(ws)

        def run2():
            c2.zero_()
            s.plan.run_recurrent(T, roles, x.data_ptr(), B * I * 2, h0.data_ptr(), c2.data_ptr(), hs2.data_ptr(), B * H * 2, params,
                                 ws2.data_ptr(), ws2.numel(), harness.stream_handle())

        class _R:
            def __init__(self, f): self.run = f
        ms_two = time_steps_on_streams([_R(run), _R(run2)], args.steps, args.warmup)
        assert bool(torch.equal(hs, hs2)), "the two streams' sequences differ"
    # the same sequence of launches replayed from a HIP graph (the cell-state reset and every kernel of the sequence)
    ms_graph = time_steps(run, args.steps, args.warmup, graph=True) if not GRAPH else None
    TIMING.clear(); TIMING.update(timing)
    desc = s.plan.describe()
    flops = sum(st["flops"] for st in desc["steps"]) * T
    hoisted = ws.numel() > max(256, s.plan.workspace_bytes()) and not args.unfused
    if hoisted:
        # input projection of all steps as one contraction (x, Wx read once, zx written once), then per step the
        # recurrent weights, that step's zx, h in and out, c in and out
        nbytes = (T * B * I * 2 + 4 * H * I * 2 + T * B * 4 * H * 4) + T * (4 * H * H * 2 + B * 4 * H * 4 + 2 * B * H * 2 + 2 * B * H * 4)
        kernels, launches = "igemm_lp_f32out_kernel 256x128 (once) + lstm_step_kernel (per step)", T + 1
    else:
        nbytes = sum(st["bytes"] for st in desc["steps"]) * T
        kernels, launches = "+".join(st["kernel"] for st in desc["steps"]), T * len(desc["steps"])
    out = base_json("sequences/sec unrolled LSTM b64 1024x1024 T128 bf16", B / (ms * 1e-3), "sequences/s", args, ms, "bf16",
                    "unrolled LSTM, batch 64, input and hidden 1024, 128 steps, bf16 weights, fp32 accumulate, "
                    + ("input projection hoisted, one recurrent kernel per step" if hoisted else
                       "gate math fused into the GEMM epilogue" if not args.unfused else "GEMM group and gate group"))
    out["us_per_step_of_sequence"] = ms * 1e3 / T
    if ms_two is not None:
        out["two_streams"] = {"value": B / (ms_two * 1e-3), "unit": "sequences/s", "ms_per_step": ms_two, "streams": 2,
                              "note": "independent batches of sequences dealt alternately to two streams; host clock, device synchronisation on both sides"}
    if ms_graph is not None:
        out["hip_graph_replay"] = {"ms_per_step": ms_graph, "us_per_step_of_sequence": ms_graph * 1e3 / T, "sequences_per_s": B / (ms_graph * 1e-3)}
    tflops, gbs = flops / (ms * 1e-3) / 1e12, nbytes / (ms * 1e-3) / 1e9
    # a step is a 64-row contraction that must finish before the next can start: bound by memory traffic and latency
    out["roofline"] = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "traffic": None,
                       "kernel": kernels, "launches_per_step": launches,
                       "avg_launch_us": ms * 1e3 / launches, "algorithmic_flops_per_step": flops,
                       "algorithmic_bytes_per_step": nbytes, "tflops": tflops}
    if not args.no_cpu:
        import oracle as O
        Ts = 8
        t0 = time.perf_counter()
        O.lstm_sequence(O.widen(d["x"][:Ts], "bf16"), O.widen(d["w"], "bf16"), O.widen(d["b"], "f32"), np.zeros((B, H)), np.zeros((B, H)), h_dtype="bf16")
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": B / (dt * T / Ts), "unit": "sequences/s", "cores": O.num_threads(), "kind": "oracle",
                               "sample": f"first {Ts} of the 128 steps, scaled to the full sequence, {dt:.1f} s"}
    return out


def bench_grads(args):
    """The four gradient operators of the contractions at the shapes of the benchmark graph's second stage (batch 64,
    128 channels, 28x28) and of its dense head, bf16 operands; each a plan of its own."""
    import torch
    import workloads as W
    from paper_1810_00952_amd import harness
    cases = [("conv2d_grad_x", (64, 128, 28, 28, 128, 3), 1, 1, True), ("conv2d_grad_w", (64, 128, 28, 28, 128, 3), 1, 1, False),
             ("conv2d_grad_x", (64, 64, 56, 56, 128, 3), 2, 1, True), ("conv2d_grad_w", (64, 64, 56, 56, 128, 3), 2, 1, False),
             ("dense_grad_x", (64, 1000, 512), 1, 0, True), ("dense_grad_w", (64, 1000, 512), 1, 0, False)]
    # ... and dy pushed back through three stacked convolutions, where all but the last result stay inside the plan
    cases.append(("conv2d_grad_x x3 in a row", (64, 128, 28, 28, 128, 3), 1, 1, True))
    rows, tot_ms, tot_flops = [], 0.0, 0.0
    for kind, dims, stride, pad, is_param in cases:
        if kind.endswith("in a row"):
            spec, data = W.grad_chain(dims[0], dims[1], dims[2], 3, "bf16")
        else:
            spec, data = W.grad_case(kind, dims, "bf16", stride, pad, second_is_param=is_param)
        s = harness.Session(spec)
        s.load(data)
        s.alloc()
        ms = time_steps(s.run, args.steps, args.warmup, graph=False)
        steps = s.plan.describe()["steps"]
        flops = sum(st["flops"] for st in steps)
        rows.append({"op": kind, "dims": list(dims), "stride": stride, "pad": pad, "kernels": [st["kernel"] for st in steps], "us": ms * 1e3,
                     "tflops": flops / (ms * 1e-3) / 1e12, "mfma_frac": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS})
        tot_ms += ms; tot_flops += flops
        del s
        torch.cuda.empty_cache()
    out = base_json("TFLOP/s gradient operators of dense / conv2d, bf16", tot_flops / (tot_ms * 1e-3) / 1e12, "TFLOP/s", args, tot_ms, "bf16",
                    "dense_grad_x/_w on 64x1000x512 and conv2d_grad_x/_w on 64x128x28x28 (3x3/1) and 64x64x56x56 -> 128 (3x3/2), bf16, N(0,1) operands")
    out["roofline"] = {"bound": "mfma", "achieved": out["value"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": out["value"] / PEAK_BF16_TFLOPS,
                       "traffic": None, "kernel": "all kernels of the seven plans"}
    out["operators"] = rows
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet18",
                    choices=["resnet18", "resnet18_f32_b1", "eltwise", "eltwise32", "gates", "lstm", "mlp", "lenet", "conv", "copy", "layout", "layout32", "block_nhwc", "maxpool", "mfma_peak", "grads", "launch_pitch", "gemm"])
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--cpu-images", type=int, default=128)
    ap.add_argument("--elements", type=int, default=0, help="copy: number of f32 elements (default 24 Mi)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="default workload: skip the MFMA calibration and the HBM-bound groups")
    ap.add_argument("--unfused", action="store_true", help="lstm: gate math as a group of its own")
    ap.add_argument("--profile-reps", type=int, default=20)
    ap.add_argument("--graph", action="store_true", help="time replays of a HIP graph that holds one step (same kernels, no host launches)")
    args = ap.parse_args()
    global GRAPH
    GRAPH = args.graph
    if args.gpus != 1:
        print("bench.py measures one GPU: this path has no multi-GPU part (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as W
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    wl = args.workload
    if wl == "resnet18":
        out = bench_resnet(args, args.batch, "bf16")
    elif wl == "resnet18_f32_b1":
        out = bench_resnet(args, 1, "f32")
    elif wl in ("eltwise", "eltwise32"):
        dtype, shape = ("bf16", (256, 64, 112, 112)) if wl == "eltwise" else ("f32", (128, 64, 112, 112))
        spec, make = W.eltwise_bias_res_relu(shape, dtype)
        n = shape[0] * shape[1] * shape[2] * shape[3]
        out = bench_graph(args, spec, make(), f"elements/sec fused bias+residual+relu {dtype}", "elements/s", n, dtype,
                          f"relu(bias_add(x) + r) on {'x'.join(map(str, shape))} {dtype}, one fusion group, N(0,1) inputs", PEAK_F32_TFLOPS)
    elif wl == "gates":
        import numpy as np
        B, H = 16384, 1024
        g = W.GraphSpec("gates")
        z = g.input("z", "f32", (B, 4 * H)); c = g.input("c", "f32", (B, H))
        o, (c2, h2) = g.op("lstm_gates", [z, c], [("f32", (B, H)), ("bf16", (B, H))])
        g.output(c2); g.output(h2)
        rng = W.rng_for(6, salt=2)
        data = {"z": W.as_dtype(W.normal(rng, (B, 4 * H)), "f32"), "c": W.as_dtype(W.normal(rng, (B, H)), "f32")}
        out = bench_graph(args, g, data, "hidden units/sec LSTM gate group", "units/s", B * H, "f32",
                          f"lstm_gates on z {B}x{4 * H} f32, c {B}x{H} f32 -> c' f32, h' bf16", PEAK_F32_TFLOPS)
    elif wl == "copy":
        n = args.elements or (24 << 20)
        g = W.GraphSpec("copy")
        x = g.input("x", "f32", (n,))
        o, (y,) = g.op("neg", [x], [("f32", (n,))])
        g.group([o]); g.output(y)
        data = {"x": W.as_dtype(W.normal(W.rng_for(6, salt=3), (n,)), "f32")}
        out = bench_graph(args, g, data, "elements/sec y = -x f32", "elements/s", n, "f32",
                          f"y = -x on {n} f32 elements (reads {4 * n} bytes, writes {4 * n} bytes)", PEAK_F32_TFLOPS)
    elif wl == "gemm":
        # a dense group at matrix-multiplication scale: relu(x W^T + b), 4096 x 4096 x 4096, bf16
        import numpy as np
        M = N = K = 4096
        g = W.GraphSpec("gemm")
        x = g.input("x", "bf16", (M, K)); w = g.param("w", "bf16", (N, K)); b = g.param("b", "f32", (N,))
        o0, (y,) = g.op("dense", [x, w], [("bf16", (M, N))])
        o1, (y,) = g.op("bias_add", [y, b], [("bf16", (M, N))], axis=1)
        o2, (y,) = g.op("relu", [y], [("bf16", (M, N))])
        g.group([o0, o1, o2]); g.output(y)
        rng = W.rng_for(6, salt=5)
        data = {"x": W.as_dtype(W.normal(rng, (M, K)), "bf16"), "w": W.as_dtype(W.kaiming_uniform(rng, (N, K), K), "bf16"),
                "b": W.as_dtype(W.uniform(rng, (N,), -0.1, 0.1), "f32")}
        out = bench_graph(args, g, data, "TFLOP/s dense + bias + ReLU 4096x4096x4096 bf16", "TFLOP/s", 2.0 * M * N * K / 1e12, "bf16",
                          "one dense group relu(x W^T + b), x 4096x4096, W 4096x4096, bf16 in, fp32 accumulate, N(0,1) / Kaiming inputs", PEAK_BF16_TFLOPS)
    elif wl == "launch_pitch":
        # a chain of 16 dependent groups of y = -x on 1024 elements: nothing but the distance between two dependent
        # launches on one stream (the figure behind the launch-boundary share of every step here)
        n, depth = 1024, 16
        g = W.GraphSpec("launch_pitch")
        v = g.input("x", "f32", (n,))
        for _ in range(depth):
            o, (v,) = g.op("neg", [v], [("f32", (n,))])
            g.group([o])
        g.output(v)
        data = {"x": W.as_dtype(W.normal(W.rng_for(6, salt=4), (n,)), "f32")}
        out = bench_graph(args, g, data, "dependent launches/sec on one stream", "launches/s", depth, "f32",
                          f"{depth} dependent groups of y = -x on {n} f32 elements, one launch each", PEAK_F32_TFLOPS)
        out["us_per_dependent_launch"] = out["ms_per_step"] * 1e3 / depth
        ms_graph = time_steps(harness_session_run(g, data), args.steps, args.warmup, graph=True)
        out["hip_graph_replay"] = {"us_per_dependent_launch": ms_graph * 1e3 / depth}
    elif wl in ("layout", "layout32"):
        dtype, shape = ("bf16", (256, 64, 112, 112)) if wl == "layout" else ("f32", (128, 64, 112, 112))
        spec, data = W.layout_case(shape, (0, 2, 3, 1), dtype)
        n = shape[0] * shape[1] * shape[2] * shape[3]
        out = bench_graph(args, spec, data, f"elements/sec channel-first to channel-last {dtype}", "elements/s", n, dtype,
                          f"layout_transform (0,2,3,1) of {'x'.join(map(str, shape))} {dtype}, N(0,1) input", PEAK_F32_TFLOPS)
    elif wl == "maxpool":
        spec, data = W.channel_last_maxpool(64, 64, 112, 112, 3, 2, 1, "bf16")
        out = bench_graph(args, spec, data, "output elements/sec max-pool 3x3/2 bf16", "elements/s", 64 * 64 * 56 * 56, "bf16",
                          "maxpool2d 3x3 stride 2 pad 1 on 64x64x112x112 bf16 (between channel-last tensors), N(0,1) input", PEAK_F32_TFLOPS)
    elif wl == "block_nhwc":
        spec, data = W.channel_last_block(64, 64, 56, 56, "bf16")
        out = bench_graph(args, spec, data, "images/sec residual block 64ch 56x56 bf16 b64 between channel-last tensors", "images/s", 64, "bf16",
                          "channel-last input -> layout_transform -> two 3x3 64->64 convolution groups (+bias, +input, ReLU) -> layout_transform "
                          "-> channel-last output, bf16, batch 64", PEAK_BF16_TFLOPS)
    elif wl == "lstm":
        out = bench_lstm(args)
    elif wl == "grads":
        out = bench_grads(args)
    elif wl == "mfma_peak":
        pk = measure_peaks()
        out = base_json("TFLOP/s bf16 MFMA chain on register operands", pk["mfma_bf16_tflops_measured"], "TFLOP/s", args, 0.0, "bf16", pk["mfma_measure"])
        out["roofline"] = {"bound": "mfma", "achieved": pk["mfma_bf16_tflops_measured"], "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                           "frac": pk["mfma_bf16_tflops_measured"] / PEAK_BF16_TFLOPS, "traffic": None, "kernel": "mfma_peak_kernel"}
    elif wl == "mlp":
        spec, data = W.mlp(32, 784, 128, 10, "f32")
        out = bench_graph(args, spec, data, "samples/sec MLP 784-128-10 f32 b32", "samples/s", 32, "f32",
                          "MLP fusion graph, f32, batch 32: dense 784->128 + bias + ReLU, dense 128->10 + bias", PEAK_F32_TFLOPS,
                          cpu=lambda: cpu_baseline_graph(spec, data, 32, "samples/s", "the same 32-sample batch"))
    elif wl == "lenet":
        spec, data = W.lenet(64, "f32")
        out = bench_graph(args, spec, data, "images/sec LeNet-shaped graph f32 b64", "images/s", 64, "f32",
                          "the paper's LeNet-shaped example as a fusion graph, f32, batch 64, 1x28x28 N(0,1) inputs: conv5x5+bias+tanh, "
                          "maxpool2, conv5x5+bias+tanh, maxpool2, flatten, dense 800->500+bias+tanh, dense 500->10+bias", PEAK_F32_TFLOPS,
                          cpu=lambda: cpu_baseline_graph(spec, data, 64, "images/s", "the same 64-image batch"))
    else:
        spec, data = W.conv_group(1, 64, 64, 56, 56, 3, 1, 1, "f32")
        out = bench_graph(args, spec, data, "images/sec single conv2d group 64->64 56x56 f32 b1", "images/s", 1, "f32",
                          "single fused conv2d group, f32, NCHW, batch 1, 64->64 channels, 56x56, 3x3, + bias + ReLU", PEAK_F32_TFLOPS,
                          cpu=lambda: cpu_baseline_graph(spec, data, 1, "images/s", "the same image"))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
