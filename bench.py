#!/usr/bin/env python3
"""Benchmark of the convolution hot path on one MI355X.

A "step" is one pass of the whole hot path -- forward, backward data, backward filter and backward
bias -- over every layer of the workload, with all inputs already resident in HBM.  The default
workload is the large grouped-conv configuration (layers 5.a, 5.b, 5.c: the GEMM-bound shapes the
metric is about).  The metric is fwd+bwd GFLOP/s = 3 * (multiply-add FLOPs of one pass) / time,
counting only algorithmic FLOPs (no credit for tile padding; bias adds and the bias-gradient
reduction add time but no FLOPs).

``--workload ip5`` / ``ip1`` (or a comma list of ip layer names) times the InnerProduct layers that
follow those convolution stacks instead: forward (bias + ReLU fused), ReLU backward, backward data,
backward filter, backward bias; same FLOP rule (2*m*k*num_output per contraction, three of them).

``--workload pg`` times the policy-gradient loss kernels on a batch of 65536 synthetic episodes
(HBM-bound: the metric there is algorithmic GB/s).

Prints ONE JSON line (rank 0 is the only rank: this benchmark is single-GPU).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X published dense fp32 matrix peak
PEAK_FP64_MFMA_TFLOPS = 78.6   # ... and fp64
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="config4", help="config0..config4, small (the eight layers of configs 0-3), dw (depthwise layers), ip5, ip1, pg, or a "
                                                    "comma list of layer names (all conv or all ip)")
    ap.add_argument("--dtype", default="f32", choices=["f32", "f64"],
                    help="base type of the convolution workloads (f64: the conv_*_f64 entry points)")
    ap.add_argument("--no-cpu-baseline", action="store_true",
                    help="skip the context legs after the timed steps (the small-layer table, the CPU oracle timing "
                         "and the two-stream schedule): what runs under the profiler")
    ap.add_argument("--cpu-sample-images", type=int, default=128)
    ap.add_argument("--cold-cache", action="store_true",
                    help="rotate every step among enough distinct sets of tensors that one pass over all sets "
                         "exceeds 512 MB (twice the 256 MB last-level cache), so no operand of a pass is still "
                         "cached from the step before")
    ap.add_argument("--overlap", action="store_true",
                    help="time the step as a training loop would schedule it on two streams: the forward passes, "
                         "then the backward-data passes on the launch stream with the filter and bias gradients of "
                         "the same layers on a second stream (own workspace); prints the whole-step rate only")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (no per-pass times): what the "
                         "microsecond-scale layers cost without the per-dispatch launch gaps")
    ap.add_argument("--separate-bias", action="store_true",
                    help="fp32 convolution workloads: call conv_backward_filter and conv_backward_bias (two reads of dy) "
                         "instead of conv_backward_filter_bias (one)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 256 MiB device copies (outside the timed region) so that a rocprofv3 "
                         "--pmc FETCH_SIZE / WRITE_SIZE run of this command holds a kernel of known traffic")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: every box of this build has a single MI355X and the "
              "path has no multi-GPU part; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import bench_probe
    import paper_1810_02272_amd as conv
    from paper_1810_02272_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (there is no CPU path)", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.copy_calibration:
        src = torch.ones(64 << 20, device=dev)  # 256 MiB read + 256 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.workload == "pg":
        return bench_pg(args, torch, conv, workloads, dev)
    is_ip = args.workload.startswith("ip")
    f64 = args.dtype == "f64"
    if f64 and is_ip:
        print("--dtype f64 applies to the convolution workloads only", file=sys.stderr)
        sys.exit(2)
    tdt = torch.float64 if f64 else torch.float32
    peak = PEAK_FP64_MFMA_TFLOPS if f64 else PEAK_FP32_MFMA_TFLOPS
    if args.workload.startswith("config"):
        cfg = int(args.workload[len("config"):])
        layers = [l for l in workloads.LAYERS if l.config == cfg]
    elif args.workload == "small":  # the eight layer shapes of configurations 0-3
        layers = [l for l in workloads.LAYERS if l.config <= 3]
    elif args.workload == "dw":
        layers = list(workloads.DW_LAYERS)
    elif args.workload in ("ip5", "ip1"):
        layers = [l for l in workloads.IP_LAYERS if l.name.startswith(args.workload + ".")]
    elif is_ip:
        layers = [workloads.IP_BY_NAME[n] for n in args.workload.split(",")]
    else:
        layers = [workloads.BY_NAME[n] for n in args.workload.split(",")]

    # ---- set-up (untimed): descriptors, inputs resident in HBM, one shared workspace ----
    state = []
    ws_bytes = 0
    for l in layers:
        if is_ip:
            d = conv.ip_desc_create(conv.IpParams(**l.params_dict()))
            ws_bytes = max(ws_bytes, conv.ip_desc_workspace_bytes(d))
            x, w, b, dy = workloads.ip_inputs(l, bias="zero")
            t = dict(layer=l, desc=d, x=x.to(dev), w=w.to(dev), b=b.to(dev), dy=dy.to(dev),
                     y=torch.empty((l.m, l.num_output), device=dev), dz=torch.empty((l.m, l.num_output), device=dev),
                     dx=torch.empty((l.m, l.k), device=dev), dw=torch.empty((l.num_output, l.k), device=dev),
                     db=torch.empty(l.num_output, device=dev))
        else:
            d = conv.conv_desc_create(conv.ConvParams(**l.params_dict()))
            ws_bytes = max(ws_bytes, conv.conv_desc_workspace_bytes_f64(d) if f64 else
                           conv.conv_desc_workspace_bytes(d))
            x, w, b, dy = (v.to(tdt) for v in workloads.layer_inputs(l, bias="zero"))
            t = dict(layer=l, desc=d, x=x.to(dev), w=w.to(dev), b=b.to(dev), dy=dy.to(dev),
                     y=torch.empty(l.y_shape, device=dev, dtype=tdt), dx=torch.empty(l.x_shape, device=dev, dtype=tdt),
                     dw=torch.empty(l.w_shape, device=dev, dtype=tdt), db=torch.empty(l.k, device=dev, dtype=tdt))
        sets = [{k: v for k, v in t.items() if isinstance(v, torch.Tensor)}]
        if args.cold_cache:
            set_bytes = sum(v.numel() * v.element_size() for v in sets[0].values())
            while len(sets) * set_bytes < (512 << 20) and len(sets) < 64:
                sets.append({k: v.clone() for k, v in sets[0].items()})
        t["sets"] = sets
        state.append(t)
    ws = torch.empty(max(ws_bytes // 4, 1), device=dev)
    stream = torch.cuda.current_stream()

    # fp32 convolution: both parameter gradients come from one pass over dy (conv_backward_filter_bias)
    fused_bias = not is_ip and not f64 and not args.separate_bias
    passes = ("fwd", "relu_bwd", "bwd_data", "bwd_filter", "bwd_bias") if is_ip else (
        "fwd", "bwd_data", "bwd_filter_bias") if fused_bias else ("fwd", "bwd_data", "bwd_filter", "bwd_bias")
    flop_passes = ("fwd", "bwd_data", "bwd_filter", "bwd_filter_bias")
    kernel_names_of = (conv.ip_desc_kernel_names if is_ip else
                       conv.conv_desc_kernel_names_f64 if f64 else conv.conv_desc_kernel_names)

    def run_pass(t, name):
        run_pass_on(t, name, stream)

    def run_pass_on(t, name, stream, wsp=None):
        d = t["desc"]
        wsp = ws if wsp is None else wsp
        if is_ip:
            if name == "fwd":
                conv.ip_forward(d, t["x"], t["w"], t["b"], t["y"], wsp, stream)
            elif name == "relu_bwd":
                conv.ip_relu_backward(d, t["y"] if t["layer"].relu else None, t["dy"], t["dz"], stream)
            elif name == "bwd_data":
                conv.ip_backward_data(d, t["w"], t["dz"], t["dx"], wsp, stream)
            elif name == "bwd_filter":
                conv.ip_backward_filter(d, t["x"], t["dz"], t["dw"], 0.0, wsp, stream)
            else:
                conv.ip_backward_bias(d, t["dz"], t["db"], 0.0, wsp, stream)
        elif f64:
            if name == "fwd":
                conv.conv_forward_f64(d, t["x"], t["w"], t["b"], t["y"], wsp, stream)
            elif name == "bwd_data":
                conv.conv_backward_data_f64(d, t["w"], t["dy"], t["dx"], wsp, stream)
            elif name == "bwd_filter":
                conv.conv_backward_filter_f64(d, t["x"], t["dy"], t["dw"], 0.0, wsp, stream)
            else:
                conv.conv_backward_bias_f64(d, t["dy"], t["db"], 0.0, wsp, stream)
        elif name == "fwd":
            conv.conv_forward(d, t["x"], t["w"], t["b"], t["y"], wsp, stream)
        elif name == "bwd_data":
            conv.conv_backward_data(d, t["w"], t["dy"], t["dx"], wsp, stream)
        elif name == "bwd_filter":
            conv.conv_backward_filter(d, t["x"], t["dy"], t["dw"], 0.0, wsp, stream)
        elif name == "bwd_filter_bias":
            conv.conv_backward_filter_bias(d, t["x"], t["dy"], t["dw"], t["db"], 0.0, wsp, stream)
        else:
            conv.conv_backward_bias(d, t["dy"], t["db"], 0.0, wsp, stream)

    step_no = [0]

    def step(events=None, only=None):
        step_no[0] += 1
        for t in state:
            t.update(t["sets"][step_no[0] % len(t["sets"])])
            for name in passes:
                if events is not None and (only is None or only == (t["layer"].name, name)):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    run_pass(t, name)
                    e1.record(stream)
                    events.append((t["layer"].name, name, e0, e1))
                else:
                    run_pass(t, name)

    # Cost of one empty dispatch on this machine, for reading the microsecond-scale layers: a one-element
    # fill, enqueued back to back.
    one = torch.zeros(1, device=dev)
    for _ in range(20):
        one.zero_()
    le0, le1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    le0.record(stream)
    for _ in range(200):
        one.zero_()
    le1.record(stream)
    torch.cuda.synchronize()
    launch_us = le0.elapsed_time(le1) * 1e3 / 200

    # What the matrix pipes deliver with nothing else in the way: a register-only loop of matrix
    # instructions on every SIMD (two waves each), with the core clock the chip sustains under it.
    # Context for the published peak that `roofline.peak` uses.
    mfma_loop = bench_probe.register_loop_rate(f64=f64)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    def time_two_streams(steps, warmup):
        """Seconds for `steps` steps scheduled as a training loop would: forward passes, then the
        backward-data chain on the launch stream with the filter and bias gradients of the same layers
        on a second stream (default priority, workspace of its own)."""
        side = torch.cuda.Stream()
        ws_side = torch.empty_like(ws)

        def overlapped_step():
            step_no[0] += 1
            for t in state:
                t.update(t["sets"][step_no[0] % len(t["sets"])])
                run_pass_on(t, "fwd", stream)
            fork = torch.cuda.Event()
            fork.record(stream)
            side.wait_event(fork)
            for t in reversed(state):
                run_pass_on(t, "bwd_data", stream)
                if fused_bias:
                    run_pass_on(t, "bwd_filter_bias", side, ws_side)
                else:
                    run_pass_on(t, "bwd_filter", side, ws_side)
                    run_pass_on(t, "bwd_bias", side, ws_side)
            join = torch.cuda.Event()
            join.record(side)
            stream.wait_event(join)

        for _ in range(warmup):
            overlapped_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            overlapped_step()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    if args.overlap:
        if is_ip:
            print("--overlap applies to the convolution workloads", file=sys.stderr)
            sys.exit(2)
        wall = time_two_streams(args.steps, args.warmup)
        flop_step = 3 * sum(l.flop_per_pass for l in layers)
        print(json.dumps({
            "metric": "conv fwd+bwd GFLOP/s, filter and bias gradients on a second stream, " + args.dtype,
            "value": round(flop_step * args.steps / wall / 1e9, 1), "unit": "GFLOP/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall / args.steps * 1e3, 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"{args.workload}: layers " + ",".join(l.name for l in layers) + ", two streams",
                       "frac_of_mfma_peak": round(flop_step * args.steps / wall / 1e12 / peak, 4)}}))
        return

    if args.graph:
        if args.cold_cache:
            print("--graph replays one captured step: it cannot rotate tensor sets (--cold-cache)", file=sys.stderr)
            sys.exit(2)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for t in state:
                for name in passes:
                    run_pass_on(t, name, torch.cuda.current_stream())
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        flop_step = 3 * sum(l.flop_per_pass for l in layers)
        print(json.dumps({
            "metric": "fwd+bwd GFLOP/s, one captured step replayed as a HIP graph, " + args.dtype,
            "value": round(flop_step * args.steps / wall / 1e9, 1), "unit": "GFLOP/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall / args.steps * 1e3, 4),
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": args.dtype, "data": "synthetic",
            "config": {"workload": f"{args.workload}: layers " + ",".join(l.name for l in layers) + ", graph replay",
                       "frac_of_mfma_peak": round(flop_step * args.steps / wall / 1e12 / peak, 4)}}))
        return

    # ---- per-pass times (untimed): HIP events around every pass on the launch stream.  An event pair
    # per pass costs the step about 2 % (48 extra queue packets at config 4), so this table comes from
    # steps of its own and the timed region below carries events around the dominant pass only. ----
    table_steps = max(3, min(args.steps, 10))
    events = []
    for _ in range(table_steps):
        step(events)
    torch.cuda.synchronize()
    acc = {}
    for lname, pname, e0, e1 in events:
        acc.setdefault((lname, pname), []).append(e0.elapsed_time(e1))
    dominant = max(((k, sum(v) / len(v)) for k, v in acc.items()), key=lambda kv: kv[1])[0]
    separate = {}
    # for reference: the two gradient passes called one by one (not part of the step; left out of a
    # counter run, whose summary matches dispatches to passes by their order inside whole steps)
    if fused_bias and not args.copy_calibration:
        ev = []
        for _ in range(table_steps):
            for t in state:
                for name in ("bwd_filter", "bwd_bias"):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    run_pass(t, name)
                    e1.record(stream)
                    ev.append((t["layer"].name, name, e0, e1))
        torch.cuda.synchronize()
        for lname, pname, e0, e1 in ev:
            separate.setdefault((lname, pname), []).append(e0.elapsed_time(e1))

    # ---- timed region: exactly --steps steps; HIP events around the dominant pass of every step ----
    dom_events = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(dom_events, dominant)
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    wall = t1 - t0
    flop_step = 3 * sum(l.flop_per_pass for l in layers)
    value = flop_step * args.steps / wall / 1e9
    ms_per_step = wall / args.steps * 1e3
    per_layer = []
    for t in state:
        l = t["layer"]
        row = {"layer": l.name, "gflop_per_pass": l.flop_per_pass / 1e9,
               "kernels": kernel_names_of(t["desc"])}
        tot = 0.0
        launches = launches_of(row["kernels"])
        if fused_bias:  # the reduce kernel finishes both gradients: the launches of the filter gradient alone
            launches["bwd_filter_bias"] = launches.pop("bwd_filter")
            launches.pop("bwd_bias", None)
        for name in passes:
            ms = sum(acc[(l.name, name)]) / len(acc[(l.name, name)])
            row[name + "_ms"] = round(ms, 5)
            tot += ms
            if name in launches:
                # kernel launches of the pass, and what is left of its time after that many empty
                # dispatches (the floor of a launch-bound pass on this machine)
                row[name + "_launches"] = launches[name]
                row[name + "_us_over_launch_floor"] = round(ms * 1e3 - launches[name] * launch_us, 2)
            if not is_ip and name in flop_passes:  # every blob of the pass moved once, against 8 TB/s
                row[name + "_alg_GBps"] = round(blob_bytes(l, name) * (2 if f64 else 1) / ms / 1e6, 1)
            if name == "bwd_filter_bias" and separate:  # the same passes called one by one, outside the step
                for sep in ("bwd_filter", "bwd_bias"):
                    row["separate_" + sep + "_ms"] = round(sum(separate[(l.name, sep)]) / len(separate[(l.name, sep)]), 5)
                row["bias_gradient_extra_ms"] = round(ms - row["separate_bwd_filter_ms"], 5)
            if name in flop_passes:
                row[name + "_tflops"] = round(l.flop_per_pass / ms / 1e9, 2)
            elif name == "bwd_bias":  # one read of dy: the HBM-bound pass
                row["bwd_bias_GBps"] = round(dy_bytes(l) * (2 if f64 else 1) / ms / 1e6, 1)
            if name in flop_passes and not is_ip and "direct" in row["kernels"]:
                row[name + "_GBps"] = round(blob_bytes(l, name) * (2 if f64 else 1) / ms / 1e6, 1)
        row["fwd_bwd_tflops"] = round(3 * l.flop_per_pass / tot / 1e9, 2)
        if not is_ip and l.name in ("1.a", "3.a", "4.a", "5.a") and "bwd_data_ms" in row:
            # first layer of its network: real training skips its backward-data pass (no gradient
            # flows into the data), so also give the rate over forward + backward filter + backward bias
            row["first_layer_without_bwd_data_tflops"] = round(
                2 * l.flop_per_pass / (tot - row["bwd_data_ms"]) / 1e9, 2)
        row["fwd_bwd_frac_of_%s_mfma_peak" % ("fp64" if f64 else "fp32")] = round(
            3 * l.flop_per_pass / tot / 1e9 / peak, 4)
        if not is_ip:
            alg = 3 * blob_bytes(l, "fwd") + (0 if fused_bias else dy_bytes(l))
            row["fwd_bwd_frac_of_hbm_peak"] = round(alg * (2 if f64 else 1) / tot / 1e6 / PEAK_HBM_GBS, 4)
            row["fwd_bwd_us"] = round(tot * 1e3, 2)
            row["launches"] = sum(launches.values())
        per_layer.append(row)

    # dominant launch: the (layer, pass) with the largest average duration
    dl, dp = dominant
    dms = sum(e0.elapsed_time(e1) for _, _, e0, e1 in dom_events) / len(dom_events)
    dstate = next(t for t in state if t["layer"].name == dl)
    dlayer = dstate["layer"]
    kernel_names = dict(kv.split("=", 1) for kv in kernel_names_of(dstate["desc"]).split(";"))
    if "bwd_filter" in kernel_names:  # the pass that also sums dy runs the filter-gradient kernel
        kernel_names["bwd_filter_bias"] = kernel_names["bwd_filter"]
    direct = not is_ip and "direct" in kernel_names.get(dp, "")
    if dp in ("bwd_bias", "relu_bwd") or direct:
        if direct:  # thin groups: every blob of the pass moved once
            bytes_launch = blob_bytes(dlayer, dp) * (2 if f64 else 1)
        else:
            bytes_launch = dy_bytes(dlayer) * (1 if dp == "bwd_bias" else 3) * (2 if f64 else 1)
        achieved = bytes_launch / (dms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(achieved / PEAK_HBM_GBS, 4), "traffic": None,
                    "algorithmic_bytes_per_launch": bytes_launch}
    else:
        achieved = dlayer.flop_per_pass / (dms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": peak,
                    "unit": "TFLOP/s", "frac": round(achieved / peak, 4), "traffic": None}
    roofline.update({"kernel": kernel_names.get(dp, dp), "layer": dl, "pass": dp, "avg_ms": round(dms, 5),
                     "algorithmic_gflop_per_launch": dlayer.flop_per_pass / 1e9})
    traffic_file = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):  # measured separately with rocprofv3 --pmc (see profiles/)
        try:
            tr = json.load(open(traffic_file))
            roofline["traffic"] = tr.get(("f64/" if f64 else "") + f"{dl}:{dp}")
            if roofline["traffic"] is None and dp == "bwd_filter_bias":  # the same kernel without the row sums
                roofline["traffic"] = tr.get(f"{dl}:bwd_filter")
            # not measured in this run: the figure of the committed rocprofv3 --pmc summary
            roofline["traffic_from"] = "profiles/hbm_traffic.json"
        except Exception:
            pass

    out = {
        "metric": ("inner-product fwd+bwd GFLOP/s (forward + ReLU backward + backward data + backward filter + "
                   "backward bias), fp32") if is_ip else
                  "conv fwd+bwd GFLOP/s (forward + backward data + backward filter + backward bias), "
                  + ("fp64" if f64 else "fp32"),
        "bias_gradient": "from the backward-filter pass's read of dy (conv_backward_filter_bias)" if fused_bias else
                         "a pass of its own (conv_backward_bias)",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: layers " + ",".join(l.name for l in layers)
                               + " (N=%d each), %s, beta=0, bias=0" % (layers[0].m if is_ip else layers[0].n,
                                                                       "+".join(passes)),
                   "frac_of_%s_mfma_peak" % ("fp64" if f64 else "fp32"): round(value / 1e3 / peak, 4),
                   "cache": ("cold: %s tensor sets per layer rotated every step"
                             % "/".join(str(len(t["sets"])) for t in state)) if args.cold_cache
                            else "warm: the same tensors every step",
                   "empty_dispatch_us": round(launch_us, 2),
                   "mfma_register_loop": mfma_loop,
                   "per_layer_from": "%d untimed steps with HIP events around every pass; the timed steps carry "
                                     "events around the roofline kernel's pass only" % table_steps},
        "roofline": roofline,
        "per_layer": per_layer,
    }

    if args.workload == "config4" and not f64 and not args.cold_cache and not args.no_cpu_baseline:
        # The eight layer shapes of configurations 0-3, from steps of their own outside the timed region:
        # they are launch-latency bound (microseconds of work per pass), so each pass is given with its
        # launch count and its time over that many empty dispatches, next to both roofline fractions.
        out["per_layer_small"] = small_layers(torch, conv, workloads, dev, launch_us)
    if not is_ip and not args.no_cpu_baseline:
        # context only (never `value`): the same steps with the filter and bias gradients on a second stream
        two = time_two_streams(args.steps, 3)
        out["two_streams"] = {"value": round(flop_step * args.steps / two / 1e9, 1), "unit": "GFLOP/s",
                              "ms_per_step": round(two / args.steps * 1e3, 4),
                              "schedule": "forward chain, then backward data on the launch stream with backward "
                                          "filter + backward bias of the same layers on a second stream"}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_ip(layers) if is_ip else cpu_baseline(layers, args.cpu_sample_images)
    print(json.dumps(out))


def launches_of(names):
    """pass -> kernel launches, from the (S=..,L=..) suffix of a descriptor's kernel names."""
    import re
    out = {}
    for kv in names.split(";"):
        k, v = kv.split("=", 1)
        m = re.search(r",L=(\d+)\)$", v)
        if m:
            out[k] = int(m.group(1))
    return out


def small_layers(torch, conv, workloads, dev, launch_us, steps=20, warmup=5):
    """Per-pass times of layers 1.a ... 4.c (fp32): HIP events around every pass over `steps` steps,
    each layer on its own tensors resident in HBM; per configuration also the time of whole steps
    enqueued back to back without events."""
    import math
    stream = torch.cuda.current_stream()
    rows, per_config = [], {}
    for cfg in range(4):
        layers = [l for l in workloads.LAYERS if l.config == cfg]
        state = []
        ws_bytes = 0
        for l in layers:
            d = conv.conv_desc_create(conv.ConvParams(**l.params_dict()))
            ws_bytes = max(ws_bytes, conv.conv_desc_workspace_bytes(d))
            x, w, b, dy = workloads.layer_inputs(l, bias="zero")
            state.append(dict(layer=l, desc=d, x=x.to(dev), w=w.to(dev), b=b.to(dev), dy=dy.to(dev),
                              y=torch.empty(l.y_shape, device=dev), dx=torch.empty(l.x_shape, device=dev),
                              dw=torch.empty(l.w_shape, device=dev), db=torch.empty(l.k, device=dev)))
        ws = torch.empty(max(ws_bytes // 4, 1), device=dev)
        calls = {
            "fwd": lambda t: conv.conv_forward(t["desc"], t["x"], t["w"], t["b"], t["y"], ws, stream),
            "bwd_data": lambda t: conv.conv_backward_data(t["desc"], t["w"], t["dy"], t["dx"], ws, stream),
            "bwd_filter_bias": lambda t: conv.conv_backward_filter_bias(t["desc"], t["x"], t["dy"], t["dw"], t["db"],
                                                                        0.0, ws, stream),
        }

        def step(events=None):
            for t in state:
                for name, fn in calls.items():
                    if events is None:
                        fn(t)
                    else:
                        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                        e0.record(stream)
                        fn(t)
                        e1.record(stream)
                        events.append((t["layer"].name, name, e0, e1))

        for _ in range(warmup):
            step()
        events = []
        for _ in range(steps):
            step(events)
        torch.cuda.synchronize()
        acc = {}
        for lname, pname, e0, e1 in events:
            acc.setdefault((lname, pname), []).append(e0.elapsed_time(e1))
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        flop_step = 3 * sum(l.flop_per_pass for l in layers)
        per_config["config%d" % cfg] = {"us_per_step": round(wall / steps * 1e6, 1),
                                        "tflops": round(flop_step * steps / wall / 1e12, 3),
                                        "frac_of_fp32_mfma_peak": round(flop_step * steps / wall / 1e12
                                                                        / PEAK_FP32_MFMA_TFLOPS, 4)}
        for t in state:
            l = t["layer"]
            names = conv.conv_desc_kernel_names(t["desc"])
            launches = launches_of(names)
            row = {"layer": l.name, "gflop_per_pass": round(l.flop_per_pass / 1e9, 4), "kernels": names}
            tot = 0.0
            for name in calls:
                v = sorted(acc[(l.name, name)])
                us = v[len(v) // 2] * 1e3  # median
                tot += us
                nl = launches["bwd_filter" if name == "bwd_filter_bias" else name]
                p = {"us": round(us, 2), "launches": nl, "us_over_launch_floor": round(us - nl * launch_us, 2),
                     "tflops": round(l.flop_per_pass / us / 1e6, 2), "alg_GBps": round(blob_bytes(l, name) / us / 1e3, 1)}
                row[name] = p
            alg = 3 * blob_bytes(l, "fwd")
            row.update({"fwd_bwd_us": round(tot, 2), "launches": sum(row[name]["launches"] for name in calls),
                        "fwd_bwd_tflops": round(3 * l.flop_per_pass / tot / 1e6, 2),
                        "frac_of_fp32_mfma_peak": round(3 * l.flop_per_pass / tot / 1e6 / PEAK_FP32_MFMA_TFLOPS, 4),
                        "frac_of_hbm_peak": round(alg / tot / 1e3 / PEAK_HBM_GBS, 4),
                        "us_at_mfma_peak": round(3 * l.flop_per_pass / PEAK_FP32_MFMA_TFLOPS / 1e6, 2),
                        "us_at_hbm_peak": round(alg / PEAK_HBM_GBS / 1e3, 2)})
            rows.append(row)
    return {"empty_dispatch_us": round(launch_us, 2), "bound": "latency: two or three kernels of 3-30 us per pass, back to back (a step takes the sum of their durations)",
            "from": "%d steps per configuration with HIP events around every pass (median); us_per_step from %d "
                    "steps enqueued back to back without events" % (steps, steps),
            "per_config": per_config, "layers": rows}


def bench_pg(args, torch, lib, workloads, dev):
    """Policy-gradient loss step (paper Appendix A/B) over one batch of finished episodes: action
    sampling, discounted rewards, Sigmoid Bottom.diff, Softmax Bottom.diff (+probabilities).
    Everything is HBM-bound: the metric is algorithmic bytes moved per second."""
    episodes, lo, hi, actions = workloads.PG_BENCH
    gamma = 0.99
    offsets, reward, aprob, random, logits, action = workloads.pg_batch(episodes, lo, hi, actions, workloads.PG_SEED)
    steps = reward.numel()
    d = {k: v.to(dev) for k, v in dict(offsets=offsets, reward=reward, aprob=aprob, random=random, logits=logits,
                                       action=action).items()}
    out = dict(act=torch.empty(steps, dtype=torch.int32, device=dev), R=torch.empty(steps, device=dev),
               bd=torch.empty(steps, device=dev), probs=torch.empty((steps, actions), device=dev),
               sbd=torch.empty((steps, actions), device=dev))
    stream = torch.cuda.current_stream()
    # algorithmic bytes per time step: every input read once, every output written once
    passes = {
        "sample_action": (lambda: lib.pg_sigmoid_sample_action(d["aprob"], d["random"], out["act"], stream), 12),
        "discount_rewards": (lambda: lib.pg_discount_rewards(d["reward"], d["offsets"], gamma, out["R"], stream), 8),
        "sigmoid_bottom_diff": (lambda: lib.pg_sigmoid_bottom_diff(d["aprob"], out["act"], out["R"], None, out["bd"],
                                                                   stream), 16),
        "softmax_bottom_diff": (lambda: lib.pg_softmax_bottom_diff(d["logits"], d["action"], out["R"], out["probs"],
                                                                   out["sbd"], stream), 8 + 12 * actions),
    }

    def step(events=None, only=None):
        for name, (fn, _) in passes.items():
            if events is None or (only is not None and only != name):
                fn()
            else:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                fn()
                e1.record(stream)
                events.append((name, e0, e1))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # per-pass times from untimed steps with events around every pass; the timed steps carry events
    # around the slowest pass only (an event pair costs about as much as the shortest kernels here)
    events = []
    for _ in range(max(3, min(args.steps, 10))):
        step(events)
    torch.cuda.synchronize()
    acc = {}
    for name, e0, e1 in events:
        acc.setdefault(name, []).append(e0.elapsed_time(e1))
    per_pass = {}
    for name, (_, bps) in passes.items():
        ms = sum(acc[name]) / len(acc[name])
        per_pass[name] = {"ms": round(ms, 5), "GBps": round(bps * steps / ms / 1e6, 1), "bytes_per_step": bps}
    dom = max(per_pass, key=lambda k: per_pass[k]["ms"])
    dom_events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(dom_events, dom)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dom_ms = sum(e0.elapsed_time(e1) for _, e0, e1 in dom_events) / len(dom_events)
    dom_gbps = round(passes[dom][1] * steps / dom_ms / 1e6, 1)
    bytes_step = sum(b for _, b in passes.values()) * steps
    value = bytes_step * args.steps / wall / 1e9
    res = {
        "metric": "policy-gradient loss step (sample action + discounted rewards + Sigmoid and Softmax Bottom.diff), "
                  "algorithmic GB/s, fp32",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"pg: {episodes} episodes of {lo}..{hi} steps = {steps} time steps, {actions} actions, "
                               f"gamma {gamma}", "time_steps_per_s": round(steps * args.steps / wall, 1)},
        "roofline": {"bound": "hbm", "achieved": dom_gbps, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": round(dom_gbps / PEAK_HBM_GBS, 4), "traffic": pg_traffic(dom), "kernel": dom,
                     "avg_ms": round(dom_ms, 5)},
        "per_pass": per_pass,
    }
    if not args.no_cpu_baseline:
        import numpy as np

        from oracle import policy_gradient as pgo
        n = min(steps, int(offsets[min(episodes, 8192)]))  # the first 8192 episodes
        off = offsets[:min(episodes, 8192) + 1].numpy()
        f64 = lambda t: t[:n].numpy().astype(np.float64)
        c0 = time.perf_counter()
        act = pgo.sigmoid_sample_action(f64(aprob), f64(random))
        R = pgo.discount_rewards(f64(reward), off, gamma)
        pgo.bottom_diff(pgo.sigmoid_dlogps(f64(aprob), act), R, True)
        _, dl = pgo.softmax_dlogps(f64(logits), action[:n].numpy())
        pgo.bottom_diff(dl, R, False)
        secs = time.perf_counter() - c0
        res["cpu_baseline"] = {"value": round(sum(b for _, b in passes.values()) * n / secs / 1e9, 3), "unit": "GB/s",
                               "cores": 1, "kind": "oracle",
                               "sample": f"first {len(off) - 1} episodes ({n} time steps), same fp32-sized byte count, "
                                         f"double-precision loops, {secs:.1f} s"}
    print(json.dumps(res))


def pg_traffic(pass_name):
    """HBM bytes of one pg pass as measured separately with rocprofv3 --pmc (see profiles/), or None."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "hbm_traffic.json")
    try:
        return json.load(open(path)).get(f"pg:{pass_name}")
    except Exception:
        return None


def blob_bytes(l, pass_name):
    """fp32 bytes of the blobs one pass of a convolution layer reads and writes, each once."""
    import math
    x, y, w = (math.prod(s) for s in (l.x_shape, l.y_shape, l.w_shape))
    return 4 * (x + y + w)  # two of them read, the third written, whichever the pass


def dy_bytes(l):
    """Bytes of the top gradient blob of a conv or ip layer."""
    if hasattr(l, "out_hw"):
        return 4.0 * l.n * l.k * l.out_hw * l.out_hw
    return 4.0 * l.m * l.num_output


def cpu_baseline_ip(layers):
    """The CPU InnerProduct oracle, as it stands, on the full batch of each layer of the workload."""
    import numpy as np

    from oracle import inner_product as ipo
    from paper_1810_02272_amd import workloads

    flop, secs, per_layer = 0.0, 0.0, {}
    for l in layers:
        op = ipo.IpOracleParams(**l.params_dict())
        x, w, b, dy = (t.numpy().astype(np.float64) for t in workloads.ip_inputs(l, bias="zero"))
        t0 = time.perf_counter()
        y = ipo.forward(op, x, w, b)
        dz = ipo.relu_backward(op, y, dy)
        ipo.backward_data(op, w, dz)
        ipo.backward_filter(op, x, dz)
        ipo.backward_bias(op, dz)
        dt = time.perf_counter() - t0
        secs += dt
        flop += 3.0 * l.flop_per_pass
        per_layer[l.name] = round(3.0 * l.flop_per_pass / dt / 1e9, 3)
    return {"value": round(flop / secs / 1e9, 3), "unit": "GFLOP/s", "cores": ipo.num_threads(), "kind": "oracle",
            "per_layer_gflops": per_layer,
            "sample": f"all rows of each layer, fwd+relu_bwd+bwd_data+bwd_filter+bwd_bias, double-precision loops, "
                      f"{secs:.1f} s"}


def cpu_baseline(layers, n_sample):
    """The CPU oracle, as it stands, on the first n_sample images of each layer of the workload."""
    import numpy as np

    import oracle
    from oracle import OracleParams
    from paper_1810_02272_amd import workloads

    flop = 0.0
    secs = 0.0
    per_layer = {}
    for l in layers:
        n = min(n_sample, l.n)
        pd = l.params_dict()
        pd["n"] = n
        op = OracleParams(**pd)
        x, w, b, dy = workloads.layer_inputs(l, bias="zero")
        x, dy = x[:n].numpy().astype(np.float64), dy[:n].numpy().astype(np.float64)
        w, b = w.numpy().astype(np.float64), b.numpy().astype(np.float64)
        t0 = time.perf_counter()
        oracle.forward(op, x, w, b)
        oracle.backward_data(op, w, dy)
        oracle.backward_filter(op, x, dy)
        oracle.backward_bias(op, dy)
        dt = time.perf_counter() - t0
        secs += dt
        flop += 3.0 * l.flop_per_pass * n / l.n
        per_layer[l.name] = round(3.0 * l.flop_per_pass * n / l.n / dt / 1e9, 3)
    return {"value": round(flop / secs / 1e9, 3), "unit": "GFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "per_layer_gflops": per_layer,
            "sample": f"first {n_sample} images of each layer, fwd+bwd_data+bwd_filter+bwd_bias, "
                      f"double-precision nested loops, {secs:.1f} s"}


if __name__ == "__main__":
    main()
