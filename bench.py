#!/usr/bin/env python3
"""Benchmark of the DeepPoly back-substitution hot path on one MI355X.

One "step" = one full DeepPoly pass (box -> bounds of every layer) over ALL inputs of the
workload, batched into the same kernel launches, with the inputs already in device memory.
Workload: the FC 9x500 configuration (the one the metric is quoted on), 100 synthetic inputs.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_FP64_MFMA_TFLOPS = 78.6      # MI355X published dense float64 matrix peak


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=1, help="index into the five synthetic configurations")
    ap.add_argument("--workload", default="", help="a named workload outside the five configurations (lenet_pool) instead of --config")
    ap.add_argument("--batch", type=int, default=0, help="inputs per pass (default: all inputs of the configuration)")
    ap.add_argument("--calib-copy-mb", type=int, default=0, help="run one plain device copy of this many MiB first (scale for HBM counters)")
    ap.add_argument("--dump", default="", help="write one CSV line per profiled kernel launch to this file")
    ap.add_argument("--early-term", action="store_true",
                    help="analyse with early termination (forward interval pass, stable neurons are not back-substituted)")
    ap.add_argument("--float-inference", action="store_true",
                    help="bounds that also cover every float32 evaluation order of the network (inference rounding)")
    ap.add_argument("--graph", action="store_true", help="replay the pass as a captured HIP graph")
    ap.add_argument("--coef-bits", type=int, default=32, choices=(32, 64),
                    help="storage of the coefficient blocks: float32 (default, the headline configuration) or float64")
    ap.add_argument("--weight-scale", type=float, default=1.0,
                    help="multiply every weight by this factor (well below 1: most ReLUs stable, as in robustly trained nets)")
    ap.add_argument("--eps", type=float, default=0.0, help="override the configuration's perturbation radius")
    ap.add_argument("--cpu-sample", type=int, default=-1, help="inputs the oracle is timed on (0: skip)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as wl
    from paper_2007_10868_amd import Net

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload:
        net = {"lenet_pool": wl.lenet_pool}[args.workload]()
    else:
        net = wl.config(args.config)
    if args.weight_scale != 1.0:
        net = wl.contracted(net, args.weight_scale)
    if args.eps > 0:
        net.eps = args.eps
    batch = args.batch or net.n_inputs
    g = Net(*net.input_shape)
    wl.build_into(net, g)
    if args.early_term:
        g.set_early_termination(True)
    if args.float_inference:
        g.set_float_inference(True)
    if args.graph:
        g.set_graph_replay(True)
    if args.coef_bits == 64:
        g.set_coefficient_storage(64)
    centers = np.stack([net.center(j % net.n_inputs) for j in range(batch)])
    t_centers = torch.tensor(centers, device="cuda")
    stream = torch.cuda.current_stream()
    g.set_stream(stream)
    _, full = g.workspace_size(batch)
    free, _ = torch.cuda.mem_get_info()
    ws_bytes = int(min(full, free * 0.6))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    g.set_workspace(ws)

    if args.calib_copy_mb > 0:          # a copy kernel of known size: reads and writes exactly this many bytes
        src = torch.ones(args.calib_copy_mb << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        g.analyze_batch_dev(t_centers, net.eps)
    torch.cuda.synchronize()
    if not args.graph:                  # per-kernel events are recorded on eager launches only
        g.profile_enable(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        g.analyze_batch_dev(t_centers, net.eps)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    if args.dump:
        g.profile_dump(args.dump)
    prof = g.profile_read()
    g.profile_enable(False)
    early = None
    if args.early_term:
        done, full_flop = g.early_termination_stats()
        early = dict(crossing_flop_done=done, crossing_flop_without_removal=full_flop,
                     fraction=round(done / full_flop, 4) if full_flop > 0 else None)
    ms_per_step = wall_ms / args.steps
    ms_per_input = ms_per_step / batch

    # one input at a time (what a caller without a batch sees); not the metric, reported beside it
    single_ms = None
    if batch > 1:
        one = t_centers[:1].contiguous()
        for _ in range(3):
            g.analyze_batch_dev(one, net.eps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 10
        for _ in range(reps):
            g.analyze_batch_dev(one, net.eps)
        torch.cuda.synchronize()
        single_ms = (time.perf_counter() - t0) * 1e3 / reps

    # the same K steps replayed as one captured HIP graph per pass (no per-kernel events there, so this is reported
    # beside the metric, which stays the eager, event-instrumented region above)
    graph_ms = None
    graph_single_ms = None
    if not args.graph and not args.early_term and ms_per_step < 2000.0:
        g.set_graph_replay(True)
        for _ in range(2):
            g.analyze_batch_dev(t_centers, net.eps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.analyze_batch_dev(t_centers, net.eps)
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        if batch > 1:                      # ... and one input at a time, replayed
            for _ in range(3):
                g.analyze_batch_dev(one, net.eps)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                g.analyze_batch_dev(one, net.eps)
            torch.cuda.synchronize()
            graph_single_ms = (time.perf_counter() - t0) * 1e3 / 10
        g.set_graph_replay(False)

    cross = prof["cross"]
    avg_launch_ms = cross["ms"] / max(cross["launches"], 1)
    flop_per_launch = cross["flop"] / max(cross["launches"], 1)
    achieved = flop_per_launch / (avg_launch_ms * 1e-3) / 1e12 if avg_launch_ms > 0 else 0.0
    traffic = None
    tfile = os.path.join(ROOT, "profiles", f"cross_kernel_{net.name}_traffic.json")
    if os.path.exists(tfile) and batch == net.n_inputs:      # counters of a committed rocprofv3 --pmc run of this workload
        traffic = json.load(open(tfile)).get("hbm_bytes_per_launch")
    roofline = dict(bound="mfma", kernel="cross_kernel (float64 MFMA implicit GEMM; all crossing launches of a pass)", achieved=round(achieved, 3),
                    peak=PEAK_FP64_MFMA_TFLOPS, unit="TFLOP/s", frac=round(achieved / PEAK_FP64_MFMA_TFLOPS, 4),
                    traffic=traffic, launches_per_step=cross["launches"] // args.steps,
                    avg_launch_us=round(avg_launch_ms * 1e3, 2), alg_flop_per_launch=flop_per_launch,
                    alg_bytes_per_launch=cross["bytes"] / max(cross["launches"], 1),
                    kernel_time_share=round(cross["ms"] / gpu_ms, 4),
                    scan_kernel_time_share=round(prof["scan"]["ms"] / gpu_ms, 4))

    # ---- the oracle, as it stands, on the host cores of this machine, on a bounded sample of the workload
    cpu = None
    n_cpu = args.cpu_sample if args.cpu_sample >= 0 else (1 if args.workload else {0: 10, 1: 10, 2: 10, 3: 1, 4: 0}[args.config])
    if n_cpu > 0:
        from oracle import OracleNet, oracle_threads
        o = OracleNet(*net.input_shape)
        wl.build_into(net, o)
        t0 = time.perf_counter()
        for j in range(n_cpu):
            if args.early_term:
                o.set_early_termination(True)
            if args.float_inference:
                o.set_float_inference(True)
            o.analyze(net.center(j), net.eps)
        cpu_ms = (time.perf_counter() - t0) * 1e3 / n_cpu
        cpu = dict(value=round(cpu_ms, 3), unit="ms/input", cores=oracle_threads(), kind="oracle",
                   sample=f"full DeepPoly pass of the float64 outward-rounded C oracle on the first {n_cpu} inputs of {net.name}")

    out = dict(metric="ms per input for full DeepPoly pass", value=round(ms_per_input, 5), unit="ms/input",
               n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=round(ms_per_step, 4),
               gpu_ms_per_step=round(gpu_ms / args.steps, 4),
               higher_is_better=False, scaling="weak", vs_baseline=None, dtype="f64", data="synthetic",
               config=dict(workload=net.name, inputs_per_step=batch, eps=net.eps, neurons=int(sum(net.n_neurons(i) for i in range(1, net.out_layer + 1) if net.layers[i - 1]["type"] != "relu")),
                           coefficient_storage="f64" if args.coef_bits == 64 else "f32", accumulate="f64 MFMA", workspace_bytes=ws_bytes,
                           early_termination=bool(args.early_term), float_inference=bool(args.float_inference),
                           graph_replay=bool(args.graph)),
               roofline=roofline, cpu_baseline=cpu)
    if single_ms is not None:
        out["single_input_latency_ms"] = round(single_ms, 4)
    if graph_ms is not None:
        out["graph_replay"] = dict(ms_per_step=round(graph_ms, 4), ms_per_input=round(graph_ms / batch, 5))
        if graph_single_ms is not None:
            out["graph_replay"]["single_input_latency_ms"] = round(graph_single_ms, 4)
    if early is not None:
        out["early_termination"] = early
    print(json.dumps(out))


if __name__ == "__main__":
    main()
