#!/usr/bin/env python3
"""Benchmark of the DeepPoly back-substitution hot path on one MI355X.

One "step" = one full DeepPoly pass (box -> bounds of every layer) over ALL inputs of the
workload, batched into the same kernel launches, with the inputs already in device memory.
Headline workload: the FC 9x500 configuration, 100 synthetic inputs (`value`).  Without --config or
--workload the other four synthetic configurations are measured as well and reported under
`configs` in the same JSON line, each with its own roofline and CPU-oracle figures.
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

# (steps, warm-up passes) of the configurations measured beside the headline one; inputs the oracle is timed on
SIDE_RUNS = {0: (20, 3), 2: (20, 3), 3: (5, 1), 4: (1, 1)}
CPU_SAMPLE = {0: 10, 1: 5, 2: 10, 3: 1, 4: 1}
CPU_ROWS_PER_LAYER = 16           # configuration 4: rows of each layer the oracle bounds (teacher forcing)


def analysed_start_layers(net):
    """Layers whose neurons are back-substituted: inputs of ReLU layers and the last layer."""
    feeds = {L["src"] for L in net.layers if L["type"] == "relu"}
    return [i for i, L in enumerate(net.layers, start=1) if L["type"] != "relu" and (i in feeds or i == len(net.layers))]


def oracle_full(args, net, wl, n_cpu):
    """The oracle as it stands, whole passes on the first n_cpu inputs."""
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
    return dict(value=round(cpu_ms, 3), unit="ms/input", cores=oracle_threads(), kind="oracle", extrapolated=False,
                sample=f"full DeepPoly pass of the float64 outward-rounded C oracle on the first {n_cpu} inputs of {net.name}")


def oracle_sampled_rows(net, wl, g, rows_per_layer):
    """A whole oracle pass over the 1M-neuron net takes hours: the oracle is handed the library's intervals of all
    earlier layers as data and bounds `rows_per_layer` evenly spaced rows of every analysed layer; a layer's time is
    scaled by rows_total / rows_sampled and the layers are summed.  Labelled as extrapolated."""
    import numpy as np
    from oracle import OracleNet, oracle_threads
    o = OracleNet(*net.input_shape)
    wl.build_into(net, o)
    o.set_ball(net.center(0), net.eps)
    starts = set(analysed_start_layers(net))
    total_ms, sampled, rows_total = 0.0, 0, 0
    for lid in range(1, o.num_layers):
        if net.layers[lid - 1]["type"] == "relu":
            o.analyze_layer(lid)
            continue
        if lid not in starts:
            continue
        glo, ghi = g.get_bounds_f64(lid, 0)
        n = glo.size
        rows = np.unique(np.linspace(0, n - 1, min(rows_per_layer, n)).astype(np.int32))
        t0 = time.perf_counter()
        o.bound_rows(lid, rows)
        dt = (time.perf_counter() - t0) * 1e3
        total_ms += dt * n / rows.size
        sampled += rows.size
        rows_total += n
        o.set_bounds(lid, glo, ghi)
    return dict(value=round(total_ms, 1), unit="ms/input", cores=oracle_threads(), kind="oracle", extrapolated=True,
                sample=f"{sampled} of {rows_total} rows of {net.name}: {rows_per_layer} evenly spaced rows of each of the {len(starts)} "
                       "back-substituted layers, bounded by the C oracle given the library's intervals of all earlier layers; "
                       "per layer time x rows_total / rows_sampled, summed (extrapolated)")


def measure(args, cfg, net, batch, steps, warmup, extras, n_cpu):
    """One workload: timed passes, per-kernel events, optional latency / graph-replay figures, oracle timing."""
    import numpy as np
    import torch
    import workloads as wl
    from paper_2007_10868_amd import Net

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

    for _ in range(warmup):
        g.analyze_batch_dev(t_centers, net.eps)
    torch.cuda.synchronize()
    if not args.graph:                  # per-kernel events are recorded on eager launches only
        g.profile_enable(True)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps):
        g.analyze_batch_dev(t_centers, net.eps)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    gpu_ms = e0.elapsed_time(e1)
    if args.dump and extras:
        g.profile_dump(args.dump)
    prof = g.profile_read()
    g.profile_enable(False)
    early = None
    if args.early_term:
        done, full_flop = g.early_termination_stats()
        # share of the ReLU inputs of the first box whose sign is decided (the regime Section 3.2 speaks about)
        n_relu_in, n_stable = 0, 0
        for L in net.layers:
            if L["type"] == "relu":
                lo, hi = g.get_bounds_f64(L["src"], 0)
                n_relu_in += lo.size
                n_stable += int(np.sum((lo >= 0) | (hi <= 0)))
        early = dict(crossing_flop_done=done, crossing_flop_without_removal=full_flop,
                     fraction=round(done / full_flop, 4) if full_flop > 0 else None,
                     stable_relu_inputs=round(n_stable / max(n_relu_in, 1), 4))
    ms_per_step = wall_ms / steps
    ms_per_input = ms_per_step / batch

    # one input at a time (what a caller without a batch sees); not the metric, reported beside it
    single_ms = None
    if batch > 1 and extras:
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
    if extras and not args.graph and not args.early_term and ms_per_step < 2000.0:
        g.set_graph_replay(True)
        for _ in range(2):
            g.analyze_batch_dev(t_centers, net.eps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            g.analyze_batch_dev(t_centers, net.eps)
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
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
        g.analyze_batch_dev(t_centers, net.eps)       # bounds of the whole batch again (the oracle leg may read them)

    cross = prof["cross"]
    avg_launch_ms = cross["ms"] / max(cross["launches"], 1)
    flop_per_launch = cross["flop"] / max(cross["launches"], 1)
    achieved = flop_per_launch / (avg_launch_ms * 1e-3) / 1e12 if avg_launch_ms > 0 else 0.0
    traffic, traffic_source = None, None
    tname = f"cross_kernel_{net.name}_traffic.json"
    tfile = os.path.join(ROOT, "profiles", tname)
    if os.path.exists(tfile) and batch == net.n_inputs:      # counters of a committed rocprofv3 --pmc run of this workload
        traffic = json.load(open(tfile)).get("hbm_bytes_per_launch")
        traffic_source = f"profiles/{tname} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command; not measured in this run)"
    roofline = dict(bound="mfma", kernel="affine crossing kernels (float64 MFMA implicit GEMM; all crossing launches of a pass)",
                    achieved=round(achieved, 3), peak=PEAK_FP64_MFMA_TFLOPS, unit="TFLOP/s", frac=round(achieved / PEAK_FP64_MFMA_TFLOPS, 4),
                    traffic=traffic, traffic_source=traffic_source, launches_per_step=cross["launches"] // steps,
                    avg_launch_us=round(avg_launch_ms * 1e3, 2), alg_flop_per_launch=flop_per_launch,
                    alg_bytes_per_launch=cross["bytes"] / max(cross["launches"], 1),
                    kernel_time_share=round(cross["ms"] / gpu_ms, 4),
                    scan_kernel_time_share=round(prof["scan"]["ms"] / gpu_ms, 4))

    # ---- the oracle, as it stands, on the host cores of this machine, on a bounded sample of the workload
    cpu = None
    if n_cpu > 0:
        if cfg == 4 and not args.early_term and not args.float_inference and args.weight_scale == 1.0:
            cpu = oracle_sampled_rows(net, wl, g, CPU_ROWS_PER_LAYER)
        else:
            cpu = oracle_full(args, net, wl, n_cpu)

    neurons = int(sum(net.n_neurons(i) for i in range(1, net.out_layer + 1) if net.layers[i - 1]["type"] != "relu"))
    res = dict(ms_per_input=ms_per_input, ms_per_step=ms_per_step, gpu_ms_per_step=gpu_ms / steps, steps=steps, warmup=warmup,
               batch=batch, neurons=neurons, ws_bytes=ws_bytes, roofline=roofline, cpu=cpu, single_ms=single_ms, graph_ms=graph_ms,
               graph_single_ms=graph_single_ms, early=early)
    del g, ws, t_centers
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=-1,
                    help="index into the five synthetic configurations: measure that one only (default: FC 9x500 as the "
                         "headline and the other four beside it)")
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

    import torch
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    all_configs = args.config < 0 and not args.workload
    cfg = 1 if args.config < 0 else args.config
    if args.workload:
        cfg = -1
        net = {"lenet_pool": wl.lenet_pool}[args.workload]()
    else:
        net = wl.config(cfg)
    if args.weight_scale != 1.0:
        net = wl.contracted(net, args.weight_scale)
    if args.eps > 0:
        net.eps = args.eps
    batch = args.batch or net.n_inputs

    if args.calib_copy_mb > 0:          # a copy kernel of known size: reads and writes exactly this many bytes
        src = torch.ones(args.calib_copy_mb << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    n_cpu = args.cpu_sample if args.cpu_sample >= 0 else (1 if args.workload else CPU_SAMPLE[cfg])
    r = measure(args, cfg, net, batch, args.steps, args.warmup, True, n_cpu)

    out = dict(metric="ms per input for full DeepPoly pass", value=round(r["ms_per_input"], 5), unit="ms/input",
               n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=round(r["ms_per_step"], 4),
               gpu_ms_per_step=round(r["gpu_ms_per_step"], 4),
               higher_is_better=False, scaling="weak", vs_baseline=None, dtype="f64", data="synthetic",
               config=dict(workload=net.name, inputs_per_step=batch, eps=net.eps, neurons=r["neurons"],
                           coefficient_storage="f64" if args.coef_bits == 64 else "f32", accumulate="f64 MFMA", workspace_bytes=r["ws_bytes"],
                           early_termination=bool(args.early_term), float_inference=bool(args.float_inference),
                           graph_replay=bool(args.graph)),
               roofline=r["roofline"], cpu_baseline=r["cpu"])
    if r["single_ms"] is not None:
        out["single_input_latency_ms"] = round(r["single_ms"], 4)
    if r["graph_ms"] is not None:
        out["graph_replay"] = dict(ms_per_step=round(r["graph_ms"], 4), ms_per_input=round(r["graph_ms"] / batch, 5))
        if r["graph_single_ms"] is not None:
            out["graph_replay"]["single_input_latency_ms"] = round(r["graph_single_ms"], 4)
    if r["early"] is not None:
        out["early_termination"] = r["early"]

    if all_configs:
        # the five synthetic configurations side by side, each batched over all of its inputs; the 1M-neuron residual
        # net runs one input per pass, one warm-up and one timed pass
        entries = []
        for c in range(5):
            if c == cfg:
                rr, nn, bb = r, net, batch
            else:
                nn = wl.config(c)
                bb = 1 if c == 4 else nn.n_inputs
                steps, warm = SIDE_RUNS[c]
                rr = measure(args, c, nn, bb, steps, warm, False, CPU_SAMPLE[c] if args.cpu_sample != 0 else 0)
            rf = rr["roofline"]
            entries.append(dict(workload=nn.name, inputs_per_step=bb, neurons=rr["neurons"], steps=rr["steps"], warmup=rr["warmup"],
                                ms_per_input=round(rr["ms_per_input"], 5), ms_per_step=round(rr["ms_per_step"], 4),
                                roofline=dict(bound=rf["bound"], kernel=rf["kernel"], achieved=rf["achieved"], peak=rf["peak"],
                                              unit=rf["unit"], frac=rf["frac"], launches_per_step=rf["launches_per_step"],
                                              kernel_time_share=rf["kernel_time_share"]),
                                cpu_baseline=rr["cpu"]))
        out["configs"] = entries
    print(json.dumps(out))


if __name__ == "__main__":
    main()
