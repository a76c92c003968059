#!/usr/bin/env python3
"""Throughput of the CaffeNet-shaped convolution stack on one MI355X.

One step = conv1..conv5 (ReLU fused, 3x3/2 max-pools after conv1, conv2, conv5) forward, backward
(data and model gradients; conv1's data gradient skipped as in the paper's FLOP rule, App. B) and
one momentum-SGD update, at batch 256 in bf16 storage with fp32 accumulation, on seeded synthetic
tensors already resident in HBM.  Prints ONE JSON line with images/s, the roofline of the dominant
kernel (timed with HIP events on the launch stream inside the timed region) and the CPU oracle's
rate on a bounded sample of the same workload.

After the timed region the same K steps are replayed as one captured HIP graph and reported beside it
(`graph_replay`: launch gaps removed; the headline value stays the eager one, whose kernels carry the events).

Order of work: warm-up steps; a few instrumented steps with events around EVERY launch (they give the
per-kernel table and name the dominant kernel class; the ~100 event records per step cost about a
tenth of the step, so this pass is not the timed one); then the timed region, in which only the dominant
class is bracketed by events -- its average launch duration in the roofline comes from there (when that
class is one of the matrix-core classes, all of them are bracketed, so that the line also carries the
rate of all the step's products together).

The steps update the weights they run on.  The upstream gradient is the seeded N(0,1) draw times a power of
two small enough that thousands of steps leave every tensor in its starting distribution; after the timed
region the tensors are read back and checked (finite, ReLU outputs about half zero, weights still N(0, 0.01))
and the run fails if they are not, so a figure from this script is a figure on the stated workload.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0
MFMA_KERNELS = ("gemm", "conv_fused", "conv_strided")          # kernel classes bound by the matrix cores
# HBM bytes per launch come from hbm_traffic.json in the package: rocprof_tables.py writes it from rocprofv3
# --pmc FETCH_SIZE / WRITE_SIZE runs of this script (scaled by the readings for the 256 MiB calibration copy
# below) together with a digest of the kernel sources; a table measured on other sources is not reported.


def measured_traffic(workload: str):
    """Kernel class -> measured HBM bytes per launch for this workload, or {} if none matches the built code."""
    from paper_1606_04487_amd import rocprof_tables as rt
    try:
        entry = json.loads(rt.TRAFFIC_JSON.read_text()).get(workload)
    except (OSError, ValueError):
        return {}, "no traffic table"
    if entry is None:
        return {}, "no traffic table for this workload"
    if entry.get("sources") != rt.sources_digest():
        return {}, f"traffic table {entry.get('summary')} was measured on other kernel sources"
    return entry["bytes_per_launch"], entry.get("summary")


def host_cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(sample_images: int):
    """The oracle, as it stands, on `sample_images` images of the same five layers (all three passes)."""
    import oracle
    from paper_1606_04487_amd import workloads as wl
    layers = wl.caffenet_stack(sample_images)
    tensors = [(L, wl.layer_tensors(L, seed=1, bf16=True)) for L in layers]
    t0 = time.perf_counter()
    for i, (L, t) in enumerate(tensors):
        s = oracle.shape(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p)
        oracle.conv_forward(s, t["X"], t["W"], t["bias"])
        oracle.conv_backward_weights(s, t["X"], t["dY"])
        oracle.bias_grad(s, t["dY"])
        if i > 0:
            oracle.conv_backward_data(s, t["dY"], t["W"])
    dt = time.perf_counter() - t0
    return {"value": sample_images / dt, "unit": "images/s", "cores": oracle.num_threads(), "kind": "oracle",
            "host_cpu": host_cpu_model(), "host_logical_cpus": os.cpu_count(),
            "sample": f"{sample_images} images through conv1-conv5 forward, model gradient and data gradient "
                      f"(conv1's data gradient skipped), direct loops in fp64, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--cpu-sample", type=int, default=64, help="images timed through the CPU oracle (0 = skip)")
    ap.add_argument("--no-events", action="store_true", help="record no events at all (no kernel table, no roofline)")
    ap.add_argument("--table-steps", type=int, default=5, help="instrumented steps before the timed region")
    ap.add_argument("--overlap", action="store_true", help="model gradients on a second stream beside the data gradients")
    ap.add_argument("--no-graph", action="store_true", help="skip the graph replay after the timed region (profiler runs)")
    ap.add_argument("--graph", action="store_true",
                    help="replay the step as one captured HIP graph (no events inside: the roofline block then comes from the instrumented steps)")
    ap.add_argument("--config", type=int, default=5, choices=[1, 2, 3, 4, 5],
                    help="workload configuration: 5 (default) is the CaffeNet-shaped stack the metric is quoted on; 1-4 are the "
                         "single layer, the CIFAR-style stack, conv1 alone and conv2-conv5 alone (per-pass times and oracle errors)")
    ap.add_argument("--conv1-dgrad", action="store_true",
                    help="also compute conv1's data gradient (the paper's FLOP rule, App. B, leaves it out; default: skipped)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1606_04487_amd import binding as B
    from paper_1606_04487_amd import workloads as wl
    from paper_1606_04487_amd.stack import ConvStack

    torch.cuda.set_device(0)
    if args.config != 5:
        from paper_1606_04487_amd import config_bench
        rec = config_bench.run_config(args.config, max(args.steps, 1))
        print(json.dumps({
            "metric": "conv fwd+bwd images/sec", "value": rec.pop("value"), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
            "warmup": 1, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "data": "synthetic",
            "dtype": "f32" if args.config != 4 else "f32+bf16", "config": {"workload": rec.pop("workload")}, **rec}))
        return
    dtype = B.BF16 if args.dtype == "bf16" else B.F32
    layers = wl.caffenet_stack(args.batch)
    stack = ConvStack(layers, dtype=dtype, ceil_mode=False, skip_first_dgrad=not args.conv1_dgrad, overlap_wgrad=args.overlap)
    data = wl.stack_tensors(layers, seed=1, bf16=(dtype == B.BF16), pooled_out=stack.output_shape()[-2:])
    stack.set_parameters(data["W"], data["bias"])
    X = torch.from_numpy(data["X"]).cuda().to(B.torch_dtype(dtype))
    # the seeded N(0,1) draw times a power of two that keeps repeated updates from blowing the weights up
    grad_scale = wl.step_upstream_scale(args.batch)
    dOut = (torch.from_numpy(data["dY"]).cuda() * grad_scale).to(B.torch_dtype(dtype))
    lr, mu = 0.01, 0.9
    W_start = [w.clone() for w in stack.W]

    # One plain device copy of known size (256 MiB read, 256 MiB written) before anything is timed: under
    # rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE readings calibrate the counters' units.
    cal_src = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    del cal_src, cal_dst

    for _ in range(args.warmup):
        stack.step(X, dOut, lr, mu)
    torch.cuda.synchronize()

    # instrumented pass: every launch bracketed, for the per-kernel table
    table_kernels, dom = {}, None
    if not args.no_events and args.table_steps > 0:
        B.profile_enable(True)
        for _ in range(args.table_steps):
            stack.step(X, dOut, lr, mu)
        torch.cuda.synchronize()
        table_kernels = B.profile_summary()
        B.profile_enable(False)
        dom = max(table_kernels, key=lambda n: table_kernels[n]["total_ms"])

    # timed region: events around the matrix-core kernel classes only (about 15 of a step's 45 launches)
    mfma_classes = [n for n in table_kernels if n.startswith(MFMA_KERNELS)]
    if dom is not None:
        B.profile_enable(True)
        B.profile_select_many(mfma_classes if dom in mfma_classes else [dom])
    # one event between steps (on the stream the steps are launched on) for the median and the spread
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    run_step = lambda: stack.step(X, dOut, lr, mu)
    if args.graph:
        # the same launches, recorded once and replayed: nothing in a step allocates, clears memory or waits
        B.profile_enable(False)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            stack.step(X, dOut, lr, mu)
        torch.cuda.synchronize()
        run_step = graph.replay
    t0 = time.perf_counter()
    marks[0].record()
    for i in range(args.steps):
        run_step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    median_ms = per_step[len(per_step) // 2] if len(per_step) % 2 else 0.5 * (per_step[len(per_step) // 2 - 1] + per_step[len(per_step) // 2])
    mean_ms = sum(per_step) / len(per_step)
    cv = (sum((t - mean_ms) ** 2 for t in per_step) / len(per_step)) ** 0.5 / mean_ms
    kernels = B.profile_summary() if dom is not None else {}
    B.profile_enable(False)
    if args.graph:
        kernels = table_kernels      # eager launches of the instrumented steps: a replayed graph carries no events

    ms_per_step = 1e3 * dt / args.steps
    images_per_s = args.batch * args.steps / dt
    flops_step = sum(3 * L.gemm_flops for L in layers)   # App. B rule: 1.6 TFLOP at 256 without conv1's data gradient
    if not args.conv1_dgrad:
        flops_step -= layers[0].gemm_flops
    workload = f"caffenet_conv1-5_relu_pool_fwd+bwd+sgd_b{args.batch}_{args.dtype}"
    traffic_table, traffic_src = measured_traffic(workload)
    roof, roof_all = None, None
    table = {}
    for name, k in table_kernels.items():
        row = {"launches_per_step": k["launches"] / args.table_steps, "avg_ms": k["total_ms"] / k["launches"],
               "ms_per_step": k["total_ms"] / args.table_steps}
        if k["flops"] > 0 and name.startswith(MFMA_KERNELS):
            row["tflops"] = k["flops"] / (k["total_ms"] * 1e-3) / 1e12
            row["frac_of_mfma_peak"] = row["tflops"] / PEAK_TFLOPS[args.dtype]
        elif k["bytes"] > 0:
            row["gbs"] = k["bytes"] / (k["total_ms"] * 1e-3) / 1e9
            row["frac_of_hbm_peak"] = row["gbs"] / PEAK_HBM_GBS
        table[name] = row

    def traffic_of(name):
        return traffic_table.get("conv_fused" if name.startswith("conv_fused") else name)

    if dom is not None and dom in kernels:
        k = kernels[dom]                                   # the dominant class, timed inside the timed region
        avg_ms = k["total_ms"] / k["launches"]
        timed_steps = args.table_steps if args.graph else args.steps
        if dom.startswith(MFMA_KERNELS):
            ach = k["flops"] / (k["total_ms"] * 1e-3) / 1e12
            roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": PEAK_TFLOPS[args.dtype],
                    "unit": "TFLOP/s", "frac": ach / PEAK_TFLOPS[args.dtype], "traffic": traffic_of(dom),
                    "traffic_source": traffic_src, "avg_launch_ms": avg_ms, "launches_per_step": k["launches"] / timed_steps,
                    "flops_per_launch": k["flops"] / k["launches"]}
            # every matrix-core class together (the products of all three passes of all five layers)
            fl = sum(kernels[n]["flops"] for n in mfma_classes if n in kernels)
            ms = sum(kernels[n]["total_ms"] for n in mfma_classes if n in kernels)
            roof_all = {"kernels": sorted(n for n in mfma_classes if n in kernels), "bound": "mfma",
                        "achieved": fl / (ms * 1e-3) / 1e12, "peak": PEAK_TFLOPS[args.dtype], "unit": "TFLOP/s",
                        "frac": fl / (ms * 1e-3) / 1e12 / PEAK_TFLOPS[args.dtype], "ms_per_step": ms / timed_steps,
                        "per_class_frac": {n: kernels[n]["flops"] / (kernels[n]["total_ms"] * 1e-3) / 1e12 / PEAK_TFLOPS[args.dtype]
                                           for n in mfma_classes if n in kernels}}
        else:
            ach = k["bytes"] / (k["total_ms"] * 1e-3) / 1e9
            roof = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": ach / PEAK_HBM_GBS, "traffic": traffic_of(dom), "traffic_source": traffic_src, "avg_launch_ms": avg_ms,
                    "launches_per_step": k["launches"] / timed_steps, "bytes_per_launch": k["bytes"] / k["launches"]}

    # the tensors the timed steps ran on: finite, not degenerate, weights still where they were drawn
    health = stack.tensor_health(W_start)
    health["steps_run"] = args.warmup + (args.table_steps if table_kernels else 0) + args.steps

    # beside the timed region: the same K steps replayed as one captured HIP graph (launch gaps removed; no
    # per-kernel events are possible inside a replay, so the headline value and the roofline stay the eager ones)
    graph_extra = None
    if not args.graph and not args.overlap and not args.no_graph:
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                stack.step(X, dOut, lr, mu)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            tg = time.perf_counter()
            for _ in range(args.steps):
                graph.replay()
            torch.cuda.synchronize()
            tg = time.perf_counter() - tg
            after = stack.tensor_health(W_start)
            graph_extra = {"ms_per_step": 1e3 * tg / args.steps, "value": args.batch * args.steps / tg, "unit": "images/s", "steps": args.steps,
                           "tensors_finite_after": after["finite"] and not stack.health_is_degenerate(after),
                           "note": "the step captured once and replayed as a HIP graph, timed after the eager region; same kernels, bit-identical results"}
        except Exception as exc:  # the eager figures above stand on their own
            graph_extra = {"error": f"{type(exc).__name__}: {exc}"}
    degenerate = stack.health_is_degenerate(health)

    cpu = cpu_baseline(args.cpu_sample) if args.cpu_sample > 0 else None
    out = {
        "metric": "conv fwd+bwd images/sec, CaffeNet-shaped conv stack, batch 256",
        "value": images_per_s, "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "ms_per_step_median": median_ms, "ms_per_step_cv": cv, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": "synthetic",
        "config": {"workload": workload,
                   "global_batch": args.batch, "conv1_data_gradient": bool(args.conv1_dgrad), "launch": "hip graph replay" if args.graph else "eager",
                   "lr": lr, "momentum": mu, "upstream_gradient": f"N(0,1) draw x 2^{int(math.log2(grad_scale))}"},
        "tensor_health": health,
        "tflops": flops_step / (ms_per_step * 1e-3) / 1e12,
        "mfma_frac_of_peak_whole_step": flops_step / (ms_per_step * 1e-3) / 1e12 / PEAK_TFLOPS[args.dtype],
        "roofline": roof, "roofline_all_mfma_kernels": roof_all, "cpu_baseline": cpu, "graph_replay": graph_extra,
        "kernels_note": f"per-kernel table from {args.table_steps} instrumented steps before the timed region",
        "kernels": table,
    }
    print(json.dumps(out))
    if degenerate:
        print("bench.py: the timed steps ran on non-finite or degenerate tensors (see tensor_health); "
              "the figures above do not measure the stated workload.", file=sys.stderr)
        sys.exit(3)


if __name__ == "__main__":
    main()
