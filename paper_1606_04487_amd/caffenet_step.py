"""One whole training iteration of a CaffeNet-shaped network through the library: the convolution phase
(conv1..conv5 with ReLU, max-pools and the two normalisation layers) and the FC phase (FC6..FC8 as whole-image
convolutions, dropout after FC6 and FC7), forward, backward and one momentum-SGD update (Sec. II-C: the two
phases; App. C, Fig. "CcT_Batch": the paper's single-node figure is the time of this whole iteration).

Prints the time per iteration, images/s and the per-kernel-class table (HIP events around every launch).
Synthetic seeded input; the upstream gradient at FC8's output is the N(0,1) draw scaled as in bench.py.

    python -m paper_1606_04487_amd.caffenet_step [--batch 256] [--dtype bf16|f32] [--steps 20] [--warmup 5]
"""
from __future__ import annotations

import argparse
import json


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    args = ap.parse_args()

    import numpy as np
    import torch
    from . import binding as B
    from . import workloads as wl
    from .stack import ConvStack

    torch.cuda.set_device(0)
    dtype = B.BF16 if args.dtype == "bf16" else B.F32
    layers = wl.caffenet_full(args.batch)
    net = ConvStack(layers, dtype=dtype, ceil_mode=False, skip_first_dgrad=True)
    data = wl.stack_tensors(layers, seed=1, bf16=(dtype == B.BF16), pooled_out=net.output_shape()[-2:])
    net.set_parameters(data["W"], data["bias"])
    X = torch.from_numpy(data["X"]).cuda().to(B.torch_dtype(dtype))
    dOut = (torch.from_numpy(data["dY"]).cuda() * wl.step_upstream_scale(args.batch)).to(B.torch_dtype(dtype))
    W0 = [w.clone() for w in net.W]
    lr, mu = 0.01, 0.9
    for _ in range(args.warmup):
        net.step(X, dOut, lr, mu)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        net.step(X, dOut, lr, mu)
        marks[i + 1].record()
    torch.cuda.synchronize()
    per = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms = sum(per) / len(per)
    B.profile_enable(True)
    for _ in range(5):
        net.step(X, dOut, lr, mu)
    torch.cuda.synchronize()
    table = B.profile_summary()
    B.profile_enable(False)
    health = net.tensor_health(W0)
    conv_flops = sum(3 * L.gemm_flops for L in layers[:5]) - layers[0].gemm_flops
    fc_flops = sum(3 * L.gemm_flops for L in layers[5:])
    out = {"workload": f"caffenet_whole_iteration_b{args.batch}_{args.dtype}", "ms_per_iteration": ms, "ms_median": per[len(per) // 2],
           "images_per_s": args.batch / (ms * 1e-3), "conv_gflop": conv_flops / 1e9, "fc_gflop": fc_flops / 1e9,
           "tflops": (conv_flops + fc_flops) / (ms * 1e-3) / 1e12, "finite": health["finite"],
           "zero_fraction_Y": health["zero_fraction_Y"], "std_W": health["std_W"]}
    print(json.dumps(out))
    print(f"\n{out['workload']}: {ms:.3f} ms per iteration (median {out['ms_median']:.3f}), {out['images_per_s']:.0f} images/s, "
          f"{out['conv_gflop']:.0f} + {out['fc_gflop']:.0f} GFLOP of products, {out['tflops']:.0f} TFLOP/s\n")
    print("| kernel class | launches/iteration | ms/iteration |\n|---|---|---|")
    tot = 0.0
    for name, k in sorted(table.items(), key=lambda kv: -kv[1]["total_ms"]):
        print(f"| {name} | {k['launches'] / 5:.0f} | {k['total_ms'] / 5:.3f} |")
        tot += k["total_ms"] / 5
    print(f"| all (every launch bracketed by events) | | {tot:.3f} |")
    if not health["finite"]:
        raise SystemExit("non-finite tensors after the run")


if __name__ == "__main__":
    main()
