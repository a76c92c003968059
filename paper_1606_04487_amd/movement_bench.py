"""Time the two data-movement steps of the explicit path on their own: batched lowering (App. C, lowering
phase) and col2im, at the five CaffeNet-shaped layers, batch 256, against the HBM roofline.

Algorithmic bytes per launch: lowering reads X once and writes D-hat once, (N*C*H*W + K*ld) * e; col2im
reads dD-hat once and writes dX once, the same count (e = 2 for bf16, 4 for fp32).  Durations come from the
library's own HIP events around each launch (omni_profile_*).  Prints one JSON line per (layer, dtype, kernel)
and a table; run it under rocprofv3 (`--kernel-trace --stats`, or `--pmc FETCH_SIZE` / `--pmc WRITE_SIZE`)
for the profiler's view of the same launches: it starts with the 256 MiB device copy that calibrates the
counters.

    python -m paper_1606_04487_amd.movement_bench [--batch 256] [--iters 10] [--dtype bf16 f32]
"""
from __future__ import annotations

import argparse
import json

PEAK_HBM_GBS = 8000.0


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--iters", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--dtype", nargs="+", default=["bf16", "f32"], choices=["bf16", "f32"])
    ap.add_argument("--layers", nargs="+", default=["conv1", "conv2", "conv3", "conv4", "conv5"])
    args = ap.parse_args()

    import torch
    from . import binding as B
    from . import workloads as wl

    torch.cuda.set_device(0)
    cal_src = torch.zeros(64 * 1024 * 1024, dtype=torch.int32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    del cal_src, cal_dst

    rows = []
    for dname in args.dtype:
        dtype = B.BF16 if dname == "bf16" else B.F32
        td, e = B.torch_dtype(dtype), (2 if dname == "bf16" else 4)
        for L in wl.caffenet_stack(args.batch):
            if L.name not in args.layers:
                continue
            d = B.conv_desc(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p, dtype)
            ld = B.conv_dhat_ld(d)
            g = torch.Generator(device="cuda").manual_seed(1)
            X = torch.randn((L.N, L.C, L.H, L.W), generator=g, device="cuda", dtype=torch.float32).to(td)
            Dhat = torch.empty((L.K, ld), dtype=td, device="cuda")
            dX = torch.empty_like(X)
            for _ in range(args.warmup):
                B.lower(d, X, Dhat, ld)
                B.col2im(d, Dhat, dX, ld)
            torch.cuda.synchronize()
            B.profile_enable(True)
            for _ in range(args.iters):
                B.lower(d, X, Dhat, ld)
                B.col2im(d, Dhat, dX, ld)
            torch.cuda.synchronize()
            summ = B.profile_summary()
            B.profile_enable(False)
            nbytes = (X.numel() + L.K * ld) * e
            for kname in ("lower", "col2im"):
                k = summ[kname]
                ms = k["total_ms"] / k["launches"]
                row = {"kernel": kname, "layer": L.name, "dtype": dname, "batch": L.N, "avg_launch_ms": ms,
                       "algorithmic_bytes": nbytes, "library_counted_bytes": k["bytes"] / k["launches"],
                       "gbs": nbytes / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
                rows.append(row)
                print(json.dumps(row), flush=True)
            del X, Dhat, dX
            torch.cuda.empty_cache()
    print("\n| kernel | layer | dtype | MB per launch | us | GB/s | of 8 TB/s |\n|---|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['kernel']} | {r['layer']} | {r['dtype']} | {r['algorithmic_bytes'] / 1e6:.0f} | {r['avg_launch_ms'] * 1e3:.1f} | "
              f"{r['gbs']:.0f} | {r['frac_of_hbm_peak']:.2f} |")


if __name__ == "__main__":
    main()
