"""Time the 3 x 3 / stride 2 max-pool kernels on their own at the three pooled layers of the CaffeNet-shaped stack
(App. C, "Data Parallelism in non-GEMM Kernels": the layers between the convolutions), batch 256, bf16.

Per layer and kernel: the forward pool reading the planes directly (the default) and staging them in LDS
(OMNI_TUNE_POOL_LDS), the backward pool with the ReLU mask writing the dense gradient and writing the rows form with
plane sums.  Each is timed twice: launched back to back (operands stay in the last-level cache between launches) and
with a 512 MiB fill between launches (operands come from memory, as inside a training step).  Algorithmic bytes:
forward x + y + winners; backward dy + pooled values + winners + dx.  Durations from the library's own HIP events.
Prints one JSON line per case and a table.  Run it under rocprofv3 (`--kernel-trace --stats` or `--pmc ...`) for the
profiler's view of the same launches.

    python -m paper_1606_04487_amd.pool_bench [--batch 256] [--iters 10]
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
    ap.add_argument("--no-cold", action="store_true", help="skip the runs with a cache-clearing fill between launches")
    args = ap.parse_args()

    import torch
    from . import binding as B

    torch.cuda.set_device(0)
    td = torch.bfloat16
    N = args.batch
    flush = torch.empty(512 << 20, dtype=torch.uint8, device="cuda")
    rows = []
    for name, C, H in (("pool1", 96, 55), ("pool2", 256, 27), ("pool5", 256, 13)):
        Ho = B.pool_output_dim(H, 3, 2, False)
        g = torch.Generator(device="cuda").manual_seed(1)
        x = torch.randn((N, C, H, H), generator=g, device="cuda").clamp_(min=0).to(td)
        dy = torch.randn((N, C, Ho, Ho), generator=g, device="cuda").to(td)
        y = torch.empty((N, C, Ho, Ho), dtype=td, device="cuda")
        am = torch.empty((N, C, Ho, Ho), dtype=torch.uint8, device="cuda")
        dx = torch.empty_like(x)
        pitch = (H * H + 7) // 8 * 8
        dx_rows = torch.zeros((C, N * pitch), dtype=td, device="cuda")
        sums = torch.empty((C, N), dtype=torch.float32, device="cuda")
        B.maxpool_forward(x, 3, 2, False, y, am)
        fwd_bytes = (x.numel() + y.numel()) * 2 + am.numel()
        bwd_bytes = (2 * y.numel() + x.numel()) * 2 + am.numel()
        cases = [
            ("forward, direct", "maxpool_forward", fwd_bytes, 0, lambda: B.maxpool_forward(x, 3, 2, False, y, am)),
            ("forward, LDS-staged", "maxpool_forward", fwd_bytes, 1, lambda: B.maxpool_forward(x, 3, 2, False, y, am)),
            ("backward + ReLU mask, dense", "maxpool_backward", bwd_bytes, 0,
             lambda: B.maxpool_relu_backward(dy, am, y, H, H, 3, 2, False, dx)),
            ("backward + ReLU mask, rows form + plane sums", "maxpool_backward", bwd_bytes + (C * N * pitch - x.numel()) * 2 + 4 * C * N, 0,
             lambda: B.maxpool_backward_rows(dy, am, y, H, H, 3, 2, False, dx_rows=dx_rows, plane_sums=sums)),
        ]
        for what, cls, nbytes, lds, fn in cases:
            B.tuning_set(B.TUNE_POOL_LDS, lds)
            rec = {"layer": name, "planes": f"{N} x {C} x {H} x {H}", "kernel": what, "algorithmic_MB": round(nbytes / 1e6, 1)}
            for cold in ((False,) if args.no_cold else (False, True)):
                for it in range(args.warmup + args.iters):
                    if it == args.warmup:
                        torch.cuda.synchronize()
                        B.profile_enable(True)
                    if cold:
                        flush.zero_()
                    fn()
                torch.cuda.synchronize()
                us = B.profile_summary()[cls]["total_ms"] / args.iters * 1e3
                B.profile_enable(False)
                key = "cold" if cold else "back_to_back"
                rec[f"us_{key}"] = round(us, 1)
                rec[f"GBs_{key}"] = round(nbytes / us / 1e3)
                rec[f"of_peak_{key}"] = round(nbytes / us / 1e3 / PEAK_HBM_GBS, 3)
            B.tuning_set(B.TUNE_POOL_LDS, 0)
            rows.append(rec)
            print(json.dumps(rec), flush=True)
    print()
    cols = [c for c in ("us_back_to_back", "GBs_back_to_back", "of_peak_back_to_back", "us_cold", "GBs_cold", "of_peak_cold") if c in rows[0]]
    print("| layer | planes | kernel | algorithmic MB | " + " | ".join(c.replace("_", " ") for c in cols) + " |")
    print("|---|---|---|---|" + "---|" * len(cols))
    for r in rows:
        print(f"| {r['layer']} | {r['planes']} | {r['kernel']} | {r['algorithmic_MB']} | " + " | ".join(str(r[c]) for c in cols) + " |")


if __name__ == "__main__":
    main()
