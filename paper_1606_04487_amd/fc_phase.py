"""The FC phase of a CaffeNet-shaped network through the same entry points (Sec. II-C: conv phase and FC phase).

FC6 (256 x 6 x 6 -> 4096) is the convolution whose 6 x 6 window covers the whole image; FC7 (4096 -> 4096) and
FC8 (4096 -> 1000) are 1 x 1 convolutions on 1 x 1 images.  Prints, per layer, the time of the forward pass,
the data gradient and the model gradient at the given batch, and the FC phase's share next to the paper's
count (80 GFLOP of the 1.6 + 0.08 TFLOP per 256-image iteration, Sec. II-C).

    python -m paper_1606_04487_amd.fc_phase [--batch 256] [--dtype bf16|f32] [--reps 10]
"""
import argparse

import torch

from . import binding as B

FC_LAYERS = [("fc6", 256, 6, 4096), ("fc7", 4096, 1, 4096), ("fc8", 4096, 1, 1000)]   # name, C, H = W = k, F


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--no-split", action="store_true", help="do not split the reductions of the narrow products over the chip")
    args = ap.parse_args()
    dtype = B.BF16 if args.dtype == "bf16" else B.F32
    td = B.torch_dtype(dtype)
    N = args.batch
    print(f"FC phase, batch {N}, {args.dtype}, reductions of narrow products {'not split' if args.no_split else 'split over the chip'}")
    print("| layer | GFLOP per pass | forward ms | data gradient ms | model gradient ms | TFLOP/s (all three) |")
    print("|---|---|---|---|---|---|")
    total_ms, total_flop = 0.0, 0.0
    for name, C, hk, F in FC_LAYERS:
        d = B.conv_desc(N, C, hk, hk, F, hk, hk, 1, 0, dtype, 0 if args.no_split else B.FLAG_SPLIT_K)
        X = torch.randn(N, C, hk, hk, device="cuda").to(td)
        W = (0.01 * torch.randn(F, C, hk, hk, device="cuda")).to(td)
        bias = torch.zeros(F, device="cuda")
        dY = torch.randn(N, F, 1, 1, device="cuda").to(td)
        ws = [torch.empty(B.conv_workspace_bytes(d, p), dtype=torch.uint8, device="cuda") for p in (0, 1, 2)]
        Y = torch.empty(N, F, 1, 1, device="cuda", dtype=td)
        dX = torch.empty_like(X)
        dW = torch.empty(F, C, hk, hk, device="cuda")
        db = torch.empty(F, device="cuda")
        times = []
        for fn in (lambda: B.conv_forward(d, X, W, bias, Y, ws[0]),
                   lambda: B.conv_backward_data(d, dY, W, dX, ws[1]),
                   lambda: B.conv_backward_weights(d, X, dY, dW, db, ws[2])):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) / args.reps)
        flop = 2.0 * N * C * hk * hk * F
        total_ms += sum(times)
        total_flop += 3 * flop
        print(f"| {name} | {flop / 1e9:.2f} | {times[0]:.3f} | {times[1]:.3f} | {times[2]:.3f} | "
              f"{3 * flop / sum(times) / 1e9:.0f} |", flush=True)
    print(f"\nFC phase forward + backward: {total_ms:.3f} ms, {total_flop / 1e9:.1f} GFLOP "
          f"({total_flop / total_ms / 1e9:.0f} TFLOP/s); the paper counts about 80 GFLOP for this phase at batch 256.")


if __name__ == "__main__":
    main()
