"""Partial-batching sweep on one MI355X: the paper's single-node experiment (Sec. III-B; App. C, Fig. (b), (c)).

At a fixed batch b, the forward pass of one layer is run b_p images at a time for b_p = 1, 2, 4, ... b and
the sweep reports, per b_p: the workspace (lowered data) in MB, the time of the matrix products alone, the
time of lowering alone, and the wall time of the whole pass.  Default layer: CaffeNet's conv2 at b = 256 in
bf16, the layer the paper's figure uses.

    python -m paper_1606_04487_amd.bp_sweep [--batch 256] [--dtype bf16|f32] [--layer 1] [--reps 5]
"""
import argparse
import time

import torch

from . import binding as B
from . import workloads as wl


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=256)
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16")
    ap.add_argument("--layer", type=int, default=1, help="index into the CaffeNet conv stack (1 = conv2)")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--split-k", action="store_true",
                    help="OMNI_FLAG_SPLIT_K: split the reduction of products with few columns (results then differ by rounding between b_p)")
    args = ap.parse_args()
    dtype = B.BF16 if args.dtype == "bf16" else B.F32
    L = wl.caffenet_stack(args.batch)[args.layer]
    t = wl.layer_tensors(L, seed=1, bf16=(dtype == B.BF16))
    td = B.torch_dtype(dtype)
    X, W = (torch.from_numpy(t[k]).cuda().to(td) for k in ("X", "W"))
    bias = torch.from_numpy(t["bias"]).cuda()
    extra = B.FLAG_SPLIT_K if args.split_k else 0
    d = B.conv_desc(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p, dtype, B.FLAG_RELU | extra)
    Y = torch.empty((L.N, L.F, L.Ho, L.Wo), dtype=td, device="cuda")
    ref = None
    print(f"layer {L.name}: b = {L.N}, {args.dtype}, GEMM {L.F} x {L.K} x ({L.N}*{L.Ho * L.Wo}), {L.gemm_flops / 1e9:.1f} GFLOP")
    print("| b_p | workspace MB | products ms | lowering ms | whole pass ms | products TFLOP/s | identical |")
    print("|---|---|---|---|---|---|---|")
    bp = 1
    while bp <= L.N:
        sub = B.conv_desc(bp, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p, dtype, extra)
        nbytes = B.conv_workspace_bytes(sub, B.PASS_FORWARD)
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        try:
            B.conv_forward_partial(d, bp, X, W, bias, Y, ws)      # warm-up
        except B.OmniError:
            # a group of b_p images of this layer does not start on a 16-byte boundary
            print(f"| {bp} | - | - | - | - | - | (groups misaligned) |", flush=True)
            bp *= 2
            continue
        torch.cuda.synchronize()
        B.profile_enable(True)
        t0 = time.perf_counter()
        for _ in range(args.reps):
            B.conv_forward_partial(d, bp, X, W, bias, Y, ws)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / args.reps
        s = B.profile_summary()
        B.profile_enable(False)
        gemm = s["gemm_forward"]["total_ms"] / args.reps
        low = s["lower"]["total_ms"] / args.reps
        if ref is None:
            ref = Y.clone()
        same = torch.equal(Y, ref) if not args.split_k else f"max diff {float((Y.float() - ref.float()).abs().max()):.2e}"
        print(f"| {bp} | {nbytes / 1e6:.1f} | {gemm:.3f} | {low:.3f} | {wall * 1e3:.3f} | "
              f"{L.gemm_flops / gemm / 1e9:.0f} | {same} |", flush=True)
        del ws
        bp *= 2


if __name__ == "__main__":
    main()
