"""Timing and oracle error of the workload configurations other than the headline stack: the single small
layer, the CIFAR-style stack, CaffeNet conv1 alone and conv2..conv5 alone (fp32 and bf16).

For every (layer, dtype, pass) one record: milliseconds per call (HIP events over `reps` back-to-back calls
after a warm-up), images/s, TFLOP/s of the pass's matrix product (2*M*K*F) and its fraction of the MFMA peak of
the dtype, and the tensor-normalised error against the CPU oracle (whole tensors for the small configurations,
sampled entries for the batch-256 layers).  The small configurations are bound by launch latency, not by the
matrix cores or HBM: their roofline fractions are reported and labelled so.  `bench.py --config N` prints the
records of configuration N as one JSON line.
"""
from __future__ import annotations

import numpy as np

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def _time(fn, reps, torch):
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def _err(got, ref):
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


def layer_records(L, dname, seed, x_dist, reps, fused, whole, samples=2000):
    """Forward, data gradient and model gradient of one layer on its own."""
    import torch
    import oracle
    from . import binding as B
    from . import workloads as wl

    dtype = B.BF16 if dname == "bf16" else B.F32
    td = B.torch_dtype(dtype)
    t = wl.layer_tensors(L, seed=seed, x_dist=x_dist, bf16=(dtype == B.BF16))
    s = oracle.shape(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p)
    d = B.conv_desc(L.N, L.C, L.H, L.W, L.F, L.k, L.k, L.s, L.p, dtype, B.FLAG_FUSED if fused else 0)
    X, W, dY = (torch.from_numpy(t[k]).cuda().to(td) for k in ("X", "W", "dY"))
    bias = torch.from_numpy(t["bias"]).cuda()
    ws = [torch.empty(B.conv_workspace_bytes(d, p), dtype=torch.uint8, device="cuda") for p in (0, 1, 2)]
    ho, wo = B.conv_output_dims(d)
    Y = torch.empty((L.N, L.F, ho, wo), dtype=td, device="cuda")
    dX = torch.empty_like(X)
    dW = torch.empty((L.F, L.C, L.k, L.k), dtype=torch.float32, device="cuda")
    db = torch.empty((L.F,), dtype=torch.float32, device="cuda")
    calls = {
        "forward": lambda: B.conv_forward(d, X, W, bias, Y, ws[0]),
        "backward_data": lambda: B.conv_backward_data(d, dY, W, dX, ws[1]),
        "backward_weights": lambda: B.conv_backward_weights(d, X, dY, dW, db, ws[2]),
    }
    rng = np.random.default_rng(seed + 1)

    def error(name):
        if whole:
            ref = {"forward": lambda: oracle.conv_forward(s, t["X"], t["W"], t["bias"]),
                   "backward_data": lambda: oracle.conv_backward_data(s, t["dY"], t["W"]),
                   "backward_weights": lambda: oracle.conv_backward_weights(s, t["X"], t["dY"])}[name]()
            got = {"forward": Y, "backward_data": dX, "backward_weights": dW}[name]
            return _err(got.float().cpu().numpy(), ref)
        got_t = {"forward": Y, "backward_data": dX, "backward_weights": dW}[name]
        idx = np.unique(rng.integers(0, got_t.numel(), size=samples if name != "backward_weights" else 200))
        got = got_t.reshape(-1)[torch.from_numpy(idx).cuda()].float().cpu().numpy()
        ref = {"forward": lambda: oracle.conv_forward_at(s, t["X"], t["W"], t["bias"], idx),
               "backward_data": lambda: oracle.conv_backward_data_at(s, t["dY"], t["W"], idx),
               "backward_weights": lambda: oracle.conv_backward_weights_at(s, t["X"], t["dY"], idx)}[name]()
        return _err(got, ref)

    out = []
    for name, fn in calls.items():
        ms = _time(fn, reps, torch)
        tf = L.gemm_flops / (ms * 1e-3) / 1e12
        out.append({"layer": L.name, "dtype": dname, "pass": name, "requested": "fused" if fused else "explicit", "path": "fused" if fused and B.conv_fused_supported(d, list(calls).index(name)) else "explicit",
                    "ms": ms, "images_per_s": L.N / (ms * 1e-3), "tflops": tf, "frac_of_mfma_peak": tf / PEAK_TFLOPS[dname],
                    "max_rel_err_vs_oracle": error(name), "error_over": "whole tensor" if whole else "sampled entries"})
    return out


def stack_record(layers, dname, ceil_mode, x_dist, reps):
    """A chained stack: one forward + backward + momentum update per step."""
    import torch
    from . import binding as B
    from . import workloads as wl
    from .stack import ConvStack

    dtype = B.BF16 if dname == "bf16" else B.F32
    st = ConvStack(layers, dtype=dtype, ceil_mode=ceil_mode, skip_first_dgrad=False)
    data = wl.stack_tensors(layers, seed=1, x_dist=x_dist, bf16=(dtype == B.BF16), pooled_out=st.output_shape()[-2:])
    st.set_parameters(data["W"], data["bias"])
    N = layers[0].N
    X = torch.from_numpy(data["X"]).cuda().to(B.torch_dtype(dtype))
    dOut = (torch.from_numpy(data["dY"]).cuda() * wl.step_upstream_scale(N)).to(B.torch_dtype(dtype))
    W0 = [w.clone() for w in st.W]
    ms = _time(lambda: st.step(X, dOut, 0.01, 0.9), reps, torch)
    B.profile_enable(True)
    for _ in range(5):
        st.step(X, dOut, 0.01, 0.9)
    torch.cuda.synchronize()
    table = {k: {"launches_per_step": v["launches"] / 5, "ms_per_step": v["total_ms"] / 5} for k, v in B.profile_summary().items()}
    B.profile_enable(False)
    flops = sum(3 * L.gemm_flops for L in layers)
    health = st.tensor_health(W0)
    return {"ms_per_step": ms, "images_per_s": N / (ms * 1e-3), "tflops": flops / (ms * 1e-3) / 1e12,
            "frac_of_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_TFLOPS[dname], "kernels": table,
            "finite": health["finite"], "zero_fraction_Y": health["zero_fraction_Y"]}


def run_config(config: int, reps: int):
    from . import workloads as wl
    if config == 1:
        L = wl.single_layer_config()
        recs = layer_records(L, "f32", 1, "uniform", reps, False, True)
        return {"workload": "single_layer_N8_3x32x32_32@5x5_f32", "bound": "launch latency (0.04 GFLOP per product)",
                "passes": recs, "value": L.N / (sum(r["ms"] for r in recs) * 1e-3)}
    if config == 2:
        layers = wl.cifar_stack(128)
        rec = stack_record(layers, "f32", True, "uniform", reps)
        per_layer = [r for i, L in enumerate(layers) for r in layer_records(L, "f32", 10 + i, "uniform", reps, False, True)]
        return {"workload": "cifar_stack_b128_f32_fwd+bwd+sgd", "bound": "launch latency (0.6-1.7 GFLOP per product)",
                "step": rec, "passes": per_layer, "value": rec["images_per_s"]}
    if config == 3:
        L = wl.caffenet_stack(256)[0]
        recs = layer_records(L, "f32", 1, "normal", reps, False, False)
        return {"workload": "caffenet_conv1_b256_f32", "bound": "mfma (fp32)", "passes": recs,
                "value": L.N / (sum(r["ms"] for r in recs) * 1e-3)}
    if config == 4:
        recs = []
        for dname, fused in (("f32", False), ("bf16", False), ("bf16", True)):
            for i, L in enumerate(wl.caffenet_stack(256)[1:]):
                recs += layer_records(L, dname, 2 + i, "normal", reps, fused, False)
        tot = {}
        for r in recs:
            key = r["dtype"] + "_" + r["requested"]
            tot[key] = tot.get(key, 0.0) + r["ms"]
        return {"workload": "caffenet_conv2-5_b256_isolated_layers", "bound": "mfma", "passes": recs, "ms_all_passes": tot,
                "value": 256 / (min(tot.values()) * 1e-3)}
    raise ValueError("configurations 1 to 4; the headline stack (5) is bench.py's default")
