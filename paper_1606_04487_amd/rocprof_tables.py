"""Turn rocprofv3 CSV output of a bench run into the short tables kept under profiles/.

Four sub-commands, each reading what one kind of rocprofv3 run wrote (`--output-format csv`):

    movement  <FETCH_SIZE csv> <WRITE_SIZE csv> <stdout>  lowering / col2im alone (movement_bench): per layer times and traffic
    stats     <kernel_stats.csv> <bench stdout>   per-class and per-kernel durations next to the library's own
                                                   event timing (from the JSON line the profiled run printed)
    traffic   <FETCH_SIZE csv> <WRITE_SIZE csv>    HBM bytes per kernel class, each counter scaled by what it read
                                                   for the 256 MiB device copy bench.py makes first; also updates
                                                   hbm_traffic.json beside this file, which bench.py reads for
                                                   `roofline.traffic`
    counters  <pmc csv> [<pmc csv> ...]            SQ counters of the matrix-core kernels
    pools     <pool_bench stdout> <pmc csv> [...]  the pool kernels alone: pool_bench's table and their SQ counters

Every table starts with the full command that produced its input.  Host-side text processing only.
"""
from __future__ import annotations

import argparse
import collections
import csv
import hashlib
import json
import re
from pathlib import Path

HERE = Path(__file__).resolve().parent
TRAFFIC_JSON = HERE / "hbm_traffic.json"
CAL_KIB = 262144.0   # the calibration copy of bench.py: 256 MiB read, 256 MiB written


def kernel_class(name: str):
    """Kernel function name -> the library's timing class (the names omni_profile_kernel_name returns)."""
    if "fused_conv_kernel" in name:
        return "conv_fused"
    if "strided_conv_kernel" in name:
        return "conv_strided_forward"
    if "PartialEpilogue" in name or "wgrad_kernel" in name or "wgrad_patch_kernel" in name or "wgrad_wide_kernel" in name:
        return "gemm_wgrad"
    if "FwdEpilogue" in name and "gemm" in name:
        return "gemm_forward"
    if "RowMajorEpilogue" in name:
        return "gemm_dgrad"
    for key, cls in (("phase_split", "lower"), ("phase_merge", "col2im"), ("lower_", "lower"), ("col2im", "col2im"),
                     ("pack_dyhat", "pack_dyhat"), ("pack_weights", "pack_khat"), ("pack_jobs", "pack_khat"), ("pack_strided_weights", "pack_khat"),
                     ("dgrad_phase_weights", "pack_khat"), ("pack_khat", "pack_khat"), ("bias_reduce", "bias_reduce"),
                     ("reduce_partials", "reduce_partials"), ("reduce_wide", "reduce_partials"), ("reduce_store", "reduce_partials"),
                     ("maxpool_fwd", "maxpool_forward"), ("maxpool_bwd", "maxpool_backward"),
                     ("maxpool_forward", "maxpool_forward"), ("maxpool_backward", "maxpool_backward"),
                     ("relu", "relu"), ("sgd", "sgd"), ("lrn", "lrn"), ("dropout", "dropout")):
        if key in name:
            return cls
    return None


def short_name(name: str) -> str:
    n = re.sub(r"\(.*", "", name).replace("void ", "").replace("omni::", "")
    return n.replace("unsigned short", "bf16")


def sources_digest() -> str:
    """Hash of the kernel sources: a traffic table is only reported for the code it was measured on."""
    h = hashlib.sha256()
    for f in sorted((HERE / "csrc").glob("*")):
        if f.suffix in (".hip", ".h"):
            h.update(f.name.encode())
            h.update(f.read_bytes())
    return h.hexdigest()[:16]


def last_json_line(path: str) -> dict:
    lines = [l for l in open(path) if l.startswith("{")]
    return json.loads(lines[-1])


def cmd_stats(a) -> None:
    rows = list(csv.DictReader(open(a.csv)))
    bench = last_json_line(a.bench_out)
    steps = a.steps
    agg = collections.OrderedDict()
    for r in rows:
        c = kernel_class(r["Name"])
        if c is None:
            continue
        e = agg.setdefault(c, [0, 0.0])
        e[0] += int(r["Calls"])
        e[1] += float(r["TotalDurationNs"])
    ev = bench.get("kernels", {})
    with open(a.out, "w") as f:
        f.write(f"# rocprofv3 kernel statistics: {a.title}\n\n")
        f.write(f"Command (run from /tmp with TMPDIR=/tmp on one MI355X):\n\n    {a.command}\n\n")
        f.write(f"The run makes {steps} steps (warm-up + instrumented + timed); the table divides by {steps}.  `bench events` is the same\n"
                "class timed by the library's own HIP events in that very run (the `kernels` table of the JSON line it printed).\n")
        roof = bench.get("roofline")
        if roof:
            f.write(f"Dominant class of that run, timed inside the timed region: {roof['kernel']}, avg launch "
                    f"{roof['avg_launch_ms'] * 1e3:.1f} us, {roof['achieved']:.0f} {roof['unit']} = {roof['frac']:.3f} of peak.\n")
        f.write(f"\nbench line of the profiled run: {bench['ms_per_step']:.3f} ms/step, {bench['value']:.0f} {bench['unit']} (profiler attached)\n\n")
        f.write("| kernel class | launches/step | rocprofv3 avg us/launch | rocprofv3 ms/step | bench events ms/step |\n|---|---|---|---|---|\n")
        for c, (calls, ns) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
            if c == "conv_fused":
                e = sum(ev.get(k, {}).get("ms_per_step", 0.0) for k in ("conv_fused_forward", "conv_fused_dgrad"))
            else:
                e = ev.get(c, {}).get("ms_per_step", float("nan"))
            f.write(f"| {c} | {calls / steps:.1f} | {ns / calls / 1e3:.1f} | {ns / steps / 1e6:.3f} | {e:.3f} |\n")
        tot = sum(v[1] for v in agg.values()) / steps / 1e6
        f.write(f"\nSum of the library's kernels: {tot:.3f} ms/step.\n\n")
        f.write("Per kernel (names shortened):\n\n| kernel | class | calls | avg us | % of GPU time |\n|---|---|---|---|---|\n")
        for r in rows:
            c = kernel_class(r["Name"])
            if c is None:
                continue
            f.write(f"| {short_name(r['Name'])} | {c} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {r['Percentage']} |\n")
    print(open(a.out).read())


def read_counter(path: str):
    per_class = collections.defaultdict(list)
    cal = 0.0
    for r in csv.DictReader(open(path)):
        v = float(r["Counter_Value"])
        if "copyBuffer" in r["Kernel_Name"]:
            cal = max(cal, v)
        c = kernel_class(r["Kernel_Name"])
        if c:
            per_class[c].append(v)
    return per_class, cal


def cmd_traffic(a) -> None:
    fe, fcal = read_counter(a.fetch)
    wr, wcal = read_counter(a.write)
    if fcal <= 0 or wcal <= 0:
        raise SystemExit("no calibration copy found in the counter files")
    ff, wf = CAL_KIB / fcal, CAL_KIB / wcal
    steps = a.steps
    table = {}
    with open(a.out, "w") as f:
        f.write(f"# HBM traffic per kernel class (rocprofv3 --pmc): {a.title}\n\n")
        f.write("Commands (each from /tmp with TMPDIR=/tmp on one MI355X; one counter per run):\n\n")
        f.write(f"    {a.command.replace('COUNTER', 'FETCH_SIZE')}\n    {a.command.replace('COUNTER', 'WRITE_SIZE')}\n\n")
        f.write("Calibration: the program first copies 256 MiB (262144 KiB) device to device; for that copy kernel FETCH_SIZE read "
                f"{fcal:.1f} and WRITE_SIZE read {wcal:.1f}, so counter values are scaled by {ff:.4f} (fetch) and {wf:.4f} (write) to KiB.\n\n")
        f.write("| kernel class | launches/step | fetched MB/launch | written MB/launch | total MB/step |\n|---|---|---|---|---|\n")
        total = 0.0
        for c in sorted(fe, key=lambda c: -(sum(fe[c]) * ff + sum(wr.get(c, [0])) * wf)):
            n = len(fe[c])
            fb = sum(fe[c]) * ff * 1024 / n / 1e6
            wb = sum(wr.get(c, [0])) * wf * 1024 / max(len(wr.get(c, [0])), 1) / 1e6
            f.write(f"| {c} | {n / steps:.1f} | {fb:.1f} | {wb:.1f} | {(fb + wb) * n / steps:.0f} |\n")
            table[c] = round((fb + wb) * 1e6)
            total += (fb + wb) * n / steps
        f.write(f"\nAll classes together: {total / 1e3:.2f} GB of HBM traffic per step.\n")
    print(open(a.out).read())
    if a.workload:
        store = json.loads(TRAFFIC_JSON.read_text()) if TRAFFIC_JSON.exists() else {}
        store[a.workload] = {"sources": sources_digest(), "summary": str(Path(a.out).name),
                             "bytes_per_launch": table, "fetch_scale": ff, "write_scale": wf}
        TRAFFIC_JSON.write_text(json.dumps(store, indent=1, sort_keys=True) + "\n")


def cmd_movement(a) -> None:
    """Lowering / col2im on their own: movement_bench's event table next to the traffic of each launch.
    The counter files list dispatches in launch order; movement_bench launches, per dtype and layer,
    (warmup + iters) pairs of (lower, col2im)."""
    def launches(path):
        rows = list(csv.DictReader(open(path)))
        cal = max(float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"])
        seq = [(kernel_class(r["Kernel_Name"]), short_name(r["Kernel_Name"]), float(r["Counter_Value"])) for r in rows
               if kernel_class(r["Kernel_Name"]) in ("lower", "col2im")]
        return seq, cal
    fe, fcal = launches(a.fetch)
    wr, wcal = launches(a.write)
    ff, wf = CAL_KIB / fcal, CAL_KIB / wcal
    events = [json.loads(l) for l in open(a.bench_out) if l.startswith("{")]
    per = 2 * (a.warmup + a.iters)
    with open(a.out, "w") as f:
        f.write(f"# Batched lowering and col2im on their own against the HBM roofline: {a.title}\n\n")
        f.write("Commands (from /tmp with TMPDIR=/tmp on one MI355X):\n\n")
        for c in a.command:
            f.write(f"    {c}\n")
        f.write("\n`us` and `GB/s` come from the first command's own output (HIP events around each launch; rocprofv3's kernel trace of the\n"
                "same run agrees, see the second table); `fetched` / `written` are FETCH_SIZE / WRITE_SIZE of one launch of that layer, scaled by the\n"
                f"readings for the 256 MiB calibration copy ({ff:.4f} and {wf:.4f}).  Algorithmic bytes: the input once plus the lowered matrix once,\n"
                "(N C H W + K ld) e.  Peak: 8000 GB/s.\n\n")
        f.write("| kernel | layer | dtype | algorithmic MB | us | GB/s | of peak | fetched MB | written MB | kernel |\n|---|---|---|---|---|---|---|---|---|---|\n")
        for i, r in enumerate(events):
            blk, which = i // 2, (0 if r["kernel"] == "lower" else 1)
            j = blk * per + 2 * a.warmup + which            # first timed launch of this (dtype, layer, kernel)
            fmb = fe[j][2] * ff * 1024 / 1e6 if j < len(fe) else float("nan")
            wmb = wr[j][2] * wf * 1024 / 1e6 if j < len(wr) else float("nan")
            assert j >= len(fe) or fe[j][0] == r["kernel"], (i, j, fe[j], r["kernel"])
            f.write(f"| {r['kernel']} | {r['layer']} | {r['dtype']} | {r['algorithmic_bytes'] / 1e6:.0f} | {r['avg_launch_ms'] * 1e3:.1f} | "
                    f"{r['gbs']:.0f} | {r['frac_of_hbm_peak']:.2f} | {fmb:.0f} | {wmb:.0f} | {fe[j][1] if j < len(fe) else ''} |\n")
        if a.stats:
            f.write("\nrocprofv3 kernel statistics of the timed run (all layers and both dtypes together per kernel):\n\n| kernel | calls | avg us |\n|---|---|---|\n")
            for r in csv.DictReader(open(a.stats)):
                if kernel_class(r["Name"]) in ("lower", "col2im"):
                    f.write(f"| {short_name(r['Name'])} | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} |\n")
        if a.reading:
            f.write("\n" + a.reading + "\n")
    print(open(a.out).read())


def cmd_counters(a) -> None:
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in a.csv:
        for r in csv.DictReader(open(path)):
            agg[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    rows = []
    for k, d in agg.items():
        v = {c: sum(x) / len(x) for c, x in d.items()}
        if v.get("SQ_INSTS_MFMA", 0) > 0:
            n = len(d["GRBM_GUI_ACTIVE"])
            rows.append((v["GRBM_GUI_ACTIVE"] * n, short_name(k), n / a.steps, v))
    rows.sort(key=lambda r: -r[0])
    with open(a.out, "w") as f:
        f.write(f"# SQ counters of the matrix-core kernels (rocprofv3 --pmc): {a.title}\n\n")
        f.write("Commands (each from /tmp with TMPDIR=/tmp on one MI355X; one counter set per run):\n\n")
        for c in a.command:
            f.write(f"    {c}\n")
        f.write("\nAverages per launch.  `MFMA busy` = SQ_VALU_MFMA_BUSY_CYCLES / SQ_BUSY_CYCLES / 32: the counter adds up the SIMDs of a\n"
                "shader engine, so 32 (8 compute units x 4 SIMDs) is every matrix core busy all the time.  `LDS conflicts` =\n"
                "SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE (share of LDS-active cycles lost to bank conflicts).  `waiting` =\n"
                "SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES.  `VALU/MFMA`, `LDS/MFMA` = instructions issued per MFMA instruction.\n\n")
        f.write("| kernel | launches/step | GRBM_GUI_ACTIVE | MFMA insts | VALU/MFMA | LDS/MFMA | VMEM_RD insts | MFMA busy | LDS conflicts | waiting |\n"
                "|---|---|---|---|---|---|---|---|---|---|\n")
        for _, name, n, v in rows:
            mb = v["SQ_VALU_MFMA_BUSY_CYCLES"] / v["SQ_BUSY_CYCLES"] / 32
            f.write(f"| {name} | {n:.1f} | {v['GRBM_GUI_ACTIVE']:.0f} | {v['SQ_INSTS_MFMA']:.0f} | "
                    f"{v['SQ_INSTS_VALU'] / v['SQ_INSTS_MFMA']:.1f} | {v['SQ_INSTS_LDS'] / v['SQ_INSTS_MFMA']:.2f} | {v['SQ_INSTS_VMEM_RD']:.0f} | "
                    f"{mb:.2f} | {v['SQ_LDS_BANK_CONFLICT'] / max(v['SQ_LDS_IDX_ACTIVE'], 1):.2f} | "
                    f"{v['SQ_WAIT_INST_ANY'] / v['SQ_WAVE_CYCLES']:.2f} |\n")
        if a.reading:
            f.write("\n" + a.reading + "\n")
    print(open(a.out).read())


def cmd_pools(a) -> None:
    """SQ counters of the pool kernels from runs of pool_bench, beside pool_bench's own table."""
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in a.csv:
        for r in csv.DictReader(open(path)):
            if "maxpool" in r["Kernel_Name"]:
                agg[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    table = [l.rstrip("\n") for l in open(a.bench_out) if l.startswith("|")]
    with open(a.out, "w") as f:
        f.write(f"# The 3 x 3 / stride 2 max-pool kernels on their own: {a.title}\n\n")
        f.write("Commands (from /tmp with TMPDIR=/tmp on one MI355X; one counter set per rocprofv3 run):\n\n")
        for c in a.command:
            f.write(f"    {c}\n")
        f.write("\nTimes by the library's HIP events (first command).  `back to back`: the same launch repeated, operands stay in the\n"
                "last-level cache; `cold`: a 512 MiB fill between launches, operands come from memory as inside a training step.\n"
                "Peak: 8000 GB/s.\n\n")
        f.write("\n".join(table) + "\n\n")
        f.write("SQ counters, averages per launch over the three layers (back-to-back launches only).  `VALU busy` = 4 x SQ_INSTS_VALU /\n"
                "(32 x SQ_BUSY_CYCLES): a wave64 vector instruction occupies its SIMD for 4 cycles and SQ_BUSY_CYCLES adds up a shader\n"
                "engine's 32 SIMDs.  `waiting` = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES.  `waves per SIMD` = 4.25 x SQ_WAVE_CYCLES / (32 x\n"
                "SQ_BUSY_CYCLES): the counter ticks once per four cycles (a kernel with exactly two resident wavefronts per SIMD reads 0.47).\n\n")
        f.write("| kernel | launches | wavefronts | VALU insts per wavefront | LDS insts per wavefront | VALU busy | waiting | waves per SIMD |\n"
                "|---|---|---|---|---|---|---|---|\n")
        for k, d in agg.items():
            v = {c: sum(x) / len(x) for c, x in d.items()}
            n = len(d["SQ_WAVES"])
            f.write(f"| {short_name(k)} | {n} | {v['SQ_WAVES']:.0f} | {v['SQ_INSTS_VALU'] / v['SQ_WAVES']:.0f} | "
                    f"{v['SQ_INSTS_LDS'] / v['SQ_WAVES']:.0f} | {4 * v['SQ_INSTS_VALU'] / (32 * v['SQ_BUSY_CYCLES']):.2f} | "
                    f"{v['SQ_WAIT_INST_ANY'] / v['SQ_WAVE_CYCLES']:.2f} | {4.25 * v['SQ_WAVE_CYCLES'] / (32 * v['SQ_BUSY_CYCLES']):.1f} |\n")
        if a.reading:
            f.write("\n" + a.reading + "\n")
    print(open(a.out).read())


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    s = sub.add_parser("stats")
    s.add_argument("csv"), s.add_argument("bench_out")
    s.add_argument("--steps", type=int, required=True), s.add_argument("--out", required=True)
    s.add_argument("--title", required=True), s.add_argument("--command", required=True)
    s.set_defaults(fn=cmd_stats)
    t = sub.add_parser("traffic")
    t.add_argument("fetch"), t.add_argument("write")
    t.add_argument("--steps", type=int, required=True), t.add_argument("--out", required=True)
    t.add_argument("--title", required=True), t.add_argument("--command", required=True, help="with COUNTER where the counter name goes")
    t.add_argument("--workload", default="", help="key under which bench.py finds the table (its config.workload)")
    t.set_defaults(fn=cmd_traffic)
    c = sub.add_parser("counters")
    c.add_argument("csv", nargs="+")
    c.add_argument("--steps", type=int, required=True), c.add_argument("--out", required=True)
    c.add_argument("--title", required=True), c.add_argument("--command", action="append", required=True)
    c.add_argument("--reading", default="")
    c.set_defaults(fn=cmd_counters)
    m = sub.add_parser("movement")
    m.add_argument("fetch"), m.add_argument("write"), m.add_argument("bench_out")
    m.add_argument("--stats", default=""), m.add_argument("--iters", type=int, default=2), m.add_argument("--warmup", type=int, default=1)
    m.add_argument("--out", required=True), m.add_argument("--title", required=True)
    m.add_argument("--command", action="append", required=True), m.add_argument("--reading", default="")
    m.set_defaults(fn=cmd_movement)
    q = sub.add_parser("pools")
    q.add_argument("bench_out"), q.add_argument("csv", nargs="+")
    q.add_argument("--out", required=True), q.add_argument("--title", required=True)
    q.add_argument("--command", action="append", required=True), q.add_argument("--reading", default="")
    q.set_defaults(fn=cmd_pools)
    a = ap.parse_args()
    a.fn(a)


if __name__ == "__main__":
    main()
