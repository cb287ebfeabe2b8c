#!/usr/bin/env python3
"""Turns the raw rocprofv3 output of bench.py runs into the short summaries under profiles/.

Three runs of the same bench.py command belong together (each in a run of its own, from /tmp on
the GPU machine, R = repository root):

    rocprofv3 --kernel-trace --stats --output-format csv -d $R/gpurun_out/<tag>/kt -o kt -- \\
        python3 $R/bench.py <bench args> --no-cpu-baseline --no-group-view
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d $R/gpurun_out/<tag>/fetch -o fetch -- \\
        python3 $R/bench.py <bench args> --steps 2 --warmup 0 --no-cpu-baseline --no-group-view --calibration-copy
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d $R/gpurun_out/<tag>/write -o write -- \\
        python3 $R/bench.py <bench args> --steps 2 --warmup 0 --no-cpu-baseline --no-group-view --calibration-copy

and then, here:

    python profile_summary.py --dir gpurun_out/<tag> --config h8192 --view rank \\
        --bench-args "<bench args>" --out profiles/<name>.md

The summary holds the kernel trace statistics, the counters scaled by what they read for a plain
copy of known size (the first reorder dispatch of the two counter runs), the algorithmic bytes of
every kernel, and -- for the dominant kernel -- the HBM bytes per launch that bench.py reports as
`roofline.traffic`.  That figure is also written to profiles/hbm_traffic_per_launch.txt next to
the SHA-256 of the kernel source it was measured on; bench.py emits it only while that hash still
matches.  Nothing here runs on the GPU.
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
KERNEL_SOURCE = os.path.join(ROOT, "paper_2205_00119_amd", "csrc", "kernels.hip")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
KIB = 1024


def short_name(name: str) -> str:
    name = name.replace("mics::(anonymous namespace)::", "").replace("void ", "")
    name = re.sub(r"mics::PtrTable|SmallTable<\d+>", "", name)
    cut = name.find("(")
    name = name if cut < 0 else name[:cut]
    name = re.sub(r",\s*>", ">", name).strip()
    if name.startswith("at::native"):
        return "at::native elementwise kernel (torch fill / zero)"
    return name


def template_args(name: str):
    m = re.search(r"<(.*)>", name)
    if not m:
        return []
    out = []
    for tok in m.group(1).split(","):
        tok = tok.strip()
        out.append({"true": True, "false": False}.get(tok, int(tok) if re.fullmatch(r"-?\d+", tok) else tok))
    return out


def algorithmic_bytes(name: str, cfg, count: int, N: int, pb: int):
    """Bytes the method must move in one launch of the kernel `name` (None: not a libmics kernel)."""
    a = template_args(name)
    p, r = cfg.p, cfg.r
    if name.startswith("reorder_"):
        return 2 * pb * N
    if name.startswith("rsa_kernel"):
        gb = 4 if a[0] == 2 else 2
        return count * (gb * p + (8 if a[3] else 4))
    if name.startswith("rsa_seg_kernel"):
        return count * (2 * p + (8 if a[1] else 4))
    if name.startswith("avg_kernel"):
        return count * (4 * r + 4)
    if name.startswith("adam_kernel"):
        return count * (16 + (14 if a[0] else 12))
    if name.startswith("avg_adam_kernel"):
        return count * (4 * r + 12 + (14 if a[1] else 12))
    return None


def one(pattern):
    hits = glob.glob(pattern, recursive=True)
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return sorted(hits)[-1]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dir", required=True, help="folder with kt/, fetch/ and write/ (fetch/write optional)")
    ap.add_argument("--config", default="h8192")
    ap.add_argument("--view", choices=["rank", "group"], default="rank")
    ap.add_argument("--variant", default="flat-bf16")
    ap.add_argument("--count", type=int, default=0, help="elements per reduce/average/Adam call if not the view's")
    ap.add_argument("--numel", type=int, default=0, help="elements of the gathered layer if not the configuration's")
    ap.add_argument("--bench-args", default="")
    ap.add_argument("--out", required=True)
    ap.add_argument("--no-traffic-file", action="store_true")
    ap.add_argument("--append", action="store_true", help="append to --out instead of replacing it")
    ap.add_argument("--title", default="", help="heading for this run (variants collected in one file)")
    args = ap.parse_args()

    import synth
    cfg = synth.CONFIGS[args.config]
    N = args.numel or cfg.N
    count = args.count or (cfg.N_pad if args.view == "group" else cfg.S)
    pb = 2
    sha = hashlib.sha256(open(KERNEL_SOURCE, "rb").read()).hexdigest()[:16]
    out = [(f"\n---\n\n## {args.title}\n\n" if args.title else "") +
           f"# rocprofv3 summary: libmics kernels, workload {cfg.name} (p={cfg.p}, k={cfg.k}, r={cfg.r}, "
           f"s={cfg.s}), {args.view} view ({count} elements per reduce/average/Adam call), one MI355X\n",
           f"Kernel source: `paper_2205_00119_amd/csrc/kernels.hip`, SHA-256 `{sha}`.\n",
           "Commands (from /tmp on the GPU box, `R` = repository root; each in a run of its own), then "
           f"`python profile_summary.py --dir {args.dir} --config {args.config} --view {args.view} "
           f"--variant {args.variant} --bench-args \"{args.bench_args}\" --out {args.out}`:\n",
           "```"]
    extra = "" if args.view == "group" or "--view" in args.bench_args else " --no-group-view"
    b = f"python3 $R/bench.py {args.bench_args}".rstrip()
    out.append(f"rocprofv3 --kernel-trace --stats --output-format csv -d $R/{args.dir}/kt -o kt -- {b} --no-cpu-baseline{extra}")
    have_pmc = os.path.isdir(os.path.join(args.dir, "fetch")) and os.path.isdir(os.path.join(args.dir, "write"))
    if have_pmc:
        for c, tag in (("FETCH_SIZE", "fetch"), ("WRITE_SIZE", "write")):
            out.append(f"rocprofv3 --pmc {c} --output-format csv -d $R/{args.dir}/{tag} -o {tag} -- {b} --steps 2 "
                       f"--warmup 0 --no-cpu-baseline{extra} --calibration-copy")
    out.append("```\n")

    # ---- kernel trace ---------------------------------------------------------------------------
    avg_ns, calls = {}, {}
    out.append("## Kernel trace (`kt_kernel_stats.csv`)\n")
    out.append("| kernel | calls | total ns | average ns | min ns | max ns | stddev | algorithmic bytes | GB/s at the average |")
    out.append("|---|---|---|---|---|---|---|---|---|")
    for row in csv.DictReader(open(one(os.path.join(args.dir, "kt", "**", "*kernel_stats.csv")))):
        n = short_name(row["Name"])
        avg_ns[n], calls[n] = float(row["AverageNs"]), int(row["Calls"])
        alg = algorithmic_bytes(n, cfg, count, N, pb)
        rate = f"{alg / avg_ns[n]:.0f}" if alg else ""
        out.append(f"| `{n}` | {row['Calls']} | {row['TotalDurationNs']} | {avg_ns[n]:.0f} | {row['MinNs']} | "
                   f"{row['MaxNs']} | {float(row['StdDev']):.0f} | {alg or ''} | {rate} |")
    out.append("\n`synth_fill_kernel` and the torch fills are input generation, outside the timed region.\n")
    log = os.path.join(args.dir, "kt.log")
    if os.path.exists(log):
        lines = [l for l in open(log) if l.startswith("{")]
        if lines:
            bench = json.loads(lines[-1])
            rf = bench["roofline"]
            out.append(f"The same run's bench.py line: ms_per_step {bench['ms_per_step']}, value {bench['value']} GB/s "
                       f"({bench['pct_of_peak_hbm']} % of 8 TB/s); `roofline`: kernel `{rf['kernel']}`, avg_launch_ms "
                       f"{rf['avg_launch_ms']} (HIP events around the s launches of a step), median "
                       f"{rf['median_launch_ms']}, min {rf['min_launch_ms']}, achieved {rf['achieved']} GB/s, frac {rf['frac']}.")
            rsa = sorted(n for n in avg_ns if n.startswith(("rsa_kernel", "rsa_seg_kernel")))
            acc = [n for n in rsa if template_args(n)[3 if n.startswith("rsa_kernel") else 1]]
            ovw = [n for n in rsa if n not in acc]
            if len(acc) == 1 and len(ovw) == 1 and cfg.s > 1:
                mix = ((cfg.s - 1) * avg_ns[acc[0]] + avg_ns[ovw[0]]) / cfg.s
                out.append(f"From the trace: ({cfg.s - 1} x {avg_ns[acc[0]] / 1e3:.2f} + {avg_ns[ovw[0]] / 1e3:.2f}) / "
                           f"{cfg.s} = {mix / 1e3:.1f} us per launch of the dominant kernel.\n")

    # ---- counters -------------------------------------------------------------------------------
    if have_pmc:
        rows, cal = {}, {}
        for tag in ("fetch", "write"):
            recs = list(csv.DictReader(open(one(os.path.join(args.dir, tag, "**", "*counter_collection.csv")))))
            recs.sort(key=lambda row: int(row["Dispatch_Id"]))
            for row in recs:
                n = short_name(row["Kernel_Name"])
                if algorithmic_bytes(n, cfg, count, N, pb) is None:
                    continue
                if tag not in cal and n.startswith("reorder_"):
                    cal[tag] = (n, float(row["Counter_Value"]))      # the calibration copy comes first
                    continue
                rows.setdefault(n, {}).setdefault(tag, []).append(float(row["Counter_Value"]))
        if len(cal) != 2:
            raise SystemExit("no calibration copy (first reorder dispatch) in the counter runs")
        cal_kib = pb * N / KIB
        ff, fw = cal_kib / cal["fetch"][1], cal_kib / cal["write"][1]
        out.append("## HBM traffic per dispatch (`--pmc FETCH_SIZE`, `--pmc WRITE_SIZE`; counters in KiB)\n")
        out.append(f"Calibration: the first reorder dispatch of these two runs (`{cal['fetch'][0]}`) is a plain copy "
                   f"(p = k = 1) of N = {N} bf16 = {cal_kib:.0f} KiB read and as much written. FETCH_SIZE reads "
                   f"{cal['fetch'][1]:.1f} and WRITE_SIZE reads {cal['write'][1]:.1f} for it, so the scale factors are "
                   f"**{ff:.4f}** (fetch) and **{fw:.4f}** (write).\n")
        out.append("| kernel | dispatches | FETCH_SIZE avg | x factor = KiB read | WRITE_SIZE avg | x factor = KiB written | traffic bytes | algorithmic bytes | ratio |")
        out.append("|---|---|---|---|---|---|---|---|---|")
        traffic = {}
        for n, v in sorted(rows.items()):
            f, w = v.get("fetch", []), v.get("write", [])
            if not f or not w:
                continue
            fa, wa = sum(f) / len(f), sum(w) / len(w)
            traffic[n] = (fa * ff + wa * fw) * KIB
            alg = algorithmic_bytes(n, cfg, count, N, pb)
            out.append(f"| `{n}` | {len(f)} | {fa:.1f} | {fa * ff:.0f} | {wa:.1f} | {wa * fw:.0f} | {traffic[n]:.0f} | {alg} | "
                       f"{traffic[n] / alg:.4f} |")
        worst = max(abs(traffic[n] / algorithmic_bytes(n, cfg, count, N, pb) - 1) for n in traffic)
        out.append(f"\nTraffic equals the algorithmic bytes to within {worst * 100:.2f} % for every kernel.  (FETCH_SIZE and "
                   "WRITE_SIZE sit between L2 and the fabric: bytes served by the Infinity Cache count as well.)")
        rsa = sorted(n for n in traffic if n.startswith(("rsa_kernel", "rsa_seg_kernel")))
        acc = [n for n in rsa if template_args(n)[3 if n.startswith("rsa_kernel") else 1]]
        ovw = [n for n in rsa if n not in acc]
        if len(acc) == 1 and len(ovw) == 1:
            per_launch = ((cfg.s - 1) * traffic[acc[0]] + traffic[ovw[0]]) / cfg.s
            out.append(f"Per launch of the dominant kernel, averaged over a step: ({cfg.s - 1} x {traffic[acc[0]]:.0f} + "
                       f"{traffic[ovw[0]]:.0f}) / {cfg.s} = {per_launch:.0f} bytes (bench.py `roofline.traffic`).\n")
            if not args.no_traffic_file:
                key = [cfg.name, args.view, args.variant]
                keep = []
                if os.path.exists(TRAFFIC_FILE):
                    keep = [l for l in open(TRAFFIC_FILE).read().splitlines()
                            if l.startswith("#") or l.split()[:3] != key]
                if not keep:
                    keep = ["# HBM bytes per launch of the dominant kernel (reduce-scatter-accumulate, averaged over a step's",
                            "# s launches) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, written by profile_summary.py.",
                            "# workload view variant sha256-16(kernels.hip) bytes fetch_factor write_factor summary"]
                keep.append(f"{cfg.name} {args.view} {args.variant} {sha} {per_launch:.0f} {ff:.4f} {fw:.4f} {args.out}")
                open(TRAFFIC_FILE, "w").write("\n".join(keep) + "\n")
    open(args.out, "a" if args.append else "w").write("\n".join(out) + "\n")
    print("\n".join(out))


if __name__ == "__main__":
    main()
