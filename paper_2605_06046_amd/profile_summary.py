"""Turns raw rocprofv3 output of bench.py into the short summaries kept under profiles/.

    python -m paper_2605_06046_amd.profile_summary <raw_dir> <workload> <out_dir>

<raw_dir> holds, for workload W (e.g. c2), the outputs of these three commands
(run from /tmp with TMPDIR=/tmp; bench.py by absolute path):

    rocprofv3 --kernel-trace --stats -d <raw_dir>/trace_W -o t --output-format csv -- \\
        python3 bench.py --workload W --no-cpu-baseline --no-configs --no-hbm-calibration --steps 200 --warmup 20
    rocprofv3 --pmc FETCH_SIZE --kernel-trace -d <raw_dir>/pmc_FETCH_SIZE_W -o p --output-format csv -- \\
        python3 bench.py --workload W --no-cpu-baseline --no-configs --no-hbm-calibration --steps 40 --warmup 4 --copy-calibration
    rocprofv3 --pmc WRITE_SIZE --kernel-trace -d <raw_dir>/pmc_WRITE_SIZE_W -o p --output-format csv -- \\
        python3 bench.py --workload W --no-cpu-baseline --no-configs --no-hbm-calibration --steps 40 --warmup 4 --copy-calibration

optionally the L2 cache's hits and misses,

    rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum --kernel-trace -d <raw_dir>/pmc_L2_W -o p --output-format csv -- \\
        python3 bench.py --workload W --no-cpu-baseline --no-configs --no-hbm-calibration --steps 40 --warmup 4

and, optionally, <raw_dir>/untraced_W.json: the output line of the first command run
without the profiler.  Under the profiler the library's own per-dispatch events are
off (fea_profile_enable refuses while a profiling tool is attached, and bench.py then
reports no kernel durations of its own), so that line is the one whose live-measured
kernel duration is set against the profiler's.

--copy-calibration makes bench.py start with three plain 1 GiB device-to-device
copies; what the counters read for them fixes the scale of each counter.
"""
from __future__ import annotations

import csv
import glob
import hashlib
import json
import os
import sys

GIB_KIB = 1 << 20   # a 1 GiB copy moves this many KiB each way


def kernel_rev(root: str) -> str:
    """Identifies the sweep kernel's code: its source files.  The counters of a summary stay valid for
    a build whose sweep source is the same and whose plan for the workload (stored next to them) is the
    same, since the kernel then does the same loads and stores."""
    h = hashlib.sha256()
    for name in ("fea_sweep_mfma.hip", "fea_sweep_core.inc", "fea_plan.h"):
        h.update(open(os.path.join(root, "paper_2605_06046_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:12]


def _one(pattern: str) -> str:
    hits = glob.glob(pattern, recursive=True)
    if not hits:
        raise SystemExit(f"nothing matches {pattern}")
    return hits[0]


def _counter(raw: str, name: str, wl: str):
    rows = [r for r in csv.DictReader(open(_one(f"{raw}/pmc_{name}_{wl}/**/*counter_collection.csv")))
            if r["Counter_Name"] == name]
    per = {}
    for r in rows:
        per.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    copies = sorted(v for k, vs in per.items() if "copyBuffer" in k for v in vs)[-3:]
    scale = GIB_KIB / (sum(copies) / len(copies))
    return per, scale, copies


def main(raw: str, wl: str, out: str) -> None:
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    os.makedirs(out, exist_ok=True)
    stats = list(csv.DictReader(open(_one(f"{raw}/trace_{wl}/**/*kernel_stats.csv"))))
    ours = [r for r in stats if r["Name"].startswith(("fea::", "void fea::"))]
    lines = ["Commands (from /tmp with TMPDIR=/tmp, bench.py by its absolute path; raw output in <raw>):",
             f"  rocprofv3 --kernel-trace --stats -d <raw>/trace_{wl} -o t --output-format csv -- python3 bench.py --workload {wl} --no-cpu-baseline --no-configs --no-hbm-calibration --steps 200 --warmup 20",
             f"  rocprofv3 --pmc FETCH_SIZE --kernel-trace -d <raw>/pmc_FETCH_SIZE_{wl} -o p --output-format csv -- python3 bench.py --workload {wl} --no-cpu-baseline --no-configs --no-hbm-calibration --steps 40 --warmup 4 --copy-calibration",
             f"  rocprofv3 --pmc WRITE_SIZE --kernel-trace -d <raw>/pmc_WRITE_SIZE_{wl} -o p --output-format csv -- python3 bench.py --workload {wl} --no-cpu-baseline --no-configs --no-hbm-calibration --steps 40 --warmup 4 --copy-calibration",
             f"  rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum --kernel-trace -d <raw>/pmc_L2_{wl} -o p --output-format csv -- python3 bench.py --workload {wl} --no-cpu-baseline --no-configs --no-hbm-calibration --steps 40 --warmup 4    (optional)",
             f"  python3 bench.py --workload {wl} --no-cpu-baseline --no-configs --no-hbm-calibration --steps 200 --warmup 20    (no profiler)",
             f"  python3 -m paper_2605_06046_amd.profile_summary <raw> {wl} profiles",
             "", "Kernel trace (library kernels only; durations in microseconds)", "",
             f"{'kernel':58s} {'calls':>6s} {'avg':>9s} {'min':>9s} {'max':>9s} {'share':>7s}"]
    for r in ours:
        lines.append(f"{r['Name'][:58]:58s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e3:9.2f} "
                     f"{float(r['MinNs']) / 1e3:9.2f} {float(r['MaxNs']) / 1e3:9.2f} {float(r['Percentage']):6.2f}%")
    sweep = max((r for r in ours if "sweep" in r["Name"]), key=lambda r: float(r["TotalDurationNs"]))
    res = {"workload": wl, "kernel": sweep["Name"], "avg_us": float(sweep["AverageNs"]) / 1e3,
           "kernel_rev": kernel_rev(root)}
    lines += ["", "HBM traffic of the sweep kernel per launch (rocprofv3 --pmc, one counter per run):"]
    total = 0.0
    for name in ("FETCH_SIZE", "WRITE_SIZE"):
        per, scale, copies = _counter(raw, name, wl)
        vals = next(v for k, v in per.items() if "sweep" in k)
        mean = sum(vals) / len(vals)
        lines.append(f"  {name}: {mean:12.1f} KiB raw over {len(vals)} launches; 1 GiB copies read "
                     f"{[round(c, 1) for c in copies]} KiB -> scale {scale:.4f} -> {mean * scale * 1024 / 1e6:9.2f} MB")
        res[name.lower() + "_kib_raw"] = mean
        res[name.lower() + "_scale"] = scale
        total += mean * scale * 1024
        for k, v in per.items():
            if "merge_kernel" in k or "plan_kernel" in k:
                lines.append(f"      ({k[:40]}: {sum(v) / len(v) * scale * 1024 / 1e6:8.2f} MB per launch)")
    res["traffic_bytes_per_launch"] = total
    bench = json.loads(open(f"{raw}/trace_{wl}.json").read().strip().splitlines()[-1])
    res["unique_kv_bytes"] = bench["roofline"]["bytes_per_launch"]
    res["plan"] = bench["plan"]
    lines += [f"  total {total / 1e6:.2f} MB per launch; algorithmic (distinct live KV blocks, K and V): "
              f"{res['unique_kv_bytes'] / 1e6:.2f} MB; ratio {total / res['unique_kv_bytes']:.3f}",
              ""]
    l2 = glob.glob(f"{raw}/pmc_L2_{wl}/**/*counter_collection.csv", recursive=True)
    if l2:   # requests the L2 served against those it passed on, per kernel
        acc = {}
        for r in csv.DictReader(open(l2[0])):
            if r["Counter_Name"] in ("TCC_HIT_sum", "TCC_MISS_sum") and r["Kernel_Name"].startswith(("fea::", "void fea::")):
                d = acc.setdefault(r["Kernel_Name"], {"TCC_HIT_sum": 0.0, "TCC_MISS_sum": 0.0, "n": 0})
                d[r["Counter_Name"]] += float(r["Counter_Value"])
                d["n"] += r["Counter_Name"] == "TCC_HIT_sum"
        lines += ["L2 cache (rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum, requests per launch):"]
        for k, d in acc.items():
            n = max(d["n"], 1)
            tot = d["TCC_HIT_sum"] + d["TCC_MISS_sum"]
            lines.append(f"  {k[:58]:58s} hits {d['TCC_HIT_sum'] / n:12.0f}  misses {d['TCC_MISS_sum'] / n:12.0f}  hit rate {d['TCC_HIT_sum'] / max(tot, 1):.3f}")
            if "sweep" in k:
                res["l2_hit_rate"] = d["TCC_HIT_sum"] / max(tot, 1)
        lines.append("")
    un = f"{raw}/untraced_{wl}.json"
    if os.path.exists(un):
        b2 = json.loads(open(un).read().strip().splitlines()[-1])
        lines += ["bench.py line of the same command without the profiler:",
                  f"  sweep avg {b2['kernel_us']['sweep']:.2f} us by HIP events vs {res['avg_us']:.2f} us by rocprofv3; "
                  f"roofline.achieved {b2['roofline']['achieved']:.0f} GB/s = {b2['roofline']['frac']:.3f} of 8000; "
                  f"whole step {b2['ms_per_step'] * 1e3:.1f} us = {b2['value']:.0f} {b2['unit']}"]
    open(os.path.join(out, f"sweep_mfma_{wl}_trace.txt"), "w").write("\n".join(lines) + "\n")
    json.dump(res, open(os.path.join(out, f"sweep_mfma_{wl}_pmc.json"), "w"), indent=1)
    print("\n".join(lines))


if __name__ == "__main__":
    if len(sys.argv) != 4:
        raise SystemExit(__doc__)
    main(*sys.argv[1:])
