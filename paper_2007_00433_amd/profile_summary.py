"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under
profiles/ (bench.py reads its `roofline.traffic` figure from the traffic table in them).

    python -m paper_2007_00433_amd.profile_summary <dir with stats/ fetch/ write/> <workload> <out stem>

Expected inputs (each produced by its own rocprofv3 run of bench.py, see the summary text):
    <dir>/stats/stats_kernel_stats.csv         --kernel-trace --stats
    <dir>/fetch/fetch_counter_collection.csv   --pmc FETCH_SIZE
    <dir>/write/write_counter_collection.csv   --pmc WRITE_SIZE
The counters are scaled by what they read for se_calib_copy_kernel, a plain copy whose
read and written byte counts are known exactly.
"""
from __future__ import annotations

import collections
import csv
import os
import sys


def kernel_key(name: str) -> str:
    """Classifies a kernel name.  The step kernels carry their mode as a template argument:
    se_step_kernel<VEC, BF16, HAS_V, HAS_WD, NT, MODE, BMAX> and
    se_coop_kernel<VEC, BF16, HAS_V, HAS_WD, NT, MODE> with MODE 0 = SESGD update,
    1 = gradient averaging (the ring baseline), 2 = average only."""
    for key in ("se_calib_copy_kernel", "se_plan_kernel", "se_consensus_kernel"):
        if key in name:
            return key
    for key in ("se_step_kernel", "se_coop_kernel"):
        if key in name and "<" in name:
            args = [a.strip() for a in name[name.index("<") + 1:name.index(">")].split(",")]
            mode = {"0": "sesgd", "1": "ring", "2": "avgonly"}.get(args[5], args[5])
            return f"{mode}"
    return ""


def counters(path: str) -> dict:
    agg = collections.defaultdict(list)
    with open(path) as f:
        for r in csv.DictReader(f):
            k = kernel_key(r["Kernel_Name"])
            if k:
                agg[k].append(float(r["Counter_Value"]))
    return {k: (sum(v) / len(v), len(v)) for k, v in agg.items()}


def main():
    src, workload, stem = sys.argv[1], sys.argv[2], sys.argv[3]
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    from paper_2007_00433_amd import workloads as wl
    w = wl.WORKLOADS[workload]
    pitch = (w.P + 1023) // 1024 * 1024              # se_pitch(P)
    rd = w.n * w.P * (8 + w.grad_bytes)              # algorithmic: the P real elements per worker
    wr = w.n * w.P * 8
    copy_bytes = w.n * pitch * w.grad_bytes          # bench.py copies one gradient buffer

    stats = {}
    with open(os.path.join(src, "stats", "stats_kernel_stats.csv")) as f:
        for r in csv.DictReader(f):
            k = kernel_key(r["Name"])
            if k:
                stats[k] = {"name": r["Name"], "calls": int(r["Calls"]), "avg_ns": float(r["AverageNs"]),
                            "min_ns": float(r["MinNs"]), "max_ns": float(r["MaxNs"])}
    fetch = counters(os.path.join(src, "fetch", "fetch_counter_collection.csv"))
    write = counters(os.path.join(src, "write", "write_counter_collection.csv"))
    f_scale = (copy_bytes / 1024.0) / fetch["se_calib_copy_kernel"][0]
    w_scale = (copy_bytes / 1024.0) / write["se_calib_copy_kernel"][0]

    out = {"workload": workload, "n": w.n, "group_size": w.group_size, "pitch": pitch,
           "copy_bytes_each_way": copy_bytes,
           "fetch_scale_kib_per_count": f_scale, "write_scale_kib_per_count": w_scale, "kernels": {}}
    lines = [f"# rocprofv3 summary: se_step / se_ring_step, {workload}-shaped workload "
             f"(n={w.n}, group_size={w.group_size}, pitch={pitch})", "",
             "Commands (run from /tmp with TMPDIR=/tmp on the MI355X box; R = repository root):", "",
             f"    rocprofv3 --kernel-trace --stats -d OUT/stats -o stats --output-format csv -- python3 R/bench.py --skip-cpu-baseline --workload {workload}",
             f"    rocprofv3 --pmc FETCH_SIZE -d OUT/fetch -o fetch --output-format csv -- python3 R/bench.py --skip-cpu-baseline --steps 6 --warmup 2 --workload {workload}",
             f"    rocprofv3 --pmc WRITE_SIZE -d OUT/write -o write --output-format csv -- python3 R/bench.py --skip-cpu-baseline --steps 6 --warmup 2 --workload {workload}",
             f"    python -m paper_2007_00433_amd.profile_summary OUT {workload} profiles/{os.path.basename(stem)}", "",
             "## Kernel durations (--kernel-trace --stats)", "",
             "Rows: `sesgd` = se_step (SESGD update), `ring` = se_ring_step (gradient averaging over all n).",
             "",
             "| what | kernel | calls | avg ns | min ns | max ns | algorithmic bytes | GB/s at avg | % of 8 TB/s |",
             "|---|---|---|---|---|---|---|---|---|"]
    for k in ("sesgd", "ring", "se_calib_copy_kernel"):
        if k not in stats:
            continue
        s = stats[k]
        alg = 2 * copy_bytes if k == "se_calib_copy_kernel" else rd + wr
        gbs = alg / s["avg_ns"]
        lines.append(f"| {k} | `{s['name'][:62]}` | {s['calls']} | {s['avg_ns']:.0f} | {s['min_ns']:.0f} | "
                     f"{s['max_ns']:.0f} | {alg} | {gbs:.1f} | {gbs / 80.0:.1f} |")
        out["kernels"][k] = {"avg_ns": s["avg_ns"], "calls": s["calls"], "algorithmic_bytes": alg,
                             "gbs": gbs}
    lines += ["", "## HBM traffic per launch (--pmc FETCH_SIZE, --pmc WRITE_SIZE; one run each)", "",
              f"Scale factors from the plain copy kernel, which reads and writes exactly {copy_bytes} bytes "
              f"({copy_bytes / 1024:.0f} KiB): FETCH_SIZE reads {fetch['se_calib_copy_kernel'][0]:.1f} -> "
              f"{f_scale:.5f} KiB per count; WRITE_SIZE reads {write['se_calib_copy_kernel'][0]:.1f} -> "
              f"{w_scale:.5f} KiB per count.", "",
              "| kernel | FETCH_SIZE avg | WRITE_SIZE avg | read bytes | written bytes | traffic bytes | algorithmic bytes | traffic / algorithmic |",
              "|---|---|---|---|---|---|---|---|"]
    for k in ("sesgd", "ring"):
        if k not in fetch or k not in write:
            continue
        rb = fetch[k][0] * f_scale * 1024.0
        wb = write[k][0] * w_scale * 1024.0
        lines.append(f"| {k} | {fetch[k][0]:.1f} | {write[k][0]:.1f} | {rb:.0f} | {wb:.0f} | {rb + wb:.0f} | "
                     f"{rd + wr} | {(rb + wb) / (rd + wr):.5f} |")
        out["kernels"].setdefault(k, {}).update({"fetch_count": fetch[k][0], "write_count": write[k][0],
                                                 "read_bytes": rb, "written_bytes": wb,
                                                 "traffic_bytes": rb + wb})
    with open(stem + ".md", "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
