#!/usr/bin/env python3
"""Turns the rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under
profiles/ (bench.py reads its `roofline.traffic` figure from the traffic table in them).

    python profile_summary.py <dir> <workload> <out stem>

<dir> holds one sub-directory and one log per rocprofv3 run of bench.py (the commands are printed
into the summary): stats/ (--kernel-trace --stats), fetch/ (--pmc FETCH_SIZE), write/
(--pmc WRITE_SIZE) and, optionally, stall/ (--pmc write-request stall counters of the L2), with
stats.log, fetch.log, write.log, stall.log holding the JSON line bench.py printed in that run.

A call of the library can be several launches (the split form issues two per chunk of columns),
so all figures are per CALL: the sum over the dispatches of a class divided by the number of
calls bench.py reports in `api_calls`.  The byte counters are scaled by what they read for
se_calib_copy_kernel, a plain copy whose read and written byte counts are known exactly.
"""
from __future__ import annotations

import collections
import csv
import json
import os
import sys

MODES = {"0": "se_step", "1": "se_ring_step", "2": "se_global_average"}
MODE_ARG = {"se_step_kernel": 5, "se_coop_kernel": 5, "se_split_reduce_kernel": 4, "se_split_finish_kernel": 3}


def kernel_class(name: str) -> str:
    """The entry point a dispatch belongs to.  The step kernels carry their mode as a template
    argument (0 = SESGD update, 1 = gradient averaging = the ring baseline in bench.py,
    2 = average only)."""
    if "se_calib_copy_kernel" in name:
        return "se_calib_copy"
    for key, pos in MODE_ARG.items():
        if key + "<" in name:
            args = [a.strip() for a in name[name.index("<") + 1:name.index(">")].split(",")]
            return MODES.get(args[pos], "")
    return ""


def short(name: str) -> str:
    return name[name.index("se::") + 4:name.index("(")] if "se::" in name and "(" in name else name


def bench_line(path: str) -> dict:
    with open(path) as f:
        lines = [l for l in f if l.startswith("{")]
    return json.loads(lines[-1])


def counter_sums(path: str) -> dict:
    """{(class, counter): sum over all dispatches}"""
    agg = collections.defaultdict(float)
    with open(path) as f:
        for r in csv.DictReader(f):
            k = kernel_class(r["Kernel_Name"])
            if k:
                agg[(k, r["Counter_Name"])] += float(r["Counter_Value"])
    return agg


def main():
    src, workload, stem = sys.argv[1], sys.argv[2], sys.argv[3]
    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, here)
    from paper_2007_00433_amd import workloads as wl
    w = wl.WORKLOADS[workload]
    pitch = (w.P + 1023) // 1024 * 1024              # se_pitch(P)
    rd = w.n * w.P * (8 + w.grad_bytes)              # algorithmic: the P real elements per worker
    wr = w.n * w.P * 8
    copy_bytes = w.n * pitch * w.grad_bytes          # bench.py copies one gradient buffer

    flags = f"--skip-cpu-baseline --reallocs 0 --workload {workload}"
    lines = [f"# rocprofv3 summary: se_step / se_ring_step, {workload}-shaped workload "
             f"(n={w.n}, group_size={w.group_size}, pitch={pitch})", "",
             "Commands (run from /tmp with TMPDIR=/tmp on the MI355X box; R = repository root):", "",
             f"    rocprofv3 --kernel-trace --stats -d OUT/stats -o stats --output-format csv -- python3 R/bench.py {flags} > OUT/stats.log",
             f"    rocprofv3 --pmc FETCH_SIZE -d OUT/fetch -o fetch --output-format csv -- python3 R/bench.py {flags} --steps 6 --warmup 2 > OUT/fetch.log",
             f"    rocprofv3 --pmc WRITE_SIZE -d OUT/write -o write --output-format csv -- python3 R/bench.py {flags} --steps 6 --warmup 2 > OUT/write.log",
             f"    rocprofv3 --pmc TCC_EA0_WRREQ_sum TCC_EA0_WRREQ_STALL_sum TCC_EA0_WRREQ_DRAM_CREDIT_STALL_sum TCC_CYCLE_sum -d OUT/stall -o stall --output-format csv -- python3 R/bench.py {flags} --steps 6 --warmup 2 > OUT/stall.log",
             f"    python3 R/profile_summary.py OUT {workload} R/profiles/{os.path.basename(stem)}", "",
             "All figures are per CALL of the entry point (a call may be several launches): the sum over",
             "its dispatches divided by the number of calls bench.py made (`api_calls` of its JSON line).", ""]

    # ---- durations
    b = bench_line(os.path.join(src, "stats.log"))
    calls = b["api_calls"]
    per_class = collections.defaultdict(list)
    with open(os.path.join(src, "stats", "stats_kernel_stats.csv")) as f:
        for r in csv.DictReader(f):
            k = kernel_class(r["Name"])
            if k:
                per_class[k].append((short(r["Name"]), int(r["Calls"]), float(r["TotalDurationNs"]),
                                     float(r["AverageNs"])))
    lines += ["## Kernel durations (--kernel-trace --stats) next to the bench line of the same process", "",
              f"bench.py in this process: `ms_per_step` {b['ms_per_step']}, `roofline.avg_launch_ms` "
              f"{b['roofline']['avg_launch_ms']} (stream events), value {b['value']} steps/s"
              + (f", ring {b['ring_baseline']['achieved_gbs']} GB/s" if "ring_baseline" in b else "") + ".", "",
              "| entry point | kernels (dispatches, average ns each) | calls | ns per call | algorithmic bytes | GB/s | % of 8 TB/s |",
              "|---|---|---|---|---|---|---|"]
    for k in ("se_step", "se_ring_step", "se_calib_copy"):
        if k not in per_class or not calls.get(k):
            continue
        total = sum(t for _, _, t, _ in per_class[k])
        per_call = total / calls[k]
        alg = 2 * copy_bytes if k == "se_calib_copy" else rd + wr
        kernels = "; ".join(f"`{n}` ({c}, {a:.0f})" for n, c, _, a in per_class[k])
        lines.append(f"| {k} | {kernels} | {calls[k]} | {per_call:.0f} | {alg} | {alg / per_call:.1f} | "
                     f"{alg / per_call / 80.0:.1f} |")

    # ---- traffic
    fpath = os.path.join(src, "fetch", "fetch_counter_collection.csv")
    wpath = os.path.join(src, "write", "write_counter_collection.csv")
    if os.path.exists(fpath) and os.path.exists(wpath):
        fetch, write = counter_sums(fpath), counter_sums(wpath)
        fcalls = bench_line(os.path.join(src, "fetch.log"))["api_calls"]
        wcalls = bench_line(os.path.join(src, "write.log"))["api_calls"]
        f_copy = fetch[("se_calib_copy", "FETCH_SIZE")] / fcalls["se_calib_copy"]
        w_copy = write[("se_calib_copy", "WRITE_SIZE")] / wcalls["se_calib_copy"]
        f_scale, w_scale = (copy_bytes / 1024.0) / f_copy, (copy_bytes / 1024.0) / w_copy
        lines += ["", "## HBM traffic per call (--pmc FETCH_SIZE, --pmc WRITE_SIZE; one run each)", "",
                  f"Scale factors from the plain copy kernel, which reads and writes exactly {copy_bytes} bytes "
                  f"({copy_bytes / 1024:.0f} KiB): FETCH_SIZE reads {f_copy:.1f} -> {f_scale:.5f} KiB per count; "
                  f"WRITE_SIZE reads {w_copy:.1f} -> {w_scale:.5f} KiB per count.", "",
                  "| entry point | FETCH_SIZE per call | WRITE_SIZE per call | read bytes | written bytes | traffic bytes | algorithmic bytes | traffic / algorithmic |",
                  "|---|---|---|---|---|---|---|---|"]
        for k in ("se_step", "se_ring_step"):
            if not fcalls.get(k) or (k, "FETCH_SIZE") not in fetch:
                continue
            fc = fetch[(k, "FETCH_SIZE")] / fcalls[k]
            wc = write[(k, "WRITE_SIZE")] / wcalls[k]
            rb, wb = fc * f_scale * 1024.0, wc * w_scale * 1024.0
            # bench.py parses this row: entry point in cell 1, traffic bytes in cell 6
            lines.append(f"| {k} | {fc:.1f} | {wc:.1f} | {rb:.0f} | {wb:.0f} | {rb + wb:.0f} | {rd + wr} | "
                         f"{(rb + wb) / (rd + wr):.5f} |")

    # ---- write-request stalls of the L2 towards memory
    spath = os.path.join(src, "stall", "stall_counter_collection.csv")
    if os.path.exists(spath):
        st = counter_sums(spath)
        scalls = bench_line(os.path.join(src, "stall.log"))["api_calls"]
        names = ["TCC_EA0_WRREQ_sum", "TCC_EA0_WRREQ_STALL_sum", "TCC_EA0_WRREQ_DRAM_CREDIT_STALL_sum", "TCC_CYCLE_sum"]
        lines += ["", "## L2 write requests towards memory and their stalls, per call (summed over all L2 channels)", "",
                  "| entry point | " + " | ".join(n[:-4] for n in names) + " | stall cycles per write request | stalled share of L2 cycles |",
                  "|---|" + "---|" * (len(names) + 2)]
        for k in ("se_step", "se_ring_step", "se_calib_copy"):
            if not scalls.get(k) or (k, names[0]) not in st:
                continue
            vals = [st[(k, nm)] / scalls[k] for nm in names]
            lines.append(f"| {k} | " + " | ".join(f"{v:.0f}" for v in vals) +
                         f" | {vals[1] / max(vals[0], 1):.2f} | {vals[1] / max(vals[3], 1):.4f} |")

    with open(stem + ".md", "w") as f:
        f.write("\n".join(lines) + "\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
