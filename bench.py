#!/usr/bin/env python3
"""Benchmark of the SESGD hot path on one MI355X.

A step is one pass of the whole hot path over the packed multi-layer buffer: regrouping,
local SGD/momentum update, group average and write-back for all n workers and all layers,
one `se_step` launch.  Inputs (params, momentum, a small pool of gradient buffers) are
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published peak HBM3E bandwidth


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--grad-pool", type=int, default=4, help="distinct gradient buffers cycled through")
    ap.add_argument("--no-pad", action="store_true", help="use pitch = P instead of se_pitch(P)")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--skip-ring", action="store_true")
    ap.add_argument("--skip-copy", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=3.0, help="target CPU time per oracle leg")
    ap.add_argument("--tune", action="append", default=[], metavar="NAME=VALUE")
    ap.add_argument("--reallocs", type=int, default=8,
                    help="after the headline region: free and re-allocate the buffers this many times "
                         "and time se_step / se_ring_step on each placement (0 = skip)")
    ap.add_argument("--call-all", action="store_true",
                    help="instead of the benchmark: call every device entry point a few times on the "
                         "workload's buffers and print one line per call (a dispatch list for profilers)")
    ap.add_argument("--all-workloads", action="store_true",
                    help="also time se_step / se_ring_step / the oracle on every configured workload "
                         "(reported under 'all_workloads'; the headline fields are unchanged)")
    return ap.parse_args()


def timed_steps(launch, steps, warmup, torch):
    """Runs warmup + steps launches on the current stream; returns (wall seconds for the
    timed steps, mean seconds per launch from stream events)."""
    stream = torch.cuda.current_stream()
    for t in range(warmup):
        launch(t, stream)
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for t in range(warmup, warmup + steps):
        launch(t, stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, ev0.elapsed_time(ev1) * 1e-3 / steps


def per_launch_ms(launch, steps, first_iter, torch):
    """One stream-event pair around every launch (iterations first_iter, first_iter+1, ...);
    returns the sorted launch durations in ms."""
    stream = torch.cuda.current_stream()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
             for _ in range(steps)]
    for t, (e0, e1) in enumerate(pairs):
        e0.record(stream)
        launch(first_iter + t, stream)
        e1.record(stream)
    torch.cuda.synchronize()
    return sorted(e0.elapsed_time(e1) for e0, e1 in pairs)


def cpu_baseline(w, pitch, target_seconds):
    """The oracle as it stands, on a column slice of the same workload, timed on this host:
    once from a single thread, once from one thread per available core on disjoint column
    blocks.  Returns steps/s extrapolated linearly in columns (columns are independent)."""
    import numpy as np
    import oracle
    from paper_2007_00433_amd import workloads as wl

    cores = len(os.sched_getaffinity(0))
    n, m = w.n, w.group_size

    def make(cols):
        x = wl.host_params(n, cols, w.param_std, 0)
        v = np.zeros_like(x)
        g = wl.host_grads(n, cols, w.grad_std, 0, 0, w.grad_dtype)
        return x, v, g

    # calibrate the single-thread rate on a small slice, then size the samples
    probe = int(min(pitch, 1 << 20))                                # beyond the host caches
    x, v, g = make(probe)
    t0 = time.perf_counter()
    oracle.step(x, g, v, m, 0, w.lr, w.mu)
    rate = probe / max(time.perf_counter() - t0, 1e-6)              # columns per second
    cols1 = int(min(pitch, max(1 << 16, rate * target_seconds / 2)))
    x, v, g = make(cols1)
    t0 = time.perf_counter()
    for t in range(2):
        oracle.step(x, g, v, m, t, w.lr, w.mu)
    single = (time.perf_counter() - t0) / 2 * (pitch / cols1)       # seconds per full step
    colsN = int(min(pitch, cols1 * max(1, cores // 2)))
    x, v, g = make(colsN)
    t0 = time.perf_counter()
    for t in range(2):
        oracle.step_threaded(x, g, v, m, t, w.lr, w.mu, threads=cores)
    multi = (time.perf_counter() - t0) / 2 * (pitch / colsN)
    return {
        "value": round(1.0 / multi, 4), "unit": "steps/s", "cores": cores, "kind": "oracle",
        "sample": f"oracle_step on the first {colsN} of {pitch} columns of all {n} rows, 2 steps, "
                  f"{cores} threads on disjoint column blocks; extrapolated linearly in columns",
        "single_thread_value": round(1.0 / single, 4),
        "single_thread_sample": f"first {cols1} columns, 2 steps, 1 thread",
        "gbytes_per_s": round(n * pitch * (16 + w.grad_bytes) / multi / 1e9, 2),
    }


def measure_workload(name, steps, warmup, cpu_seconds, torch, se, wl):
    """steps/s and effective GB/s of se_step and se_ring_step on one workload, plus the oracle."""
    w = wl.WORKLOADS[name]
    n, m, P = w.n, w.group_size, w.P
    pitch = se.se_pitch(P)
    offs = w.layer_offsets(pitch)
    bf16 = w.grad_dtype == "bf16"
    step_fn = se.se_step_bf16g if bf16 else se.se_step
    ring_fn = se.se_ring_step_bf16g if bf16 else se.se_ring_step
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1)
    x = torch.zeros(n, pitch, device="cuda")
    x[:, :P] = torch.randn(P, device="cuda", generator=gen) * w.param_std
    v = torch.zeros(n, pitch, device="cuda")
    pool = []
    for _ in range(2):
        g = torch.zeros(n, pitch, device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)
        for i in range(n):
            g[i, :P] = (torch.randn(P, device="cuda", generator=gen) * w.grad_std).to(g.dtype)
        pool.append(g)
    mu = w.mu if w.mu else 0.9          # the tiny config has mu = 0: time it with a momentum buffer anyway
    nbytes = se.se_step_bytes(P, n, w.grad_bytes, True)
    k = max(steps, 20) if nbytes < 1e9 else max(5, steps // 5) if nbytes > 2e10 else steps
    _, per = timed_steps(lambda t, s: step_fn(x, pool[t % 2], v, offs, n, m, t, w.lr, mu, s), k, warmup, torch)
    _, rper = timed_steps(lambda t, s: ring_fn(x, pool[t % 2], v, offs, n, w.lr, mu, s), k, warmup, torch)
    res = {"n": n, "group_size": m, "params_per_worker": P, "pitch": pitch, "grad_dtype": w.grad_dtype,
           "bytes_per_step": nbytes, "steps_timed": k,
           "se_step": {"steps_per_s": round(1.0 / per, 2), "gbs": round(nbytes / per / 1e9, 1),
                       "frac_of_peak": round(nbytes / per / 1e9 / HBM_PEAK_GBS, 4)},
           "se_ring_step": {"steps_per_s": round(1.0 / rper, 2), "gbs": round(nbytes / rper / 1e9, 1),
                            "frac_of_peak": round(nbytes / rper / 1e9 / HBM_PEAK_GBS, 4)}}
    if nbytes < 1e9:
        # launch-bound shapes: the same loop captured once in a HIP graph (K steps with their
        # iteration numbers baked in) and replayed, which removes the per-launch host cost
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for t in range(k):
                step_fn(x, pool[t % 2], v, offs, n, m, t, w.lr, mu, side)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 20
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        gper = (time.perf_counter() - t0) / (reps * k)
        res["se_step_in_graph"] = {"steps_per_s": round(1.0 / gper, 2), "steps_per_graph": k,
                                   "gbs": round(nbytes / gper / 1e9, 1)}
        del graph
    del x, v, pool
    torch.cuda.empty_cache()
    if cpu_seconds > 0:
        res["cpu_baseline"] = cpu_baseline(w, pitch, cpu_seconds)
    return res


def call_all(w, torch, se, reps=3):
    """Every device entry point on buffers of one shape, so that a profiler run shows their
    counters side by side.  One line per call with its mean time from stream events."""
    n, m, P = w.n, w.group_size, w.P
    pitch = se.se_pitch(P)
    offs = w.layer_offsets(pitch)
    bf16 = w.grad_dtype == "bf16"
    x = torch.randn(n, pitch, device="cuda") * w.param_std
    v = torch.zeros(n, pitch, device="cuda")
    g = (torch.randn(n, pitch, device="cuda") * w.grad_std).to(torch.bfloat16 if bf16 else torch.float32)
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    step = se.se_step_bf16g if bf16 else se.se_step
    ring = se.se_ring_step_bf16g if bf16 else se.se_ring_step
    calls = [
        ("se_step", lambda t: step(x, g, v, offs, n, m, t, w.lr, 0.9), 16 + w.grad_bytes),
        ("se_step, one group", lambda t: step(x, g, v, offs, n, n, t, w.lr, 0.9), 16 + w.grad_bytes),
        ("se_ring_step", lambda t: ring(x, g, v, offs, n, w.lr, 0.9), 16 + w.grad_bytes),
        ("se_ring_step, no momentum", lambda t: ring(x, g, None, offs, n, w.lr, 0.0), 8 + w.grad_bytes),
        ("se_global_average", lambda t: se.se_global_average(x, offs, n), 8),
        ("se_consensus", lambda t: se.se_consensus(x, offs, n, out), 4),
    ]
    stream = torch.cuda.current_stream()
    for name, call, bytes_per_element in calls:
        call(0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for t in range(1, 1 + reps):
            call(t)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        print(f"{name:28s} {ms:9.3f} ms  {n * P * bytes_per_element / ms / 1e6:8.1f} GB/s", flush=True)


def realloc_spread(w, pitch, offs, count, steps, torch, se):
    """The same binary and inputs run at different speeds depending on where the driver places
    the buffers.  Frees and re-allocates params, momentum and one gradient buffer `count` times
    (the caching allocator is emptied in between, so every round is a fresh hipMalloc) and times
    se_step and se_ring_step on each placement."""
    n, m, P = w.n, w.group_size, w.P
    bf16 = w.grad_dtype == "bf16"
    step_fn = se.se_step_bf16g if bf16 else se.se_step
    ring_fn = se.se_ring_step_bf16g if bf16 else se.se_ring_step
    nbytes = se.se_step_bytes(P, n, w.grad_bytes, True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    step_gbs, ring_gbs = [], []
    for _ in range(count):
        torch.cuda.empty_cache()
        x = torch.zeros(n, pitch, device="cuda")
        x[:, :P] = torch.randn(P, device="cuda", generator=gen) * w.param_std
        v = torch.zeros(n, pitch, device="cuda")
        g = torch.zeros(n, pitch, device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)
        for i in range(n):
            g[i, :P] = (torch.randn(P, device="cuda", generator=gen) * w.grad_std).to(g.dtype)
        _, per = timed_steps(lambda t, s: step_fn(x, g, v, offs, n, m, t, w.lr, w.mu, s), steps, 3, torch)
        _, rper = timed_steps(lambda t, s: ring_fn(x, g, v, offs, n, w.lr, w.mu, s), steps, 3, torch)
        step_gbs.append(nbytes / per / 1e9)
        ring_gbs.append(nbytes / rper / 1e9)
        del x, v, g
    torch.cuda.empty_cache()

    def summary(vals):
        vals = sorted(vals)
        return {"min": round(vals[0], 1), "median": round(vals[len(vals) // 2], 1),
                "max": round(vals[-1], 1), "count": len(vals)}
    return summary(step_gbs), summary(ring_gbs)


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (all {args.gpus} requested ranks would "
              "need a second device); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2007_00433_amd import binding as se
    from paper_2007_00433_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    for kv in args.tune:
        name, value = kv.split("=")
        se.se_set_tuning(name, int(value))

    w = wl.WORKLOADS[args.workload]
    if args.call_all:
        call_all(w, torch, se)
        return
    n, m, P = w.n, w.group_size, w.P
    pitch = P if args.no_pad else se.se_pitch(P)
    offs = w.layer_offsets(pitch)
    bf16 = w.grad_dtype == "bf16"
    step_fn = se.se_step_bf16g if bf16 else se.se_step
    ring_fn = se.se_ring_step_bf16g if bf16 else se.se_ring_step

    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    x = torch.zeros(n, pitch, device="cuda")
    x[:, :P] = torch.randn(P, device="cuda", generator=gen) * w.param_std
    v = torch.zeros(n, pitch, device="cuda")
    pool = []
    for _ in range(max(1, args.grad_pool)):
        g = torch.zeros(n, pitch, device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)
        for i in range(n):
            g[i, :P] = (torch.randn(P, device="cuda", generator=gen) * w.grad_std).to(g.dtype)
        pool.append(g)
    torch.cuda.synchronize()

    def launch_step(t, stream):
        step_fn(x, pool[t % len(pool)], v, offs, n, m, t, w.lr, w.mu, stream)

    def launch_ring(t, stream):
        ring_fn(x, pool[t % len(pool)], v, offs, n, w.lr, w.mu, stream)

    wall, per_launch = timed_steps(launch_step, args.steps, args.warmup, torch)
    bytes_per_launch = se.se_step_bytes(P, n, w.grad_bytes, True)
    achieved = bytes_per_launch / per_launch / 1e9
    # spread of single launches, outside the timed region: median and fastest of the same count
    each = per_launch_ms(launch_step, args.steps, args.warmup + args.steps, torch)

    # HBM bytes per launch measured offline with rocprofv3 --pmc: the `se_step` row of the traffic
    # table in profiles/se_step_<workload>_n<n>_m<m>.md (written by profile_summary.py)
    traffic = None
    prof = os.path.join(ROOT, "profiles", f"se_step_{args.workload}_n{n}_m{m}.md")
    traffic_source = None
    if os.path.exists(prof):
        traffic_source = (f"profiles/{os.path.basename(prof)}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                          "this program, scaled by the plain copy kernel; measured in separate, earlier "
                          "processes, not in this run")
        with open(prof) as f:
            text = f.read()
        if f"pitch={pitch})" in text:
            for line in text.splitlines():
                cells = [c.strip() for c in line.split("|")]
                if len(cells) == 10 and cells[1] == "se_step" and cells[6].isdigit():
                    traffic = int(cells[6])

    out = {
        "metric": "SESGD steps/sec and achieved HBM GB/s (% of peak), n=16 ResNet-50-shaped"
                  if args.workload == "resnet50" else f"SESGD steps/sec, {args.workload}",
        "value": round(args.steps / wall, 3),
        "unit": "steps/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if not bf16 else "f32 (bf16 gradient storage)",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}-shaped packed buffer", "n_workers": n,
                   "group_size": m, "tensors": len(w.sizes), "params_per_worker": P,
                   "pitch": pitch, "lr": w.lr, "momentum": w.mu, "grad_dtype": w.grad_dtype,
                   "grad_buffers_cycled": len(pool),
                   "tuning": {k: se.se_get_tuning(k) for k in se.TUNING_KNOBS}},
        "roofline": {"bound": "hbm", "kernel": "se_coop_kernel" if se.se_get_tuning("cooperative") == 1 else "se_step_kernel", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_source": traffic_source if traffic else None,
                     "bytes_per_launch": bytes_per_launch,
                     "avg_launch_ms": round(per_launch * 1e3, 5),
                     "median_launch_ms": round(each[len(each) // 2], 5),
                     "min_launch_ms": round(each[0], 5)},
    }
    # practical ceiling: a plain streaming copy over buffers of the same size
    nb = pool[0].numel() * pool[0].element_size()
    if not args.skip_copy and len(pool) > 1:
        a_buf, b_buf = pool[0].reshape(-1), pool[1].reshape(-1)
        _, cper = timed_steps(lambda t, stream: se.se_calib_copy(b_buf, a_buf, nb, stream),
                              max(10, args.steps // 2), 3, torch)
        out["copy_ceiling"] = {"achieved_gbs": round(2 * nb / cper / 1e9, 1), "bytes_per_launch": 2 * nb,
                               "kernel": "se_calib_copy_kernel"}
    if not args.skip_ring:
        rwall, rper = timed_steps(launch_ring, args.steps, args.warmup, torch)
        out["ring_baseline"] = {"value": round(args.steps / rwall, 3), "unit": "steps/s",
                                "achieved_gbs": round(bytes_per_launch / rper / 1e9, 1),
                                "frac": round(bytes_per_launch / rper / 1e9 / HBM_PEAK_GBS, 4)}
    if not args.skip_copy and len(pool) > 1:
        # one direction only: what the memory system gives to reads and to writes apart from their mix
        a_buf, b_buf = pool[0].reshape(-1), pool[1].reshape(-1)
        _, rper = timed_steps(lambda t, stream: se.se_calib_oneway(b_buf, a_buf, nb, 1, stream), 10, 3, torch)
        _, wper = timed_steps(lambda t, stream: se.se_calib_oneway(b_buf, a_buf, nb, 2, stream), 10, 3, torch)
        out["copy_ceiling"]["read_only_gbs"] = round(nb / rper / 1e9, 1)
        out["copy_ceiling"]["write_only_gbs"] = round(nb / wper / 1e9, 1)
        # torch's own device-to-device copy of the same buffers (on the current stream), for comparison
        _, tper = timed_steps(lambda t, stream: b_buf.copy_(a_buf), 10, 3, torch)
        out["copy_ceiling"]["torch_copy_gbs"] = round(2 * nb / tper / 1e9, 1)
        pool[1].normal_(0, w.grad_std)             # the writer left a pattern behind
    # Context only (other hardware, end-to-end training, not this path's metric): what the
    # paper reports, and its own communication-time model evaluated on this layer list.
    model = {}
    for lat in (1e-4, 5e-3):
        r = se.se_comm_model(w.layer_offsets(), 4, n, n // m, 125e6, lat)
        model[f"latency_{lat * 1e3:g}ms"] = {"ring_s": round(r["ring_seconds"], 4),
                                              "sesgd_s": round(r["sesgd_seconds"], 4),
                                              "ratio": round(r["ring_seconds"] / r["sesgd_seconds"], 3),
                                              "ring_handshakes": r["ring_handshakes"],
                                              "sesgd_handshakes": r["sesgd_handshakes"]}
    out["paper_context"] = {
        "reported": "1.7x end-to-end training speed-up over Ring-SGD (DenseNet121/CIFAR100, 16 workers = "
                    "4 nodes x 4 Tesla K80, 1 Gbps Ethernet, 0.1 ms latency, 4 groups); almost 5x at 5 ms "
                    "latency; cluster measurements, not comparable with a single-GPU step rate",
        "comm_model_1gbps_per_iteration": model,
    }
    # how many times each entry point was called: lets a profiler's per-kernel totals of this
    # run be turned into per-call figures
    out["api_calls"] = {"se_step": args.warmup + 2 * args.steps,
                        "se_ring_step": 0 if args.skip_ring else args.warmup + args.steps,
                        "se_calib_copy": 0 if args.skip_copy or len(pool) < 2 else 3 + max(10, args.steps // 2)}
    released = False
    if args.reallocs > 0:
        del pool, x, v
        released = True
        rsteps = args.steps if bytes_per_launch < 2e10 else max(4, args.steps // 5)
        srl, rrl = realloc_spread(w, pitch, offs, args.reallocs, rsteps, torch, se)
        out["roofline"]["realloc_gbs"] = srl
        out["roofline"]["realloc_frac_min"] = round(srl["min"] / HBM_PEAK_GBS, 4)
        if "ring_baseline" in out:
            out["ring_baseline"]["realloc_gbs"] = rrl
        for key in ("se_step", "se_ring_step"):
            out["api_calls"][key] += args.reallocs * (3 + rsteps)
    if not args.skip_cpu_baseline:
        if not released:
            del pool, x, v
            released = True
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(w, pitch, args.cpu_seconds)
    if args.all_workloads:
        # The paper's schedule sends layer l while backward computes layer l-1 (Sec. 2.1) and pays
        # a fixed latency per layer (Sec. 2.3).  The GPU analogue: one se_step_ex call per tensor,
        # back to front, against the single fused launch timed above.
        L = len(w.sizes)

        def launch_per_layer(t, stream):
            for l in range(L - 1, -1, -1):
                se.se_step_ex(x, pool[t % len(pool)], v, offs, n, m, t, w.lr, w.mu, 0.0, 0,
                              first_layer=l, last_layer=l + 1, grads_are_bf16=bf16, stream=stream)

        if released:                            # x, v, pool were released above
            x = torch.zeros(n, pitch, device="cuda")
            v = torch.zeros(n, pitch, device="cuda")
            pool = [torch.zeros(n, pitch, device="cuda", dtype=torch.bfloat16 if bf16 else torch.float32)]
        lsteps = max(5, args.steps // 5)
        lwall, _ = timed_steps(launch_per_layer, lsteps, 2, torch)

        # the same calls spread round-robin over 4 streams (layers are independent, so their
        # launches may overlap, as the per-parameter hooks of the paper's implementation do)
        sides = [torch.cuda.Stream() for _ in range(4)]
        begin = torch.cuda.Event()
        ends = [torch.cuda.Event() for _ in sides]

        def launch_per_layer_streams(t, stream):
            begin.record(stream)
            for side in sides:
                side.wait_event(begin)
            for l in range(L - 1, -1, -1):
                se.se_step_ex(x, pool[t % len(pool)], v, offs, n, m, t, w.lr, w.mu, 0.0, 0,
                              first_layer=l, last_layer=l + 1, grads_are_bf16=bf16,
                              stream=sides[l % len(sides)])
            for side, end in zip(sides, ends):
                end.record(side)
                stream.wait_event(end)

        swall, _ = timed_steps(launch_per_layer_streams, lsteps, 2, torch)
        # The same 161 calls recorded once into a HIP graph and replayed: what the GPU needs for
        # them without the per-call cost of the host (Python, argument checks, launch).
        side = torch.cuda.Stream()
        launch_per_layer(0, side)
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            launch_per_layer(1, torch.cuda.current_stream())
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(lsteps):
            graph.replay()
        torch.cuda.synchronize()
        gwall = time.perf_counter() - t0
        del graph

        # Buckets, as data-parallel frameworks cut their gradient exchange: consecutive tensors
        # (back to front) are stepped together once they add up to 1 Mi elements or more.
        buckets = se.se_layer_buckets(w.layer_offsets(), 1 << 20)

        def launch_buckets(t, stream):
            for first, last in buckets:
                se.se_step_ex(x, pool[t % len(pool)], v, offs, n, m, t, w.lr, w.mu, 0.0, 0,
                              first_layer=first, last_layer=last, grads_are_bf16=bf16, stream=stream)

        bwall, _ = timed_steps(launch_buckets, lsteps, 2, torch)
        out["per_layer_schedule"] = {"launch_calls_per_step": L,
                                     "steps_per_s": round(lsteps / lwall, 3),
                                     "fused_over_per_layer": round(out["value"] * lwall / lsteps, 3),
                                     "steps_per_s_on_4_streams": round(lsteps / swall, 3),
                                     "steps_per_s_replayed_from_a_graph": round(lsteps / gwall, 3),
                                     "buckets_of_1Mi_elements": len(buckets),
                                     "steps_per_s_in_buckets": round(lsteps / bwall, 3)}
        out["all_workloads"] = {}
        # the paper's own four networks (Sec. 4.1) at its 16 workers in 4 groups: its
        # communication-time model (Sec. 2.2, 3.1) on each layer list, 1 Gbps Ethernet
        out["paper_context"]["comm_model_paper_networks"] = {}
        for name in ("resnet18", "resnet50", "densenet121", "vgg16"):
            pw = wl.WORKLOADS[name]
            r = se.se_comm_model(pw.layer_offsets(), 4, 16, 4, 125e6, 1e-4)
            out["paper_context"]["comm_model_paper_networks"][name] = {
                "tensors": len(pw.sizes), "ring_s": round(r["ring_seconds"], 4), "sesgd_s": round(r["sesgd_seconds"], 4),
                "ring_handshakes": r["ring_handshakes"], "sesgd_handshakes": r["sesgd_handshakes"]}
        for name in ("tiny", "resnet20", "resnet18", "densenet121", "resnet50", "vgg16", "bert_base", "bert_base_full"):
            out["all_workloads"][name] = measure_workload(
                name, args.steps, args.warmup, 0.0 if args.skip_cpu_baseline else 1.0, torch, se, wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
