"""Calls every device entry point of the library a few times on one synthetic workload.

A program to put under a profiler (``rocprofv3 ... -- python3 -m paper_2007_00433_amd.call_all
--workload vgg16``): it makes one dispatch list that contains every kernel of the library on
buffers of the same shape, so that their counters can be read side by side.  Prints one line
per call with its mean time from stream events.
"""
import argparse

import torch

from . import binding as se
from . import workloads as wl


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="resnet50", choices=sorted(wl.WORKLOADS))
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()

    w = wl.WORKLOADS[args.workload]
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
        for t in range(1, 1 + args.reps):
            call(t)
        e1.record(stream)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.reps
        print(f"{name:28s} {ms:9.3f} ms  {n * P * bytes_per_element / ms / 1e6:8.1f} GB/s", flush=True)


if __name__ == "__main__":
    main()
