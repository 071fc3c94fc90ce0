"""Builds libsesgd.so in-tree with hipcc for gfx950.

    python -m paper_2007_00433_amd.build

Flags that matter for the numerics: no contraction (the two FMAs per element are
explicit), no fast-math, fp32 denormals kept, packed-fp32 instructions disabled (a feature
of the device pass only; see check_device_pass_takes_the_feature).
"""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libsesgd.so")
SOURCES = ["se_api.cpp", "se_plan.hip", "se_step.hip", "se_coop.hip", "se_split.hip", "se_consensus.hip",
           "se_calib.hip"]

HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    "-ffp-contract=off", "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
]


FEATURE_FLAGS = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"

PROBE = """#include <hip/hip_runtime.h>
__global__ void probe(float2 *a, const float2 *b, float s)
{ int i = threadIdx.x; float2 x = a[i], y = b[i]; x.x = x.x * s + y.x; x.y = x.y * s + y.y; a[i] = x; }
"""


def check_device_pass_takes_the_feature(hipcc: str) -> None:
    """hipcc hands -target-feature to the host pass too, which does not know an AMDGPU feature
    and says so for every source (clang's -Xarch_device cannot scope a flag that takes an
    argument).  That note is filtered from the compile output below, so the device pass is
    asked on its own first: it must accept the feature silently, and a kernel that would
    otherwise get a packed fp32 instruction must come out without one."""
    with tempfile.TemporaryDirectory() as tmp:
        src, asm = os.path.join(tmp, "probe.hip"), os.path.join(tmp, "probe.s")
        with open(src, "w") as f:
            f.write(PROBE)
        base = [hipcc, "--offload-arch=gfx950", "-O3", "-ffp-contract=fast", "--cuda-device-only", "-S",
                "-o", asm, src]
        r = subprocess.run(base + FEATURE_FLAGS, capture_output=True, text=True)
        if r.returncode != 0 or "not a recognized feature" in r.stderr:
            raise RuntimeError("the gfx950 device pass rejects -packed-fp32-ops:\n" + r.stderr)
        if "v_pk_" in open(asm).read():
            raise RuntimeError("packed fp32 instructions were emitted despite -packed-fp32-ops")


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    check_device_pass_takes_the_feature(hipcc)

    def compile_one(src: str) -> str:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + HIP_FLAGS + FEATURE_FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        # the host pass's note about the device-only feature (checked above) is dropped; every
        # other diagnostic is shown
        noise = (HOST_PASS_NOTE, "warning generated", "warnings generated")
        rest = [l for l in r.stderr.splitlines() if l.strip() and not any(q in l for q in noise)]
        if rest:
            print("\n".join(rest), file=sys.stderr, flush=True)
        if r.returncode != 0:
            raise subprocess.CalledProcessError(r.returncode, cmd, r.stdout, r.stderr)
        return obj

    # one hipcc per source, side by side (the two big kernel files dominate)
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-q" not in sys.argv))
