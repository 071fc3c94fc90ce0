"""Host code under AddressSanitizer + UBSan (no GPU): the oracle on exactly-sized buffers,
and the C ABI's host side linked against mock launchers that check every launch's argument
block against what the kernels assume and that layer ranges are tiled exactly once."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1"]


def run(exe):
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the process
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.run(["gcc", "-std=c11", "-ffp-contract=off", *SAN, "-o", exe,
                    os.path.join(HERE, "host", "oracle_san_main.c"), "-lm"], check=True)
    assert "0 failures" in run(exe)


@pytest.mark.skipif(not os.path.exists("/opt/rocm/include/hip/hip_runtime.h"), reason="HIP headers not installed")
def test_api_host_side_against_mock_launchers(tmp_path):
    exe = str(tmp_path / "api_mock")
    cmd = ["g++", "-std=c++17", *SAN, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", "-o", exe,
           os.path.join(HERE, "host", "api_mock_main.cpp"),
           os.path.join(ROOT, "paper_2007_00433_amd", "csrc", "se_api.cpp"),
           "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True)
    out = run(exe)
    assert " 0 failures" in out, out
