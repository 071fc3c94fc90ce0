"""The C ABI used from plain C (no Python, no torch; the system HIP runtime): the program
tests/host/c_abi_check.c is built by __graft_entry__.build() and run here on the GPU."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(HERE, "host", "c_abi_check.bin")


def test_c_program_is_built():
    assert os.path.exists(EXE), "run __graft_entry__.build() first"


@pytest.mark.gpu
def test_plain_c_caller_matches_the_oracle():
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "0 mismatches" in r.stdout
