"""The runnable programs of the package keep working: call_all on the smallest workloads."""
import sys

import pytest


@pytest.mark.gpu
@pytest.mark.parametrize("workload", ["tiny", "resnet20"])
def test_call_all_runs(workload, monkeypatch, capsys):
    from paper_2007_00433_amd import call_all
    monkeypatch.setattr(sys, "argv", ["call_all", "--workload", workload, "--reps", "2"])
    call_all.main()
    lines = [l for l in capsys.readouterr().out.splitlines() if "GB/s" in l]
    assert [l.split("  ")[0].strip() for l in lines] == [
        "se_step", "se_ring_step", "se_ring_step, no momentum", "se_global_average", "se_consensus"]
