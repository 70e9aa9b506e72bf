"""The per-workgroup phase trace (a diagnostic second build of the library) still runs and reports every phase
(needs an MI355X)."""
import os
import re
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_phase_trace_reports_every_phase_of_a_small_launch(gpu_device):
    if not os.path.exists(os.path.join(ROOT, "paper_2003_00532_amd", "libgemm_f64_trace.so")):
        pytest.fail("libgemm_f64_trace.so is not built (run __graft_entry__.build())")
    res = subprocess.run([sys.executable, "-m", "paper_2003_00532_amd.phase_trace", "--workload", "c1_2048"], cwd=ROOT,
                         capture_output=True, text=True, timeout=110)
    assert res.returncode == 0, res.stderr[-2000:]
    out = res.stdout
    assert "1024 workgroups" in out and "variant mfma_64x64x16" in out, out
    phases = {}
    for name in ("entry -> first stage barrier", "K loop", "epilogue (C update)", "whole life"):
        m = re.search(re.escape(name) + r"\s+mean\s+([\d.]+)", out)
        assert m, (name, out)
        phases[name] = float(m.group(1))
    # a 64 x 64 tile of K = 2048 holds 55 us of matrix work; four of them share a compute unit
    assert 50.0 < phases["K loop"] < 400.0 and phases["whole life"] >= phases["K loop"], phases
    m = re.search(r"compute units seen (\d+)", out)
    assert m and int(m.group(1)) == 256, out
    m = re.search(r"shader clock over workgroup lifetimes: mean (\d+) MHz", out)
    assert m and 1500 < int(m.group(1)) < 3000, out
