"""Host-side pieces of bench.py that need no GPU: the refusal of more than one GPU, the traffic figure read from the
tracked profile, the paper's context."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2 and "ONE GPU" in res.stderr and res.stdout.strip() == ""


def test_traffic_comes_from_the_tracked_profile_with_its_build_id():
    for letter, variant in (("d", "mfma_128x128x16"), ("s", "mfma_128x128x32")):
        value, src = bench.traffic_from_profile(letter, variant, "c3_8192", "some-other-build")
        assert value is not None and 2e9 < value < 3e10, "the headline kernel's counter summary must be tracked"
        assert src["file"].startswith("profiles/") and os.path.exists(os.path.join(ROOT, src["file"]))
        assert src["profile_build_id"] and src["same_build"] is False
        same = bench.traffic_from_profile(letter, variant, "c3_8192", src["profile_build_id"])[1]
        assert same["same_build"] is True
    assert bench.traffic_from_profile("d", "no_such_variant", "c3_8192", "x") == (None, None)


def test_paper_context_quotes_the_papers_machine():
    ctx = bench.PAPER_CONTEXT
    assert ctx["peak_gflops_per_core"] == 75.2 and 61 < ctx["best_gflops"] < 62 and "i7-8700K" in ctx["machine"]
    json.dumps(ctx)
    # the fixture with the paper's printed figures pins the GFLOPS convention these numbers are quoted in
    assert os.path.exists(os.path.join(ROOT, "tests", "golden", "paper_gflops_convention.txt"))
