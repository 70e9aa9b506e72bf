"""The CPU oracles under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU): buffers end exactly
at the last logical element, so touching padding after the last row or anything past the end is reported."""
import os
import subprocess

from oracle import build as oracle_build

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracles_are_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_sanitize")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-omit-frame-pointer",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
           *oracle_build.SOURCES, os.path.join(HERE, "oracle_sanitize_driver.c"), "-o", exe, "-lm"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-3000:]
    env = dict(os.environ)
    # the sanitizer runtime is linked statically, so whatever else the environment preloads does not matter
    env.update(ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="3")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, (run.stdout[-1000:], run.stderr[-3000:])
    assert "oracle sanitizer run ok" in run.stdout
