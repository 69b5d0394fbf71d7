"""The C oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU).

The oracle is what every parity claim rests on, so an out-of-bounds read in it would be a silent
error in the reference.  tests/oracle_sanitizer_main.c drives every entry point over small shapes that
reach the loop bounds; the build uses the oracle's own flags plus the sanitizers, and any finding
aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_runs_clean_under_asan_and_ubsan(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-Wall", "-Wextra", "-o", exe,
           os.path.join(ROOT, "oracle", "mbulyan_oracle.c"), os.path.join(ROOT, "tests", "oracle_sanitizer_main.c"), "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0:verify_asan_link_order=0"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "oracle sanitizer run: ok" in r.stdout
