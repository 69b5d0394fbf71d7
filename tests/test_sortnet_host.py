"""The compile-time comparator networks of the coordinate kernels (csrc/sortnet.hpp: Batcher's
merge-exchange for any N), run on the host: zero-one principle for every N up to 64, exhaustive up to
N = 14, and the packed 16-bit and 64-bit comparators against std::sort.  Needs hipcc, no GPU."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def test_every_network_sorts(tmp_path):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("no hipcc")
    exe = tmp_path / "sortnet_host"
    build = subprocess.run([hipcc, "-std=c++17", "-O1", "--offload-arch=gfx950", "-Wno-unused-command-line-argument",
                            os.path.join(HERE, "sortnet_host_main.hip"), "-o", str(exe)],
                           capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-2000:]
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=600)
    assert run.returncode == 0, run.stdout[-2000:] + run.stderr[-2000:]
    assert "0 of 64 networks fail" in run.stdout
