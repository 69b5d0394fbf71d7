"""Build libmbulyan.so (gfx950) in-tree with hipcc.

    python paper_1905_04374_amd/build.py [-j N] [--force]

(run as a script: importing the package needs the library this makes)

Objects go to paper_1905_04374_amd/_build/, the library next to this file.
The coordinate-pass sources are compiled once per group of theta values
(-DMB_GROUP=g) so the register-resident sorting networks build in parallel.
"""
from __future__ import annotations

import argparse
import os
import re
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmbulyan.so")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")

ARCH = "gfx950"
# packed fp32 VALU instructions are switched off on purpose: some of their forms have given wrong
# results on these machines now and then, with no error
COMMON = ["-std=c++17", "-O3", f"--offload-arch={ARCH}", "-fPIC",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument", f"-I{INCLUDE}"]
# inputs are finite by contract: lets a comparator be one v_min_f32 + one v_max_f32
NO_NANS = ["-fno-honor-nans"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: the HIP library cannot be built")
    return exe


def units():
    """(object name, source, extra flags)"""
    u = [("api.o", "api.hip", []),
         ("dist.o", "dist.hip", []),
         ("dist_gram.o", "dist_gram.hip", []),
         ("select.o", "select.hip", []),
         ("rowops.o", "rowops.hip", []),
         ("host_chunks.o", "host_chunks.hip", [])]
    # the coordinate kernels: per group of theta values, and per storage format of the gradients
    # (fp32, bf16 = -DMB_IN16=1, fp16 = -DMB_IN16=2)
    for g in range(8):
        u.append((f"coordwise_g{g}.o", "coordwise.hip", NO_NANS + [f"-DMB_GROUP={g}"]))
        u.append((f"coordwise16_g{g}.o", "coordwise.hip", NO_NANS + [f"-DMB_GROUP={g}", "-DMB_IN16=1"]))
        u.append((f"coordwiseh_g{g}.o", "coordwise.hip", NO_NANS + [f"-DMB_GROUP={g}", "-DMB_IN16=2"]))
    for g in range(8):
        u.append((f"coordwise_alg1_g{g}.o", "coordwise_alg1.hip", NO_NANS + [f"-DMB_GROUP={g}"]))
        u.append((f"coordwise_alg1_16_g{g}.o", "coordwise_alg1.hip", NO_NANS + [f"-DMB_GROUP={g}", "-DMB_IN16=1"]))
        u.append((f"coordwise_alg1_h_g{g}.o", "coordwise_alg1.hip", NO_NANS + [f"-DMB_GROUP={g}", "-DMB_IN16=2"]))
    return u


def _local_includes(path: str, seen: set) -> set:
    """The headers beside the sources that `path` includes with quotes, directly or through them."""
    with open(path) as fh:
        names = re.findall(r'^\s*#\s*include\s+"([^"]+)"', fh.read(), flags=re.M)
    for name in names:
        dep = os.path.join(CSRC, name)
        if dep not in seen and os.path.exists(dep):
            seen.add(dep)
            _local_includes(dep, seen)
    return seen


def _deps_newer(obj: str, src: str) -> bool:
    """An object depends on its own source, the headers beside it that it includes and this file;
    the C-ABI layer also on the public headers (no other source includes them)."""
    t = os.path.getmtime(obj)
    deps = [os.path.join(CSRC, src), __file__]
    deps += sorted(_local_includes(os.path.join(CSRC, src), set()))
    if src in ("api.hip", "host_chunks.hip"):
        deps += [os.path.join(INCLUDE, name) for name in os.listdir(INCLUDE)]
    return any(os.path.getmtime(dep) > t for dep in deps)


def build(jobs: int = 8, force: bool = True, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    cc = hipcc()

    def compile_one(unit):
        obj, src, extra = unit
        objp = os.path.join(OBJ, obj)
        if not force and os.path.exists(objp) and not _deps_newer(objp, src):
            return objp
        cmd = [cc, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", objp]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src} ({obj}):\n{r.stdout}\n{r.stderr}")
        return objp

    # biggest units first so the pool stays busy: the sorting networks for large theta, and the
    # Algorithm-1 units (two kernels per theta) before the others
    def weight(u):
        name = u[0]
        if name.startswith("coordwise") and name[-4] == "g":
            return -2 * int(name[-3]) - (1 if "alg1" in name else 0)
        return 1
    order = sorted(units(), key=weight)
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        objs = list(pool.map(compile_one, order))
    cmd = [cc, f"--offload-arch={ARCH}", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("-j", type=int, default=min(8, os.cpu_count() or 1))
    ap.add_argument("--force", action="store_true")
    ap.add_argument("-v", action="store_true")
    a = ap.parse_args()
    print(build(a.j, a.force, a.v))
    sys.exit(0)
