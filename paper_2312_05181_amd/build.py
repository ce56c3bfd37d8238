"""Builds libtpx.so (host planner + C ABI + gfx950 kernels) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtpx.so")
SELFTEST_SRC = os.path.join(HERE, "examples", "reshard_selftest.cpp")
SELFTEST = os.path.join(HERE, "tpx_selftest")
HOST_SOURCES = ["layout.cpp", "planner.cpp", "dataset.cpp", "api.cpp"]
HIP_SOURCES = ["kernels.hip"]
# the host pass does not know the device-only feature flag and says so once per file: harmless noise
NOISE = "'-packed-fp32-ops' is not a recognized feature"


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if err:
        print(err, file=sys.stderr, flush=True)
    if res.returncode:
        raise RuntimeError(f"{cmd[0]} failed with status {res.returncode}")


def build(verbose: bool = True) -> str:
    """Compile every source (host files as C++, kernels for gfx950) and link the shared library."""
    os.makedirs(OBJ, exist_ok=True)
    common = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    jobs = []
    for s in HOST_SOURCES:
        jobs.append([hipcc(), "-x", "c++", "-c", *common, os.path.join(CSRC, s), "-o", os.path.join(OBJ, s + ".o")])
    for s in HIP_SOURCES:
        jobs.append([hipcc(), "-c", *common, "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
                     "-packed-fp32-ops", os.path.join(CSRC, s), "-o", os.path.join(OBJ, s + ".o")])
    with ThreadPoolExecutor(len(jobs)) as ex:
        list(ex.map(lambda c: _run(c, verbose), jobs))
    objs = [os.path.join(OBJ, s + ".o") for s in HOST_SOURCES + HIP_SOURCES]
    _run([hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs], verbose)
    # a stand-alone user of the C ABI (host code only; finds libtpx.so next to itself)
    _run([hipcc(), "-O2", "-std=c++17", "-I", os.path.join(ROOT, "include"), SELFTEST_SRC, "-L", HERE, "-ltpx",
          "-Wl,-rpath,$ORIGIN", "-o", SELFTEST], verbose)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)
