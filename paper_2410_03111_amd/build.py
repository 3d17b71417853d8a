"""Builds liblorc.so (host code + gfx950 kernels) in-tree with hipcc.  No torch involved."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "liblorc.so")

COMMON = ["-O3", "-std=c++17", "-fPIC", "-pthread", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
HIP_FLAGS = [
    "--offload-arch=gfx950",
    # packed-fp32 forms are switched off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]
NOISE = ("packed-fp32-ops", "is not a recognized feature")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if not any(n in l for n in NOISE))
    if r.returncode != 0:
        raise RuntimeError(f"{cmd[0]} failed ({r.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    cxx = shutil.which("g++") or "g++"
    os.makedirs(OBJ, exist_ok=True)
    jobs = []
    for s in sources():
        o = os.path.join(OBJ, os.path.basename(s) + ".o")
        if s.endswith(".hip"):
            jobs.append(([hipcc, *COMMON, *HIP_FLAGS, "-c", s, "-o", o], o))
        else:  # plain host C++: hipcc would treat it as device code
            jobs.append(([cxx, *COMMON, "-c", s, "-o", o], o))
    with ThreadPoolExecutor(max_workers=min(8, len(jobs))) as ex:
        list(ex.map(lambda j: _run(j[0], verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", *[o for _, o in jobs], "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
