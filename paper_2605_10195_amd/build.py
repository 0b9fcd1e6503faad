"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""

from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libspex_tree.so")
SOURCES = ["api.cpp", "page_table.cpp", "planner.cpp", "sched.cpp", "kernels.hip"]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build_library(verbose: bool = False) -> str:
    """Always recompiles; returns the path of the shared library."""
    common = [hipcc(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Wall", "-Wno-unused-function", "-x", "hip"]
    # The kernels are compiled on their own with -fno-honor-nans: masking is done by selects on
    # integer compares and never by NaN tests, and without the flag every fmaxf on an MFMA result
    # costs an extra instruction that quiets a NaN which cannot occur.  Host code keeps NaN
    # semantics (argument checks rely on them).
    kernels_obj = os.path.join(HERE, "kernels.o")
    _run(common + ["-fno-honor-nans", "-c", os.path.join(CSRC, "kernels.hip"), "-o", kernels_obj], verbose)
    host = [os.path.join(CSRC, s) for s in SOURCES if s != "kernels.hip"]
    _run(common + ["-shared"] + host + ["-x", "none", kernels_obj, "-o", LIB_PATH], verbose)
    os.remove(kernels_obj)
    return LIB_PATH


PROBE_PATH = os.path.join(HERE, "hbm_probe")


def build_probe(verbose: bool = False) -> str:
    """Compile the stand-alone HBM bandwidth probe (measurement aid, not part of the library)."""
    cmd = [hipcc(), "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", os.path.join(CSRC, "hbm_probe.hip"), "-o", PROBE_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    return PROBE_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probe(verbose=True))
