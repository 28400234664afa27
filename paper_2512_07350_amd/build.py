"""Build the C-ABI library (``liblp_mi355x.so``) from ``csrc/`` with hipcc for gfx950.

Run as ``python -m paper_2512_07350_amd.build``.  The shared object is written
next to this file so that it travels with the source tree; nothing is installed.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "liblp_mi355x.so")

SOURCES = ["lp_plan.cpp", "lp_latent.hip", "lp_attention.hip", "lp_block.hip"]

# Packed-FP32 instructions are kept off for every device translation unit.
HOST = ["-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC, "-Wall", "-Wno-unused-function"]
DEVICE = HOST + ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# The reconstruction's binary32 operation order is part of its contract: no contraction there.
PER_FILE = {"lp_latent.hip": ["-ffp-contract=off"]}


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Always rebuilds."""
    hipcc = _hipcc()
    objs = []
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(obj_dir, src + ".o")
        flags = DEVICE if src.endswith(".hip") else HOST
        cmd = [hipcc, *flags, *PER_FILE.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj]
        _run(cmd, verbose)
        objs.append(obj)
    tmp = LIB + ".tmp.%d" % os.getpid()
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs], verbose)
    os.replace(tmp, LIB)
    return LIB


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature and says so; that line is noise
    out = "\n".join(l for l in res.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if res.returncode != 0:
        raise RuntimeError("build step failed: %s\n%s" % (" ".join(cmd), out))
    if verbose and out.strip():
        print(out, flush=True)


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
