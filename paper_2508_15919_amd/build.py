"""Builds libhfxattn.so for gfx950 with hipcc, in-tree next to this file."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhfxattn.so")
SOURCES = ["hfx_kernels.hip", "hfx_api.cpp", "hfx_plan.cpp", "hfx_sched.cpp"]
# -fno-honor-nans: no floating-point operation in the kernels is ever fed a NaN (possibly-NaN scores
# are masked through integer selects first), and without it every max carries a canonicalising twin.
# Device code only: the host side validates its floating-point arguments with NaN tests.
# The atomic optimizer is switched off: it rewrites thread 0's ticket fetch into a form that
# waits for the counter's reply on the spot, and the reply is only needed an item later.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Xarch_device", "-fno-honor-nans",
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False, extra_flags=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra_flags, "-o", LIB]
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".cpp") else [path])
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
