"""Compile the HIP sources of the rTop-k library into ``librtopk.so`` (gfx950)."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "librtopk.so")
# the same sources with RTOPK_DEBUG_CHECKS: the master entry points verify their
# preconditions (index range, ascending slices) on the device before they launch
DEBUG_LIB_PATH = os.path.join(HERE, "librtopk_debug.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950",
    # packed-fp32 instruction selection is kept off for every device function
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC", "-shared",
]


def sources() -> list:
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, debug: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out_path = DEBUG_LIB_PATH if debug else LIB_PATH
    cmd = [hipcc] + HIPCC_FLAGS + (["-DRTOPK_DEBUG_CHECKS"] if debug else []) + ["-o", out_path] + sources()
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass warns that it does not know the device-only target feature
    noise = ("packed-fp32-ops", "is not a recognized feature")
    out = "\n".join(l for l in res.stdout.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, flush=True)
    return out_path


if __name__ == "__main__":
    print(build(verbose="-q" not in sys.argv, debug="--debug" in sys.argv))
