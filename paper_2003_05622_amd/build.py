"""Compiles the HIP library (csrc/hps.hip -> libhps.so) for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "hps.hip")
# HPS_LIB: load this already built library instead (the sanitizer run of the host-side tests)
LIB = os.environ.get("HPS_LIB") or os.path.join(_HERE, "libhps.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # keep hipcc from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build(verbose: bool = False) -> str:
    """Always compiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-o", tmp, SRC]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose:
        print(res.stdout)
    os.replace(tmp, LIB)
    return LIB


def ensure_built() -> str:
    """Path of the library; compiles only when no library is there."""
    return LIB if os.path.exists(LIB) else build()


if __name__ == "__main__":
    print(build(verbose=True))
