"""Compiles the HIP sources under csrc/ into libhbp.so (gfx950) next to this file."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SOURCES = ["hbp_api.hip", "hbp_build.hip", "hbp_spmv.hip"]
LIB = os.path.join(_HERE, "libhbp.so")


def build_library(verbose: bool = False) -> str:
    """hipcc --offload-arch=gfx950; always recompiles.  Packed-fp32 code generation is turned
    off for all device code."""
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-munsafe-fp-atomics",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-fPIC", "-shared", "-I" + os.path.join(ROOT, "include")]
    cmd += [os.path.join(_HERE, "csrc", s) for s in SOURCES]
    cmd += ["-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libhbp.so")
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
