"""Compiles the HIP sources under csrc/ into libhbp.so (gfx950) next to this file."""
from __future__ import annotations

import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SOURCES = ["hbp_api.hip", "hbp_build.hip", "hbp_spmv.hip", "hbp_spmv_f64.hip"]
LIB = os.path.join(_HERE, "libhbp.so")

# Packed-fp32 code generation is turned off for all device code.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-fPIC",
         "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(_HERE, "csrc")]


def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed building libhbp.so")


def build_library(verbose: bool = False) -> str:
    """hipcc --offload-arch=gfx950; always recompiles (the translation units in parallel)."""
    with tempfile.TemporaryDirectory(prefix="hbp_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]
        cmds = [["hipcc", *FLAGS, "-c", os.path.join(_HERE, "csrc", s), "-o", o] for s, o in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=len(cmds)) as pool:
            list(pool.map(lambda c: _run(c, verbose), cmds))
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
