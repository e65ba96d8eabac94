"""Build libtide_route.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libtide_route.so")
INCLUDE = os.path.join(os.path.dirname(_HERE), "include")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
    # hipcc must not form packed-fp32 instructions from ordinary float code on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def build_library(verbose: bool = False, *, out: str = LIB_PATH, defines: tuple = ()) -> str:
    """Compile every HIP source into libtide_route.so; always recompiles.  `out` / `defines` make an
    instrumented build beside it (timeline.py)."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        raise RuntimeError("hipcc not found: libtide_route cannot be built on this machine")
    tmp = out + ".tmp"
    cmd = [hipcc, *HIPCC_FLAGS, *[f"-D{d}" for d in defines], "-I", INCLUDE, "-o", tmp, os.path.join(CSRC, "tide_route.hip")]
    run = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or run.returncode:
        print(run.stdout + run.stderr)
    if run.returncode:
        raise RuntimeError(f"hipcc failed ({run.returncode}): {' '.join(cmd)}")
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
