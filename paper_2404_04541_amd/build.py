"""Build the HIP library in-tree: paper_2404_04541_amd/libspgemm_gfx950.so."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "csrc", "spgemm_api.hip")
LIB = os.path.join(_HERE, "libspgemm_gfx950.so")
LIB_CLOCKS = os.path.join(_HERE, "libspgemm_gfx950_clocks.so")   # the same sources with -DSPG_PHASE_CLOCKS (profiling only)

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-munsafe-fp-atomics",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False, phase_clocks: bool = False) -> str:
    """Compile csrc/ for gfx950 with hipcc (cross-compiles without a GPU).  phase_clocks: the profiling
    variant whose dense kernels read the shader clock at phase boundaries (used by phase_profile.py only)."""
    out_path = LIB_CLOCKS if phase_clocks else LIB
    cmd = ["hipcc", *FLAGS, *(["-DSPG_PHASE_CLOCKS=1"] if phase_clocks else []), "-o", out_path, SRC]
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return out_path


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_library(verbose=True, phase_clocks=True))
