"""Build the C-ABI library (libgc3.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libgc3.so")
SOURCES = ["program.cpp", "plan.cpp", "comm.cpp", "interp_kernel.hip"]


def build(verbose: bool = False, defines: Sequence[str] = (), out: Optional[str] = None) -> str:
    """Compile every source for gfx950 and link libgc3.so; returns its path.
    `defines` (e.g. ["GC3_FENCE_MODE=0"]) and `out` build a tuning variant elsewhere."""
    os.makedirs(LIB_DIR, exist_ok=True)
    out = out or LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", out] + [f"-D{d}" for d in defines] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose and res.stderr:
        print(res.stderr)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
