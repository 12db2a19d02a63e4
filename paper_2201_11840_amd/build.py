"""Build the C-ABI library (libgc3.so) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import json
import os
import re
import subprocess
from typing import Dict, List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libgc3.so")
SOURCES = ["program.cpp", "plan.cpp", "residency.cpp", "comm.cpp", "interp_kernel.hip"]


def build(verbose: bool = False, defines: Sequence[str] = (), out: Optional[str] = None) -> str:
    """Compile every source for gfx950 and link libgc3.so; returns its path.
    `defines` (e.g. ["GC3_FENCE_MODE=0"]) and `out` build a tuning variant elsewhere."""
    os.makedirs(LIB_DIR, exist_ok=True)
    out = out or LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument", "-Rpass-analysis=kernel-resource-usage",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", out] + [f"-D{d}" for d in defines] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    usage = kernel_resource_usage(res.stderr)
    with open(os.path.splitext(out)[0] + ".resources.json", "w") as f:
        json.dump(usage, f, indent=1)
    other = "\n".join(l for l in res.stderr.splitlines()
                      if "-Rpass-analysis" not in l and "remark:" not in l and "packed-fp32-ops" not in l   # host pass: harmless
                      and not re.match(r"\s+\d*\s*\|", l))
    if verbose:
        if other.strip():
            print(other)
        for k in usage:
            print(f"  {k['name']}: {k['vgprs']} VGPRs, {k['sgprs']} SGPRs, scratch {k['scratch_bytes']} B/lane, "
                  f"LDS {k['lds_bytes']} B, occupancy {k['occupancy']} waves/SIMD")
    return out


EXAMPLE_SRC = os.path.join(HERE, "examples", "allreduce_c_abi.cpp")
EXAMPLE_BIN = os.path.join(LIB_DIR, "allreduce_c_abi")


def build_example(verbose: bool = False) -> str:
    """Compile the stand-alone C++ example against the header and link it with the built library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Wall", "-Wno-unused-command-line-argument",
           "-I", os.path.join(ROOT, "include"), EXAMPLE_SRC, "-L", LIB_DIR, "-lgc3", "-Wl,-rpath,$ORIGIN", "-o", EXAMPLE_BIN]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on the example:\n" + res.stdout + res.stderr)
    return EXAMPLE_BIN


def kernel_resource_usage(remarks: str) -> List[Dict]:
    """The compiler's per-kernel resource report (register counts, scratch, LDS, occupancy) from its
    -Rpass-analysis=kernel-resource-usage remarks."""
    out: List[Dict] = []
    fields = {"VGPRs": "vgprs", "TotalSGPRs": "sgprs", "ScratchSize [bytes/lane]": "scratch_bytes",
              "LDS Size [bytes/block]": "lds_bytes", "Occupancy [waves/SIMD]": "occupancy"}
    for line in remarks.splitlines():
        m = re.search(r"remark: [^:]*:\d+:\d+:\s+(.*?): (\S+) \[-Rpass-analysis", line) or \
            re.search(r"remark:\s+(?:\S+:\d+:\d+:\s+)?(.*?): (\S+) \[-Rpass-analysis", line)
        if not m:
            continue
        key, val = m.group(1).strip(), m.group(2)
        if key in ("Function Name", "Name"):
            out.append({"name": val})
        elif key in fields and out:
            out[-1][fields[key]] = int(val)
    return [k for k in out if "vgprs" in k]


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_example(verbose=True))
