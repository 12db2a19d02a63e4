"""Seeded synthetic input buffers (host side).  Holds none of the method's arithmetic.

The paper's workloads are buffer-size sweeps of synthetic data (Section 7,
experimental setup); these generators produce per-rank host arrays with the
value distributions of the benchmark configurations.  Storage convention:
f32 -> numpy float32, f16 -> numpy float16, bf16 -> numpy uint16 bit patterns.
The same arrays feed the GPU runtime (uploaded as raw bytes) and the tests'
CPU checks.
"""
from __future__ import annotations

from typing import List

import numpy as np

STORAGE = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}
ITEMSIZE = {"f32": 4, "f16": 2, "bf16": 2}
SENTINEL16 = 0x7E7E  # 16-bit pattern outputs are pre-filled with (a NaN in fp16 and in bf16)


def _narrow(x32: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return x32
    if dtype == "f16":
        return x32.astype(np.float16)
    if dtype == "bf16":
        import torch
        t = torch.from_numpy(np.ascontiguousarray(x32)).to(torch.bfloat16)
        return t.view(torch.int16).numpy().view(np.uint16).copy()
    raise ValueError(f"unknown dtype {dtype}")


def make_inputs(ranks: int, elems: int, dtype: str, dist: str, seed: int) -> List[np.ndarray]:
    """One array of `elems` values per rank, rank r drawn from PCG64(seed + r).

    dist: 'int8'   integers uniform on {-8..8} (sums of a few ranks stay exact),
          'uniform' U(-1,1), 'normal' N(0,1); drawn in float32 then narrowed to
          `dtype` with round-to-nearest-even."""
    out = []
    for r in range(ranks):
        rng = np.random.Generator(np.random.PCG64(seed + r))
        if dist == "int8":
            x = rng.integers(-8, 9, size=elems).astype(np.float32)
        elif dist == "uniform":
            x = rng.random(elems, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)
        elif dist == "normal":
            x = rng.standard_normal(elems, dtype=np.float32)
        else:
            raise ValueError(f"unknown distribution {dist}")
        out.append(_narrow(x, dtype))
    return out


def sentinel_outputs(ranks: int, elems: int, dtype: str) -> List[np.ndarray]:
    """Output buffers pre-filled with a recognisable byte pattern, so that a
    location the collective must not write can be checked bytewise."""
    st = STORAGE[dtype]
    nbytes = elems * ITEMSIZE[dtype]
    pat = np.full(nbytes // 2, SENTINEL16, dtype=np.uint16)
    return [pat.view(st).copy() for _ in range(ranks)]
