"""Element-wise reduction of the oracle: the sum, in the buffer's own data type.

The paper's reduction is element-wise and addition is the one operator it names (Section 3.1);
`reduce`, `rrc`, `rrcs` and `rrs` apply it (Section 4.2).  It names no precision;
the reading taken here is one correctly rounded add per hop in the buffer's
type: IEEE binary32 add for f32; for the 16-bit types both operands are widened
to binary32 (exact), added there, and rounded to nearest-even back to 16 bits,
subnormals kept.  binary32 has 24 >= 2p+2 significand bits for p = 11 (fp16)
and p = 8 (bf16), so the double rounding equals a single correctly rounded
16-bit add.

Storage: f32 -> numpy float32, f16 -> numpy float16, bf16 -> numpy uint16
holding the upper 16 bits of the binary32 pattern.
"""
from __future__ import annotations

import numpy as np

DTYPES = ("f32", "f16", "bf16")
STORAGE = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}
ITEMSIZE = {"f32": 4, "f16": 2, "bf16": 2}


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32: exact, the pattern is the upper half."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 bit patterns, to nearest with ties to even.

    Adding 0x7FFF plus the lowest kept bit to the binary32 pattern and dropping
    the low 16 bits rounds the magnitude to nearest-even; a carry out of the
    significand correctly bumps the exponent (up to infinity).  NaNs are mapped
    to a quiet NaN of the same sign so the carry cannot turn them into inf."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)
    isnan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    qnan = ((u >> np.uint32(16)) | np.uint32(0x0040)).astype(np.uint16)
    return np.where(isnan, qnan, rounded)


def add(a: np.ndarray, b: np.ndarray, dtype: str) -> np.ndarray:
    """One hop of the reduction: element-wise a + b in `dtype`."""
    if dtype == "f32":
        return np.add(a, b, dtype=np.float32)
    if dtype == "f16":
        wide = a.astype(np.float32) + b.astype(np.float32)
        with np.errstate(over="ignore"):
            return wide.astype(np.float16)  # numpy rounds to nearest-even, keeps subnormals
    if dtype == "bf16":
        with np.errstate(over="ignore", invalid="ignore"):
            return f32_to_bf16_bits(bf16_bits_to_f32(a) + bf16_bits_to_f32(b))
    raise ValueError(f"unknown dtype {dtype}")


def to_float64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of stored values to float64 (for comparisons)."""
    if dtype == "bf16":
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)
