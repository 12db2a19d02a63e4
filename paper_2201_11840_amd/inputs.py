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


# Floating-point formats as (bits, exponent bits, stored significand bits).
FORMAT = {"f32": (32, 8, 23), "f16": (16, 5, 10), "bf16": (16, 8, 7)}
SPECIAL_CLASSES = ("random_bits", "tiny", "huge", "zeros", "ties", "inf_nan")


def special_classes(elems: int, seed: int) -> np.ndarray:
    """Class index (into SPECIAL_CLASSES) of every element position of make_special(.., seed)."""
    return np.random.Generator(np.random.PCG64(seed)).integers(0, len(SPECIAL_CLASSES), size=elems)


def make_special(ranks: int, elems: int, dtype: str, seed: int) -> List[np.ndarray]:
    """Per-rank arrays of bit patterns chosen so that element-wise sums over ranks meet the corner cases of
    floating-point addition.  Every element position belongs to one class (the same on all ranks, from
    PCG64(seed)); rank r then draws its own pattern within the class from PCG64(seed + 1 + r):

      random_bits  any bit pattern at all (infinities and NaNs included)
      tiny         exponent field 0..2: subnormal operands, sums that land subnormal or cross into the normal range
      huge         the two largest finite exponents: overflow to +-inf, or cancellation
      zeros        +0 / -0 (and now and then a tiny value): signed-zero rules
      ties         rank 0 holds a mid-range value with a random significand, every other rank an odd multiple
                   (1..15, either sign) of HALF a unit in the last place of it: exact sums fall half-way between
                   two representable values, where only round-to-nearest-even gives the right answer
      inf_nan      +-inf, quiet and signalling NaNs with random payloads, mixed with finite values

    Returned in the storage convention of make_inputs (f32 / f16 as numpy floats, bf16 as uint16 patterns)."""
    bits, ebits, mbits = FORMAT[dtype]
    utype = np.uint32 if bits == 32 else np.uint16
    cls = special_classes(elems, seed)
    shared = np.random.Generator(np.random.PCG64(seed + 7919))
    emax = (1 << ebits) - 1                               # exponent field of inf / NaN
    tie_exp = shared.integers(mbits + 6, emax - 6, size=elems)    # exponent field of the ties' anchor, well inside
    out = []
    for r in range(ranks):
        rng = np.random.Generator(np.random.PCG64(seed + 1 + r))
        sign = rng.integers(0, 2, size=elems).astype(np.uint64)
        mant = rng.integers(0, 1 << mbits, size=elems).astype(np.uint64)

        def pack(exp_field, mant_field):
            return ((sign << np.uint64(bits - 1)) | (exp_field.astype(np.uint64) << np.uint64(mbits)) | mant_field)

        pat = rng.integers(0, 1 << bits, size=elems, dtype=np.uint64)                       # random_bits
        pat = np.where(cls == 1, pack(rng.integers(0, 3, size=elems), mant), pat)          # tiny
        pat = np.where(cls == 2, pack(rng.integers(emax - 2, emax, size=elems), mant), pat)  # huge, finite
        zero_or_tiny = np.where(rng.integers(0, 8, size=elems) == 0, mant & np.uint64(3), np.uint64(0))
        pat = np.where(cls == 3, pack(np.zeros(elems, np.int64), zero_or_tiny), pat)       # zeros
        if r == 0:
            tie = pack(tie_exp, mant)
        else:
            # (2j+1) * 2^(E - bias - mbits - 1): the odd number's leading bit becomes the hidden one
            odd = 2 * rng.integers(0, 8, size=elems) + 1                                    # 1, 3, .., 15
            lead = np.floor(np.log2(odd)).astype(np.int64)                                  # 0..3
            frac = ((odd - (1 << lead)).astype(np.uint64) << (np.uint64(mbits) - lead.astype(np.uint64)))
            tie = pack(tie_exp - (mbits + 1) + lead, frac)
        pat = np.where(cls == 4, tie, pat)
        kind = rng.integers(0, 4, size=elems)
        nan_payload = np.maximum(mant, np.uint64(1))
        infnan = np.where(kind == 0, pack(np.full(elems, emax), np.zeros(elems, np.uint64)),        # +-inf
                 np.where(kind == 1, pack(np.full(elems, emax), nan_payload),                        # any NaN
                 np.where(kind == 2, pack(np.full(elems, emax), nan_payload | np.uint64(1 << (mbits - 1))),  # quiet NaN
                          pack(rng.integers(1, emax, size=elems), mant))))                           # finite
        pat = np.where(cls == 5, infnan, pat)
        arr = pat.astype(utype)
        out.append(arr.view(np.float32) if dtype == "f32" else arr.view(np.float16) if dtype == "f16" else arr)
    return out


def make_inputs(ranks: int, elems: int, dtype: str, dist: str, seed: int) -> List[np.ndarray]:
    """One array of `elems` values per rank, rank r drawn from PCG64(seed + r).

    dist: 'int8'   integers uniform on {-8..8} (sums of a few ranks stay exact),
          'uniform' U(-1,1), 'normal' N(0,1); drawn in float32 then narrowed to
          `dtype` with round-to-nearest-even;
          'special' the corner cases of floating-point addition (make_special)."""
    if dist == "special":
        return make_special(ranks, elems, dtype, seed)
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
