"""Plain definitions of the collectives (postconditions).  Test infrastructure.

Section 3.2: a collective's postcondition gives, for each index of each output
buffer, the input chunk or reduction chunk that must end there.
    AllReduce (Section 7.1):  every rank's output chunk j is the reduction of
        chunk j of all ranks.
    AllToAll  (Section 7.3):  chunk i of rank j ends on rank i at index j.
    AllToNext (Section 7.4):  rank i's buffer ends on rank i+1; the last rank
        sends nothing, so rank 0's output is never written.
    ReduceScatter / AllGather (the two halves of an AllReduce, Section 2):  with k
        output (input) chunks per rank, output chunk j of rank r is the reduction of
        chunk r*k + j of all ranks / output chunk q*k + j of every rank is chunk j
        of rank q.
Written as brute-force loops over ranks and chunks, independent of the interpreter.
"""
from __future__ import annotations

from collections import Counter
from typing import List, Optional, Sequence

import numpy as np

from . import numeric


def symbolic_expected(collective: str, ranks: int, in_chunks: int, out_chunks: int) -> List[List[Optional[Counter]]]:
    """expected[r][j]: multiset of (rank, input index) required in output chunk j of
    rank r, or None where the collective leaves the output untouched."""
    exp: List[List[Optional[Counter]]] = []
    for r in range(ranks):
        row: List[Optional[Counter]] = []
        for j in range(out_chunks):
            if collective == "allreduce":
                row.append(Counter({(q, j): 1 for q in range(ranks)}))
            elif collective == "alltoall":
                per = out_chunks // ranks          # chunks exchanged per rank pair
                src, k = j // per, j % per
                row.append(Counter({(src, r * per + k): 1}))
            elif collective == "alltonext":
                row.append(None if r == 0 else Counter({(r - 1, j): 1}))
            elif collective == "reducescatter":
                row.append(Counter({(q, r * out_chunks + j): 1 for q in range(ranks)}))
            elif collective == "allgather":
                row.append(Counter({(j // in_chunks, j % in_chunks): 1}))
            else:
                raise ValueError(f"no postcondition known for {collective}")
        exp.append(row)
    return exp


def check_symbolic(collective: str, ranks: int, in_chunks: int, out_chunks: int, out_bufs) -> None:
    """Raise AssertionError unless the symbolic outputs meet the postcondition."""
    exp = symbolic_expected(collective, ranks, in_chunks, out_chunks)
    for r in range(ranks):
        for j in range(out_chunks):
            got = out_bufs[r][j]
            assert got == exp[r][j], f"rank {r} output chunk {j}: got {got}, postcondition {exp[r][j]}"


def allreduce_sum_f64(inputs: Sequence[np.ndarray], dtype: str) -> np.ndarray:
    """Element-wise sum over ranks, accumulated in float64 rank by rank."""
    acc = np.zeros(inputs[0].size, dtype=np.float64)
    for a in inputs:
        acc += numeric.to_float64(a, dtype)
    return acc


def alltoall_expected(inputs: Sequence[np.ndarray]) -> List[np.ndarray]:
    """out[i] chunk j = in[j] chunk i, for R ranks and R chunks per rank."""
    R = len(inputs)
    ce = inputs[0].size // R
    outs = []
    for i in range(R):
        o = np.empty_like(inputs[0])
        for j in range(R):
            o[j * ce:(j + 1) * ce] = inputs[j][i * ce:(i + 1) * ce]
        outs.append(o)
    return outs


def alltonext_expected(inputs: Sequence[np.ndarray], outputs_before: Sequence[np.ndarray]) -> List[np.ndarray]:
    """out[i+1] = in[i]; out[0] keeps whatever it held before the run."""
    outs = [outputs_before[0].copy()]
    for i in range(1, len(inputs)):
        outs.append(inputs[i - 1].copy())
    return outs


def reducescatter_sum_f64(inputs: Sequence[np.ndarray], dtype: str) -> List[np.ndarray]:
    """out[r] = the r-th of R equal parts of the element-wise sum over ranks (float64)."""
    total = allreduce_sum_f64(inputs, dtype)
    R = len(inputs)
    part = total.size // R
    return [total[r * part:(r + 1) * part].copy() for r in range(R)]


def allgather_expected(inputs: Sequence[np.ndarray]) -> List[np.ndarray]:
    """Every rank's output is the concatenation of all ranks' inputs in rank order."""
    cat = np.concatenate(list(inputs))
    return [cat.copy() for _ in inputs]
