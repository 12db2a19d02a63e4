"""The synthetic benchmark configurations: program + dtype + size + input recipe.

Each entry stands in for one of the paper's buffer-size-sweep experiments
(Section 7): Ring AllReduce on one node, direct AllToAll, Hierarchical
AllReduce on 2 nodes x 8 GPUs, AllToNext on 3 nodes x 8 GPUs.  Ranks are
virtual ranks on one GPU.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List

from . import programs
from .inputs import ITEMSIZE
from .ir import Program

MiB = 1 << 20


@dataclass
class Workload:
    name: str
    build: Callable[[], Program]
    dtype: str
    bytes_per_rank: int      # size of the input buffer of one rank
    dist: str
    seed: int

    @property
    def elems_per_rank(self) -> int:
        return self.bytes_per_rank // ITEMSIZE[self.dtype]


def ring_ar_r4() -> Workload:
    return Workload("ring_allreduce_r4_f32_64KiB", lambda: programs.ring_allreduce(4),
                    "f32", 16384 * 4, "int8", 11840)


def direct_a2a_r8() -> Workload:
    return Workload("direct_alltoall_r8_f16_1MiB", lambda: programs.direct_alltoall(8),
                    "f16", 1 * MiB, "normal", 21840)


def ring_ar_r8x8(mib: int) -> Workload:
    return Workload(f"ring_allreduce_r8_x8_f32_{mib}MiB", lambda: programs.ring_allreduce(8, instances=8),
                    "f32", mib * MiB, "uniform", 31840)


def hier_ar_2x8(mib: int = 64) -> Workload:
    return Workload(f"hier_allreduce_2x8_bf16_{mib}MiB", lambda: programs.hierarchical_allreduce(2, 8),
                    "bf16", mib * MiB, "normal", 41840)


def alltonext_3x8(mib: int = 32) -> Workload:
    return Workload(f"alltonext_3x8_f16_{mib}MiB", lambda: programs.alltonext(3, 8),
                    "f16", mib * MiB, "normal", 51840)


def all_workloads() -> List[Workload]:
    return [ring_ar_r4(), direct_a2a_r8(),
            ring_ar_r8x8(1), ring_ar_r8x8(16), ring_ar_r8x8(64), ring_ar_r8x8(256),
            hier_ar_2x8(), alltonext_3x8()]


def next_row_workloads() -> List[Workload]:
    """Programs beyond the five benchmark configurations: the rrs fusion (Section 4.2), All Pairs
    AllReduce (Section 7.1.2), one logical ring spread over several channels in the paper's
    32 KB - 3 MB regime (Section 7.1.1), Two-Step AllToAll (Section 7.3), and the ring ReduceScatter /
    AllGather helpers of Section 2 as collectives of their own (64 MiB per rank on the wide side)."""
    return [
        Workload("ring_allreduce_rrs_r8_x8_f32_64MiB", lambda: programs.ring_allreduce(8, instances=8, use_rrs=True),
                 "f32", 64 * MiB, "uniform", 61840),
        Workload("allpairs_allreduce_r8_f32_64MiB", lambda: programs.allpairs_allreduce(8), "f32", 64 * MiB, "uniform", 62840),
        Workload("allpairs_allreduce_r8_f32_256KiB", lambda: programs.allpairs_allreduce(8), "f32", MiB // 4, "uniform", 62841),
        Workload("mc_ring_allreduce_r8_c4_f32_256KiB", lambda: programs.multichannel_ring_allreduce(8, 4),
                 "f32", MiB // 4, "uniform", 63840),
        Workload("ring_allreduce_r8_f32_256KiB", lambda: programs.ring_allreduce(8), "f32", MiB // 4, "uniform", 63841),
        Workload("mc_ring_allreduce_r8_c4_f32_2MiB", lambda: programs.multichannel_ring_allreduce(8, 4),
                 "f32", 2 * MiB, "uniform", 63842),
        Workload("ring_allreduce_r8_f32_2MiB", lambda: programs.ring_allreduce(8), "f32", 2 * MiB, "uniform", 63843),
        Workload("twostep_alltoall_3x8_f16_48MiB", lambda: programs.twostep_alltoall(3, 8), "f16", 48 * MiB, "normal", 64840),
        Workload("ring_reducescatter_r8_x8_f32_64MiB", lambda: programs.ring_reduce_scatter(8, instances=8),
                 "f32", 64 * MiB, "uniform", 65840),
        Workload("ring_allgather_r8_x8_f32_8MiB", lambda: programs.ring_allgather(8, instances=8),
                 "f32", 8 * MiB, "uniform", 66840),
    ]


def dram_workloads() -> List[Workload]:
    """The local `copy` and `reduce` instructions on their own (no connection, no FIFO) over 2 - 4 GiB of buffers,
    8 to 16 times the 256 MiB memory-side cache: what device memory sustains for the interpreter's tile moves."""
    return [
        Workload("local_copy_r8_f32_256MiB", lambda: programs.local_stream(8, 8), "f32", 256 * MiB, "uniform", 67840),
        Workload("local_reduce_r8_f32_256MiB", lambda: programs.local_stream(8, 8, reduce=True), "f32", 256 * MiB,
                 "uniform", 67841),
    ]


def by_name() -> Dict[str, Workload]:
    return {w.name: w for w in all_workloads() + next_row_workloads() + dram_workloads()}
