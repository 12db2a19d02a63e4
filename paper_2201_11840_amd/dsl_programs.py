"""The paper's collective algorithms written in the DSL (Sections 2, 5.1 and 7), compiled by compiler.py.

The paper's own listings are not reproduced; these are restatements of the prose.
"""
from __future__ import annotations

from typing import List, Optional

from .compiler import compile_program
from .dsl import GC3Program, chunk, parallelize
from .ir import Program


def reduce_scatter(ranks: List[int], offset: int, count: int, ch: Optional[int] = None, buf: str = "input") -> None:
    """Ring ReduceScatter (Section 2): the group of `count` chunks with number q starts on ring position
    q+1, is reduced into every following position and ends on position q."""
    G = len(ranks)
    for q in range(G):
        idx = offset + q * count
        c = chunk(ranks[(q + 1) % G], buf, idx, count)
        for hop in range(2, G + 1):
            c = chunk(ranks[(q + hop) % G], buf, idx, count).reduce(c, ch=ch)


def all_gather(ranks: List[int], offset: int, count: int, ch: Optional[int] = None, buf: str = "input") -> None:
    """Ring AllGather (Section 2): the group owned by position q is copied q -> q+1 -> ... for G-1 hops."""
    G = len(ranks)
    for q in range(G):
        idx = offset + q * count
        c = chunk(ranks[q], buf, idx, count)
        for hop in range(1, G):
            c = c.copy(ranks[(q + hop) % G], buf, idx, ch=ch)


def ring_allreduce(R: int, instances: int = 1, **opts) -> Program:
    """Section 7.1.1: ReduceScatter then AllGather over all ranks, offset 0, count 1; `instances` wraps
    the whole program in parallelize()."""
    with GC3Program(f"dsl_ring_allreduce_r{R}_x{instances}", "allreduce", R, R, inplace=True) as p:
        with parallelize(instances):
            reduce_scatter(list(range(R)), 0, 1)
            all_gather(list(range(R)), 0, 1)
    return compile_program(p, **opts)


def ring_reduce_scatter(R: int, instances: int = 1, **opts) -> Program:
    """Section 2's ReduceScatter helper as a collective: ring reduction inside the input buffer (which is
    overwritten), then the owned chunk is copied to the output."""
    with GC3Program(f"dsl_ring_reducescatter_r{R}_x{instances}", "reducescatter", R, R, 1) as p:
        with parallelize(instances):
            reduce_scatter(list(range(R)), 0, 1)
            for r in range(R):
                chunk(r, "input", r).copy(r, "output", 0)
    return compile_program(p, **opts)


def ring_allgather(R: int, instances: int = 1, **opts) -> Program:
    """Section 2's AllGather helper as a collective: every rank's chunk goes once round the ring."""
    with GC3Program(f"dsl_ring_allgather_r{R}_x{instances}", "allgather", R, 1, R) as p:
        with parallelize(instances):
            for q in range(R):
                c = chunk(q, "input", 0).copy(q, "output", q)
                for hop in range(1, R):
                    c = c.copy((q + hop) % R, "output", q)
    return compile_program(p, **opts)


def hierarchical_allreduce(N: int, G: int, intra_parallel: bool = True, **opts) -> Program:
    """Sections 2 and 5.1: intra-group ReduceScatter on channel 0 (parallelized by N), cross-group
    ReduceScatter and AllGather on channel 1, intra-group AllGather on channel 2 (parallelized by N)."""
    with GC3Program(f"dsl_hier_allreduce_{N}x{G}", "allreduce", N * G, N * G, inplace=True) as p:
        for n in range(N):
            local = [n * G + g for g in range(G)]
            if intra_parallel:
                with parallelize(N):
                    reduce_scatter(local, 0, N, ch=0)
            else:
                reduce_scatter(local, 0, N, ch=0)
        for g in range(G):
            cross = [n * G + g for n in range(N)]
            reduce_scatter(cross, g * N, 1, ch=1)
        for g in range(G):
            cross = [n * G + g for n in range(N)]
            all_gather(cross, g * N, 1, ch=1)
        for n in range(N):
            local = [n * G + g for g in range(G)]
            if intra_parallel:
                with parallelize(N):
                    all_gather(local, 0, N, ch=2)
            else:
                all_gather(local, 0, N, ch=2)
    return compile_program(p, **opts)


def allpairs_allreduce(R: int, via_scratch: bool = False, **opts) -> Program:
    """Section 7.1.2: every rank receives chunk r from every rank, sums, and broadcasts the result.
    `via_scratch`: the chunks are first copied into the receiver's scratch buffer and reduced locally."""
    with GC3Program(f"dsl_allpairs_allreduce_r{R}" + ("_scratch" if via_scratch else ""), "allreduce", R, R,
                    inplace=True) as p:
        for r in range(R):
            acc = chunk(r, "input", r)
            for d in range(1, R):
                c = chunk((r + d) % R, "input", r)
                if via_scratch:
                    c = c.copy(r, "scratch", d - 1)
                acc = acc.reduce(c)
            for d in range(1, R):
                acc.copy((r + d) % R, "input", r)
    return compile_program(p, **opts)


def direct_alltoall(R: int, **opts) -> Program:
    """Section 7.3: chunk j of rank i goes to rank j, index i, one transfer per pair."""
    with GC3Program(f"dsl_direct_alltoall_r{R}", "alltoall", R, R, R, inplace=False) as p:
        for i in range(R):
            for j in range(R):
                chunk(i, "input", j).copy(j, "output", i)
    return compile_program(p, **opts)


def twostep_alltoall(N: int, G: int, **opts) -> Program:
    """Section 7.3: chunks bound for one remote group are first gathered contiguously in scratch on the
    local rank with the destination's local index, then cross the group boundary in one aggregated
    transfer of G chunks."""
    R = N * G
    with GC3Program(f"dsl_twostep_alltoall_{N}x{G}", "alltoall", R, R, R, inplace=False) as p:
        slot = lambda n, m: m if m < n else m - 1
        for n in range(N):
            for l in range(G):
                src = n * G + l
                for m in range(N):
                    for k in range(G):
                        dst = m * G + k
                        if m == n:
                            chunk(src, "input", dst).copy(dst, "output", src, ch=0)
                        else:
                            chunk(src, "input", dst).copy(n * G + k, "scratch", slot(n, m) * G + l, ch=0)
        for n in range(N):
            for k in range(G):
                for m in range(N):
                    if m != n:
                        chunk(n * G + k, "scratch", slot(n, m) * G, G).copy(m * G + k, "output", n * G, ch=1)
    return compile_program(p, **opts)


def alltonext(N: int, G: int, **opts) -> Program:
    """Section 7.4: rank i's buffer goes to rank i+1; across a group boundary chunk k is carried by the
    k-th rank of the source group and handed on by the k-th rank of the next group."""
    R = N * G
    with GC3Program(f"dsl_alltonext_{N}x{G}", "alltonext", R, G, G, inplace=False) as p:
        for i in range(R - 1):
            j = i + 1
            for k in range(G):
                c = chunk(i, "input", k)
                if i // G == j // G:
                    c.copy(j, "output", k, ch=k)
                    continue
                g = i // G
                relay1, relay2 = g * G + k, (g + 1) * G + k
                if relay1 != i:
                    c = c.copy(relay1, "scratch", 0, ch=k)
                if relay2 != j:
                    c = c.copy(relay2, "scratch", 1, ch=k)
                c.copy(j, "output", k, ch=k)
    return compile_program(p, **opts)
