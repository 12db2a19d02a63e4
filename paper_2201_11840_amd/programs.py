"""CPU generators that emit GC3-IR for the collective algorithms the paper evaluates.

The DSL listings of the paper (hierarchical AllReduce, the ring ReduceScatter /
AllGather helpers, Two-Step AllToAll) are not reproduced here; each schedule is
rebuilt from the prose: Section 2 (hierarchical AllReduce walk-through on N=2
nodes x G=3 GPUs), Section 7.1.1 (Ring AllReduce), Section 7.3 (AllToAll) and
Section 7.4 (AllToNext).  Lowering follows Section 4.2: a remote copy is a
`send` plus a `recv`, a remote reduce is a `send` plus an `rrc`, and back-to-back
pairs are fused into `rcs` / `rrcs` / `rrs` (instruction fusion paragraph).
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence, Tuple

from .ir import Program, ThreadBlock

Dep = Tuple[ThreadBlock, int]


# ---------------------------------------------------------------------------
# Ring helpers: ReduceScatter and AllGather along a ring (Section 2)
# ---------------------------------------------------------------------------

def _emit_ring_reduce_scatter(tb: ThreadBlock, pos: int, G: int, index: Callable[[int], int],
                              count: int, fuse: bool, deps: Sequence[Dep], buf: str = "i") -> int:
    """Ring ReduceScatter as seen by the rank at ring position `pos` of `G`.

    The chunk group with ring number q starts on position q+1, is reduced into
    the same index on every following position and ends, fully reduced, on
    position q (Section 2: GPU 1 sends chunks 0,1 to GPU 2, which adds its own
    and sends to GPU 0).  Returns the step of the last instruction (the `rrc`
    that produces this rank's reduced group)."""
    ref = lambda q: (buf, index(q % G))
    last = tb.add("send", src=ref(pos - 1), count=count, deps=deps)
    for k in range(1, G - 1):
        if fuse:
            last = tb.add("rrcs", src=ref(pos - 1 - k), dst=ref(pos - 1 - k), count=count)
        else:
            tb.add("rrc", src=ref(pos - 1 - k), dst=ref(pos - 1 - k), count=count)
            last = tb.add("send", src=ref(pos - 1 - k), count=count)
    return tb.add("rrc", src=ref(pos), dst=ref(pos), count=count)


def _emit_ring_all_gather(tb: ThreadBlock, pos: int, G: int, index: Callable[[int], int],
                          count: int, fuse: bool, deps: Sequence[Dep], buf: str = "i") -> int:
    """Ring AllGather: the group owned by position q is copied q -> q+1 -> ... for
    G-1 hops (Section 2, final two phases).  Returns the step of the last `recv`."""
    ref = lambda q: (buf, index(q % G))
    tb.add("send", src=ref(pos), count=count, deps=deps)
    for k in range(1, G - 1):
        if fuse:
            tb.add("rcs", dst=ref(pos - k), count=count)
        else:
            tb.add("recv", dst=ref(pos - k), count=count)
            tb.add("send", src=ref(pos - k), count=count)
    return tb.add("recv", dst=ref(pos + 1), count=count)


# ---------------------------------------------------------------------------
# Ring AllReduce (Section 7.1.1) with parallelize(k) instancing (Section 5.1)
# ---------------------------------------------------------------------------

def ring_allreduce(R: int, instances: int = 1, fuse: bool = True, use_rrs: bool = False,
                   name: Optional[str] = None) -> Program:
    """In-place Ring AllReduce on R ranks: ReduceScatter then AllGather over all
    ranks, offset 0, count 1; each chunk goes round the ring twice, 2R-2
    communication steps (Sections 7.1.1 and 7.1.2).

    `instances` = parallelize(k) of the whole program: k replicas, replica j on
    channel j and on 1/k of every ring chunk (IR chunk index = ringChunk*k + j),
    so the buffer has R*k chunks (Section 5.1, chunk parallelization).

    fuse=True gives the single-thread-block schedule send, rrcs x (R-1),
    rcs x (R-2), recv (2R-1 instructions); fuse=False gives the 4(R-1)
    unfused instructions.  use_rrs replaces the first R-2 `rrcs` by `rrs`: their
    local result is overwritten by the AllGather later (Section 4.2, rrs)."""
    if R < 2:
        raise ValueError("ring needs at least 2 ranks")
    if use_rrs and not fuse:
        raise ValueError("rrs is a fused instruction")
    k = instances
    prog = Program(name or f"ring_allreduce_r{R}_x{k}", "allreduce", R, R * k, R * k, inplace=True)
    for j in range(k):
        index = lambda q, j=j: q * k + j
        for r in range(R):
            tb = prog.tb(r, send=(r + 1) % R, recv=(r - 1) % R, chan=j)
            ref = lambda q: ("i", index(q % R))
            if not fuse:
                _emit_ring_reduce_scatter(tb, r, R, index, 1, False, ())
                _emit_ring_all_gather(tb, r, R, index, 1, False, ())
                continue
            tb.add("send", src=ref(r - 1))
            for s in range(1, R - 1):
                if use_rrs:
                    tb.add("rrs", src=ref(r - 1 - s))
                else:
                    tb.add("rrcs", src=ref(r - 1 - s), dst=ref(r - 1 - s))
            # the last reduction produces the chunk this rank owns: it must be
            # stored, and it is also the first send of the AllGather -> rrcs
            tb.add("rrcs", src=ref(r), dst=ref(r))
            for s in range(1, R - 1):
                tb.add("rcs", dst=ref(r - s))
            tb.add("recv", dst=ref(r + 1))
    return prog


def ring_reduce_scatter(R: int, instances: int = 1, name: Optional[str] = None) -> Program:
    """The ring ReduceScatter helper of Section 2 as a collective of its own, out of place: the input has
    R*k chunks, the output k; output chunk j of rank r is the sum over all ranks of input chunk r*k + j.
    The group with ring number q starts on rank q+1 and is summed on its way round to rank q.  The
    intermediate hops use `rrs` (nothing is stored locally, Section 4.2) and the last hop an `rrc` into
    the output, so the input buffers stay as they were."""
    if R < 2:
        raise ValueError("ring needs at least 2 ranks")
    k = instances
    prog = Program(name or f"ring_reducescatter_r{R}_x{k}", "reducescatter", R, R * k, k, inplace=False)
    for j in range(k):
        for r in range(R):
            tb = prog.tb(r, send=(r + 1) % R, recv=(r - 1) % R, chan=j)
            ref = lambda q: ("i", (q % R) * k + j)
            tb.add("send", src=ref(r - 1))
            for s in range(1, R - 1):
                tb.add("rrs", src=ref(r - 1 - s))
            tb.add("rrc", src=ref(r), dst=("o", j))
    return prog


def ring_allgather(R: int, instances: int = 1, name: Optional[str] = None) -> Program:
    """The ring AllGather helper of Section 2 as a collective of its own, out of place: the input has k
    chunks, the output R*k; output chunk q*k + j of every rank is input chunk j of rank q.  Every rank
    copies its own chunks into place and passes each group on for R-1 hops."""
    if R < 2:
        raise ValueError("ring needs at least 2 ranks")
    k = instances
    prog = Program(name or f"ring_allgather_r{R}_x{k}", "allgather", R, k, R * k, inplace=False)
    for j in range(k):
        for r in range(R):
            tb = prog.tb(r, send=(r + 1) % R, recv=(r - 1) % R, chan=j)
            out = lambda q: ("o", (q % R) * k + j)
            tb.add("send", src=("i", j))
            tb.add("copy", src=("i", j), dst=out(r))
            for s in range(1, R - 1):
                tb.add("rcs", dst=out(r - s))
            tb.add("recv", dst=out(r + 1))
    return prog


def multichannel_ring_allreduce(R: int, channels: int, name: Optional[str] = None) -> Program:
    """One logical ring spread over several channels (Section 7.1.1, the schedule used for
    small and medium buffers: the channel differs from operation to operation of the one
    ring).  Ring chunk q travels on channel q mod channels, so
    a rank has one thread block per channel and the chunks of different
    channels overlap their sends and receives.  No cross-thread-block
    dependencies are needed: every location a thread block touches belongs to
    the ring chunks of its own channel."""
    if R < 2 or channels < 1:
        raise ValueError("bad ring shape")
    channels = min(channels, R)
    prog = Program(name or f"mc_ring_allreduce_r{R}_c{channels}", "allreduce", R, R, R, inplace=True)
    # Trace the algorithm chunk by chunk, hop by hop, in global time order; the
    # hop h of every chunk forms one communication step.
    for r in range(R):
        for c in range(channels):
            prog.tb(r, send=(r + 1) % R, recv=(r - 1) % R, chan=c)
    # step h = 0 .. 2R-2 : at step h rank r handles ring chunk q = (r - 1 - h) mod R
    for r in range(R):
        for h in range(2 * R - 1):
            q = (r - 1 - h) % R
            tb = prog.tb(r, send=(r + 1) % R, recv=(r - 1) % R, chan=q % channels)
            ref = ("i", q)
            if h == 0:
                tb.add("send", src=ref)
            elif h < R:
                tb.add("rrcs", src=ref, dst=ref)
            elif h < 2 * R - 2:
                tb.add("rcs", dst=ref)
            else:
                tb.add("recv", dst=ref)
    return prog


# ---------------------------------------------------------------------------
# All Pairs AllReduce (Section 7.1.2)
# ---------------------------------------------------------------------------

def allpairs_allreduce(R: int, name: Optional[str] = None, via_scratch: bool = False) -> Program:
    """Two communication steps: every rank receives chunk r from every other rank,
    sums them, and broadcasts the result to every other rank (Section 7.1.2).
    R chunks, in-place.  Rank r has one thread block per peer p (send p, recv p,
    channel 0) running: send in[p]; rrc in[r]; send in[r]; recv in[p].  The
    reductions into chunk r by different thread blocks are chained by
    cross-thread-block dependencies so the association order is fixed, and the
    broadcast waits for the last of them.

    `via_scratch`: the unfused form - the chunk from the k-th peer is received into
    scratch[k] and a thread block without peers, once all have arrived, adds the scratch
    chunks to in[r] one by one with the local `reduce` instruction (same association order)."""
    if R < 2:
        raise ValueError("needs at least 2 ranks")
    prog = Program(name or f"allpairs_allreduce_r{R}" + ("_scratch" if via_scratch else ""), "allreduce", R, R, R,
                   inplace=True)
    for r in range(R):
        peers = [(r + d) % R for d in range(1, R)]
        tbs = [prog.tb(r, send=p, recv=p, chan=0) for p in peers]
        for tb, p in zip(tbs, peers):
            tb.add("send", src=("i", p))
        prev: Optional[Dep] = None
        if via_scratch:
            arrived = [(tb, tb.add("recv", dst=("s", k))) for k, tb in enumerate(tbs)]
            local = prog.tb(r, send=-1, recv=-1, chan=0)
            for k in range(R - 1):
                # one wait for all arrivals (their semaphores are polled side by side), then R-1 local adds
                prev = (local, local.add("reduce", src=("s", k), dst=("i", r), deps=arrived if k == 0 else ()))
        else:
            for tb in tbs:
                step = tb.add("rrc", src=("i", r), dst=("i", r), deps=[prev] if prev else ())
                prev = (tb, step)
        for tb in tbs:
            tb.add("send", src=("i", r), deps=[prev])
        for tb, p in zip(tbs, peers):
            tb.add("recv", dst=("i", p))
    return prog


# ---------------------------------------------------------------------------
# Hierarchical AllReduce (Section 2, Section 7.2)
# ---------------------------------------------------------------------------

def hierarchical_allreduce(N: int, G: int, fuse: bool = True, phases: int = 4,
                           name: Optional[str] = None) -> Program:
    """In-place AllReduce on N groups ("nodes") of G ranks with N*G chunks in four
    phases (Section 2): (1) ring ReduceScatter inside every group on groups of N
    chunks, (2) ring ReduceScatter across groups between ranks of equal local
    index on single chunks, (3) the matching AllGather across groups, (4) ring
    AllGather inside every group.  Rank n*G+l ends phase 1 owning the group sum
    of chunks l*N .. l*N+N-1 and phase 2 owning the full sum of chunk l*N+n.

    One thread block per (rank, phase), phase p on channel p-1; the first
    instruction of a phase waits on the last instruction of the previous one
    (cross-thread-block dependency, Section 5.2 synchronisation insertion).
    `phases` < 4 emits a prefix of the algorithm (used to check the walk-through
    states)."""
    if N < 2 or G < 2:
        raise ValueError("hierarchical AllReduce needs N >= 2 groups of G >= 2 ranks")
    C = N * G
    prog = Program(name or f"hier_allreduce_{N}x{G}", "allreduce", N * G, C, C, inplace=True)
    last: Dict[int, Dep] = {}
    if phases >= 1:
        for n in range(N):
            for l in range(G):
                r = n * G + l
                tb = prog.tb(r, send=n * G + (l + 1) % G, recv=n * G + (l - 1) % G, chan=0)
                step = _emit_ring_reduce_scatter(tb, l, G, lambda q: q * N, N, fuse, ())
                last[r] = (tb, step)
    if phases >= 2:
        for l in range(G):
            for n in range(N):
                r = n * G + l
                tb = prog.tb(r, send=((n + 1) % N) * G + l, recv=((n - 1) % N) * G + l, chan=1)
                step = _emit_ring_reduce_scatter(tb, n, N, lambda q, l=l: l * N + q, 1, fuse, [last[r]])
                last[r] = (tb, step)
    if phases >= 3:
        for l in range(G):
            for n in range(N):
                r = n * G + l
                tb = prog.tb(r, send=((n + 1) % N) * G + l, recv=((n - 1) % N) * G + l, chan=2)
                step = _emit_ring_all_gather(tb, n, N, lambda q, l=l: l * N + q, 1, fuse, [last[r]])
                last[r] = (tb, step)
    if phases >= 4:
        for n in range(N):
            for l in range(G):
                r = n * G + l
                tb = prog.tb(r, send=n * G + (l + 1) % G, recv=n * G + (l - 1) % G, chan=3)
                _emit_ring_all_gather(tb, l, G, lambda q: q * N, N, fuse, [last[r]])
    return prog


# ---------------------------------------------------------------------------
# AllToAll (Section 7.3)
# ---------------------------------------------------------------------------

def direct_alltoall(R: int, name: Optional[str] = None) -> Program:
    """One-step AllToAll: chunk j of rank i ends on rank j at index i, as a set of
    point-to-point sends and receives between all ranks (Section 7.3).  Rank i
    has a thread block per distance d = 1..R-1 (send peer i+d, receive peer
    i-d, channel 0) holding `send in[i+d]; recv out[i-d]`; the diagonal chunk is
    a local copy."""
    if R < 1:
        raise ValueError("needs at least one rank")
    prog = Program(name or f"direct_alltoall_r{R}", "alltoall", R, R, R, inplace=False)
    for i in range(R):
        if R == 1:
            prog.tb(i).add("copy", src=("i", 0), dst=("o", 0))
            continue
        for d in range(1, R):
            tb = prog.tb(i, send=(i + d) % R, recv=(i - d) % R, chan=0)
            tb.add("send", src=("i", (i + d) % R))
            tb.add("recv", dst=("o", (i - d) % R))
        prog.tb(i, send=(i + 1) % R, recv=(i - 1) % R, chan=0).add("copy", src=("i", i), dst=("o", i))
    return prog


def twostep_alltoall(N: int, G: int, name: Optional[str] = None) -> Program:
    """Two-Step AllToAll on N groups of G ranks (Section 7.3): instead of one small
    cross-group send per (source rank, destination rank) pair, the G chunks a
    rank holds for the G ranks of another group are first gathered, inside the
    source group, on the rank whose local index equals the destination's local
    index, contiguously in scratch; then one aggregated cross-group transfer of
    G chunks per (rank, remote group) moves them to the destination.

    Rank (n,l) chunk for rank (m,k), m != n:  step 1 copies it to rank (n,k)
    scratch[(m', l)] (m' = m's slot among the N-1 remote groups); step 2 sends
    scratch[(m', 0..G-1)] (count G) from (n,k) to (m,k), which receives into
    output indices n*G .. n*G+G-1.  Same-group chunks go directly."""
    if N < 1 or G < 1 or N * G < 2:
        raise ValueError("bad shape")
    R = N * G
    prog = Program(name or f"twostep_alltoall_{N}x{G}", "alltoall", R, R, R, inplace=False)

    def slot(n: int, m: int) -> int:  # position of remote group m among n's remote groups
        return m if m < n else m - 1

    # step 1: intra-group movement (channel 0); a thread block alternates its
    # sends and receives so that it never has more than one send outstanding
    gathered: Dict[Tuple[int, int], List[Dep]] = {}
    remote = lambda n: [m for m in range(N) if m != n]
    for n in range(N):
        for l in range(G):
            me = n * G + l
            local = prog.tb(me, send=n * G + (l + 1) % G, recv=n * G + (l - 1) % G, chan=0) if G > 1 \
                else prog.tb(me, chan=0)
            local.add("copy", src=("i", me), dst=("o", me))
            for m in remote(n):
                st = local.add("copy", src=("i", m * G + l), dst=("s", slot(n, m) * G + l))
                gathered.setdefault((me, m), []).append((local, st))
            for d in range(1, G):
                ks, kr = (l + d) % G, (l - d) % G
                tb = prog.tb(me, send=n * G + ks, recv=n * G + kr, chan=0)
                tb.add("send", src=("i", n * G + ks))
                tb.add("recv", dst=("o", n * G + kr))
                for m in remote(n):
                    tb.add("send", src=("i", m * G + ks))
                    st = tb.add("recv", dst=("s", slot(n, m) * G + kr))
                    gathered.setdefault((me, m), []).append((tb, st))
    # step 2: one aggregated cross-group transfer per (rank, remote group) (channel 1)
    for n in range(N):
        for k in range(G):
            me = n * G + k
            for dm in range(1, N):
                m = (n + dm) % N
                tb = prog.tb(me, send=m * G + k, recv=((n - dm) % N) * G + k, chan=1)
                tb.add("send", src=("s", slot(n, m) * G), count=G, deps=gathered[(me, m)])
    for n in range(N):
        for k in range(G):
            me = n * G + k
            for dm in range(1, N):
                m = (n - dm) % N  # the group we receive from
                tb = prog.tb(me, send=((n + dm) % N) * G + k, recv=m * G + k, chan=1)
                tb.add("recv", dst=("o", m * G), count=G)
    return prog


# ---------------------------------------------------------------------------
# AllToNext (Section 7.4)
# ---------------------------------------------------------------------------

def alltonext(N: int, G: int, name: Optional[str] = None) -> Program:
    """AllToNext on N groups of G ranks: rank i sends its whole buffer (G chunks) to
    rank i+1, the last rank sends nothing and rank 0 receives nothing
    (Section 7.4).  Inside a group chunk k goes directly on channel k.  At a
    group boundary the buffer is divided so every rank of the group carries one
    part across: chunk k goes  last-of-group -> rank k of the source group
    (scratch 0) -> rank k of the next group (scratch 1) -> first-of-next-group
    (output k), all on channel k, and a hop whose two ends coincide is skipped.
    Relays forward with `rcs`."""
    if N < 1 or G < 1:
        raise ValueError("bad shape")
    R = N * G
    prog = Program(name or f"alltonext_{N}x{G}", "alltonext", R, G, G, inplace=False)
    for i in range(R - 1):
        j = i + 1
        if i // G == j // G:
            for k in range(G):
                prog.tb(i, send=j, chan=k).add("send", src=("i", k))
                prog.tb(j, recv=i, chan=k).add("recv", dst=("o", k))
            continue
        g = i // G
        for k in range(G):
            relay1 = g * G + k
            relay2 = (g + 1) * G + k
            # hop 1: i -> relay1 (skipped when relay1 is i itself, k = G-1)
            if relay1 != i:
                prog.tb(i, send=relay1, chan=k).add("send", src=("i", k))
                first_src: Tuple[int, str] = (relay1, "rcs")
            else:
                first_src = (i, "send")
            # hop 2: relay1 -> relay2 ; hop 3: relay2 -> j (skipped when relay2 is j, k = 0)
            if first_src[1] == "send":
                prog.tb(i, send=relay2, chan=k).add("send", src=("i", k))
            else:
                prog.tb(relay1, send=relay2, recv=i, chan=k).add("rcs", dst=("s", 0))
            if relay2 != j:
                prog.tb(relay2, send=j, recv=relay1, chan=k).add("rcs", dst=("s", 1))
                prog.tb(j, recv=relay2, chan=k).add("recv", dst=("o", k))
            else:
                prog.tb(j, recv=relay1, chan=k).add("recv", dst=("o", k))
    return prog


# ---------------------------------------------------------------------------
# Local instructions on their own (Section 4.2: copy and reduce without any connection)
# ---------------------------------------------------------------------------

def local_stream(R: int, tbs_per_rank: int = 8, reduce: bool = False, name: Optional[str] = None) -> Program:
    """No communication at all, thread block j of `tbs_per_rank` on every rank handling its own chunks, no FIFO,
    no flag.  `copy`: out of place, output chunk j = input chunk j.  `reduce`: in place on 2 x tbs_per_rank
    chunks, chunk j += chunk tbs_per_rank + j (two streams read, one written).  Over buffers larger than the
    memory-side cache this is the rate at which the interpreter streams device memory, i.e. the ceiling for
    the user-buffer part of every collective's traffic."""
    if R < 1 or tbs_per_rank < 1:
        raise ValueError("bad shape")
    T = tbs_per_rank
    if reduce:
        prog = Program(name or f"local_reduce_r{R}_x{T}", "custom", R, 2 * T, 2 * T, inplace=True)
        for r in range(R):
            for j in range(T):
                prog.tb(r, chan=j).add("reduce", src=("i", T + j), dst=("i", j))
        return prog
    prog = Program(name or f"local_copy_r{R}_x{T}", "custom", R, T, T, inplace=False)
    for r in range(R):
        for j in range(T):
            prog.tb(r, chan=j).add("copy", src=("i", j), dst=("o", j))
    return prog
