"""Lowering and scheduling of a traced DSL program into GC3-IR (Sections 4 and 5 of the paper).

Pipeline: traced chunk operations (Chunk DAG, Section 4.1) -> instances for parallelized fragments
(Section 5.1) -> instruction nodes with processing and communication edges (Instruction DAG,
Section 4.2) -> peephole fusion into rcs / rrcs / rrs (Section 4.2) -> channel assignment
(Section 5.2: user directives first, else the lowest valid channel; a fused chain shares one channel;
instances get channels of their own) -> thread blocks per (send peer, receive peer, channel), a global
topological order by dependency depth and reverse depth, greedy assignment (Section 5.2) ->
cross-thread-block dependencies for the processing edges that leave a thread block (Section 5.2,
synchronisation insertion).
"""
from __future__ import annotations

import copy
import heapq
from dataclasses import dataclass, field
from math import gcd
from typing import Dict, List, Optional, Set, Tuple

from .dsl import GC3Program
from .ir import Program, ThreadBlock


class CompileError(RuntimeError):
    pass


@dataclass
class Node:
    id: int
    rank: int
    opcode: str
    src: Optional[Tuple[str, int]]
    dst: Optional[Tuple[str, int]]
    count: int
    ch: Optional[int]          # user channel directive, None = compiler's choice
    inst: int                  # instance of a parallelized fragment
    order: int                 # position of the originating chunk operation in the trace
    push_order: int = -1       # trace position of the operation whose send this node performs
    send_peer: int = -1
    recv_peer: int = -1
    preds: Dict[int, Set[str]] = field(default_factory=dict)   # processing edges: node -> {"raw","war","waw"}
    comm_from: Optional[int] = None
    comm_to: Optional[int] = None
    alive: bool = True
    tb: Optional["_Tb"] = None


@dataclass
class _Tb:
    rank: int
    send: int = -1
    recv: int = -1
    chan: Tuple[int, int] = (0, 0)
    last_pos: int = -1
    obj: Optional[ThreadBlock] = None
    alias: Optional["_Tb"] = None      # set when this thread block was merged into another

    def resolve(self) -> "_Tb":
        t = self
        while t.alias is not None:
            t = t.alias
        return t


def _lcm(a: int, b: int) -> int:
    return a * b // gcd(a, b)


def compile_program(prog: GC3Program, fuse: bool = True, use_rrs: bool = False) -> Program:
    R = prog.ranks
    F = 1
    for op in prog.ops:
        F = _lcm(F, op.par)

    # ---- instances: every operation on refined chunks (1/F of a chunk) --------------------------------
    concrete = []   # (kind, src(rank,buf,idx,cnt), dst, ch, inst, order)
    for op in prog.ops:
        n = op.par
        (sr, sb, si, sc), (dr, db, di, dc) = op.src, op.dst
        if (sc * F) % n:
            raise CompileError("parallelize factor does not divide the referenced range")
        cnt = sc * F // n
        for i in range(n):
            concrete.append((op.kind, (sr, sb, si * F + i * cnt, cnt), (dr, db, di * F + i * cnt, cnt), op.ch, i, op.order))

    # ---- instruction generation with processing edges -----------------------------------------------
    nodes: List[Node] = []
    last_writer: Dict[Tuple[int, str, int], int] = {}
    readers: Dict[Tuple[int, str, int], Set[int]] = {}

    def new(rank, opcode, src, dst, count, ch, inst, order) -> Node:
        nd = Node(len(nodes), rank, opcode, src, dst, count, ch, inst, order)
        nodes.append(nd)
        return nd

    # processing edges per location: (producer, consumer) -> location -> kinds.  An instruction with count > 1
    # covers several chunks, and a later instruction may touch only some of them.
    edge_locs: Dict[Tuple[int, int], Dict[Tuple[int, str, int], Set[str]]] = {}

    def edge(nd: Node, pred: int, kind: str, loc: Tuple[int, str, int]) -> None:
        if pred != nd.id:
            nd.preds.setdefault(pred, set()).add(kind)
            edge_locs.setdefault((pred, nd.id), {}).setdefault(loc, set()).add(kind)

    def reads(nd: Node, rank, buf, idx, cnt) -> None:
        for k in range(cnt):
            loc = (rank, buf, idx + k)
            if loc in last_writer:
                edge(nd, last_writer[loc], "raw", loc)
            readers.setdefault(loc, set()).add(nd.id)

    def writes(nd: Node, rank, buf, idx, cnt) -> None:
        for k in range(cnt):
            loc = (rank, buf, idx + k)
            if loc in last_writer:
                edge(nd, last_writer[loc], "waw", loc)
            for rd in readers.get(loc, ()):
                edge(nd, rd, "war", loc)
            last_writer[loc] = nd.id
            readers[loc] = set()

    for kind, (sr, sb, si, cnt), (dr, db, di, _), ch, inst, order in concrete:
        if sr == dr:                                    # local operation: a single instruction
            nd = new(sr, kind, (sb, si), (db, di), cnt, ch, inst, order)
            reads(nd, sr, sb, si, cnt)
            if kind == "reduce":
                reads(nd, dr, db, di, cnt)
            writes(nd, dr, db, di, cnt)
            continue
        snd = new(sr, "send", (sb, si), None, cnt, ch, inst, order)      # remote: send + recv / rrc
        snd.send_peer, snd.push_order = dr, order
        reads(snd, sr, sb, si, cnt)
        if kind == "copy":
            rcv = new(dr, "recv", None, (db, di), cnt, ch, inst, order)
        else:
            rcv = new(dr, "rrc", (db, di), (db, di), cnt, ch, inst, order)
            reads(rcv, dr, db, di, cnt)
        rcv.recv_peer = sr
        writes(rcv, dr, db, di, cnt)
        snd.comm_to, rcv.comm_from = rcv.id, snd.id

    def successors() -> Dict[int, List[int]]:
        succ: Dict[int, List[int]] = {n.id: [] for n in nodes if n.alive}
        for n in nodes:
            if not n.alive:
                continue
            for p in n.preds:
                succ[p].append(n.id)
            if n.comm_from is not None:
                succ[n.comm_from].append(n.id)
        return succ

    def reverse_depth() -> Dict[int, int]:
        succ = successors()
        memo: Dict[int, int] = {}
        for n in reversed([n for n in nodes if n.alive]):      # trace order is topological
            memo[n.id] = 1 + max((memo[s] for s in succ[n.id]), default=-1)
        return memo

    # ---- instruction fusion (peephole) ------------------------------------------------------------------
    if fuse:
        rdepth = reverse_depth()
        for r_node in nodes:
            if not r_node.alive or r_node.opcode not in ("recv", "rrc"):
                continue
            cands = [s for s in nodes if s.alive and s.opcode == "send" and s.rank == r_node.rank
                     and s.src == r_node.dst and s.count == r_node.count and s.inst == r_node.inst
                     and r_node.id in s.preds and set(s.preds) - {r_node.id} <= set(r_node.preds)
                     and (s.ch is None or r_node.ch is None or s.ch == r_node.ch)]
            if not cands:
                continue
            s_node = max(cands, key=lambda s: (rdepth[s.id], -s.order))   # the send on the longest path
            r_node.opcode = "rcs" if r_node.opcode == "recv" else "rrcs"
            r_node.send_peer, r_node.push_order = s_node.send_peer, s_node.push_order
            r_node.comm_to = s_node.comm_to
            nodes[s_node.comm_to].comm_from = r_node.id
            if r_node.ch is None:
                r_node.ch = s_node.ch
            for p, kinds in s_node.preds.items():
                if p != r_node.id:
                    r_node.preds.setdefault(p, set()).update(kinds)
            s_node.alive = False
            for x in nodes:
                if x.alive and s_node.id in x.preds:
                    kinds = x.preds.pop(s_node.id)
                    if x.id != r_node.id:
                        x.preds.setdefault(r_node.id, set()).update(kinds)
        if use_rrs:
            # The local store of an rrcs may be dropped when, for EVERY chunk it covers, the reduced value is
            # overwritten later and not read before that.  Decided per location: with count > 1 a later write
            # may cover only part of the range, and the rest must keep the reduced value.
            consumers: Dict[int, List[int]] = {}
            for (producer, consumer) in edge_locs:
                consumers.setdefault(producer, []).append(consumer)
            for n in nodes:
                if not (n.alive and n.opcode == "rrcs"):
                    continue
                droppable = True
                for k in range(n.count):
                    loc = (n.rank, n.dst[0], n.dst[1] + k)
                    kinds: Set[str] = set()
                    for x in consumers.get(n.id, ()):
                        if nodes[x].alive:
                            kinds |= edge_locs[(n.id, x)].get(loc, set())
                    if "raw" in kinds or "waw" not in kinds:
                        droppable = False
                        break
                if droppable:
                    n.opcode, n.dst = "rrs", None

    alive = [n for n in nodes if n.alive]

    # ---- channel assignment: one channel per chain of communication edges -------------------------------
    parent = {n.id: n.id for n in alive}

    def find(x: int) -> int:
        while parent[x] != x:
            parent[x] = parent[parent[x]]
            x = parent[x]
        return x

    for n in alive:
        if n.comm_to is not None:
            parent[find(n.id)] = find(n.comm_to)
    chains: Dict[int, List[Node]] = {}
    for n in alive:
        if n.comm_to is not None or n.comm_from is not None:
            chains.setdefault(find(n.id), []).append(n)

    root_of = {id(c): r for r, c in chains.items()}
    user_channels = [n.ch for n in alive if n.ch is not None]
    base_fresh = max(user_channels, default=-1) + 1 + len(chains)      # beyond anything assigned otherwise

    def attempt(separate: Dict[int, int]):
        """Assign channels and thread blocks, then schedule.  Returns (order, None) or (None, a pop that
        could not be scheduled because its connection would have to deliver out of order)."""
        for n in alive:
            n.tb = None
        state: List[Dict] = [{"send": {}, "recv": {}} for _ in range(R)]    # (peer, chan) -> _Tb

        def place(chain: List[Node], chan: Tuple[int, int], commit: bool) -> bool:
            """Can the chain's instructions live in thread blocks with one send and one receive peer each,
            one sending and one receiving thread block per connection (Section 5, GC3-IR)?"""
            trial = state if commit else copy.deepcopy(state)     # a dry run works on a copy

            for n in chain:
                st = trial[n.rank]
                ts = st["send"].get((n.send_peer, chan)) if n.send_peer >= 0 else None
                tr = st["recv"].get((n.recv_peer, chan)) if n.recv_peer >= 0 else None
                if n.send_peer >= 0 and n.recv_peer >= 0:
                    if ts is None and tr is None:
                        t = _Tb(n.rank, n.send_peer, n.recv_peer, chan)
                    elif ts is not None and tr is None:
                        if ts.recv not in (-1, n.recv_peer):
                            return False
                        ts.recv, t = n.recv_peer, ts
                    elif tr is not None and ts is None:
                        if tr.send not in (-1, n.send_peer):
                            return False
                        tr.send, t = n.send_peer, tr
                    elif ts is tr:
                        t = ts
                    elif ts.recv == -1 and tr.send == -1:
                        # a send-only and a receive-only thread block on this channel become one
                        ts.recv, tr.alias, t = tr.recv, ts, ts
                        for d in (st["send"], st["recv"]):
                            for key, val in d.items():
                                if val is tr:
                                    d[key] = ts
                    else:
                        return False        # a thread block would need two send or two receive peers
                    st["send"][(n.send_peer, chan)] = t
                    st["recv"][(n.recv_peer, chan)] = t
                elif n.send_peer >= 0:
                    t = ts if ts is not None else _Tb(n.rank, n.send_peer, -1, chan)
                    st["send"][(n.send_peer, chan)] = t
                else:
                    t = tr if tr is not None else _Tb(n.rank, -1, n.recv_peer, chan)
                    st["recv"][(n.recv_peer, chan)] = t
                if commit:
                    n.tb = t
            return True

        for chain in sorted(chains.values(), key=lambda c: min(n.order for n in c)):
            wanted = {n.ch for n in chain if n.ch is not None}
            insts = {n.inst for n in chain}
            if len(wanted) > 1 or len(insts) > 1:
                raise CompileError("a chain of fused instructions carries conflicting channel directives")
            inst = insts.pop()
            if wanted:
                c = wanted.pop()
                if not place(chain, (c, inst), commit=False):
                    raise CompileError(f"channel {c} cannot serve this transfer: a thread block would need two peers; use another ch=")
            else:
                c = 0
                if root_of[id(chain)] in separate:                   # a channel of its own (see below)
                    c = base_fresh + separate[root_of[id(chain)]]
                while not place(chain, (c, inst), commit=False):     # the lowest valid channel
                    c += 1
                    if c > 4096:
                        raise CompileError("no valid channel found")
            place(chain, (c, inst), commit=True)

        for n in alive:
            if n.tb is not None:
                n.tb = n.tb.resolve()

        # ---- global order (Section 5.2): list scheduling by dependency depth, then reverse depth -------------
        # Instructions are taken one by one in a topological order of the processing and communication
        # edges, lower depth first, higher reverse depth second.  A connection is a FIFO, so the order in
        # which its pushes are scheduled is the order in which the matching pops must be scheduled: a pop
        # becomes eligible only when its push is the oldest unconsumed one on its connection.
        preds_all = {n.id: set(n.preds) | ({n.comm_from} if n.comm_from is not None else set()) for n in alive}
        succ_all: Dict[int, List[int]] = {n.id: [] for n in alive}
        for i, ps in preds_all.items():
            for p in ps:
                succ_all[p].append(i)
        order_ids = [n.id for n in alive]                      # trace order is a topological order
        depth = {i: 0 for i in order_ids}
        for i in order_ids:
            for p in preds_all[i]:
                depth[i] = max(depth[i], depth[p] + 1)
        rdep = {i: 0 for i in order_ids}
        for i in reversed(order_ids):
            for sx in succ_all[i]:
                rdep[i] = max(rdep[i], rdep[sx] + 1)
        indeg = {i: len(ps) for i, ps in preds_all.items()}
        key = lambda i: (depth[i], -rdep[i], nodes[i].order, i)
        fifo: Dict[Tuple[int, int, Tuple[int, int]], List[int]] = {}
        blocked: Dict[Tuple[int, int, Tuple[int, int]], Dict[int, int]] = {}
        heap: List[Tuple[int, int, int, int]] = []

        def conn_in(n: Node):
            return (n.recv_peer, n.rank, n.tb.chan)

        def offer(i: int) -> None:
            n = nodes[i]
            if n.comm_from is not None:
                q = fifo.get(conn_in(n), [])
                if not q or q[0] != n.comm_from:
                    blocked.setdefault(conn_in(n), {})[n.comm_from] = i
                    return
            heapq.heappush(heap, key(i))

        for i in order_ids:
            if indeg[i] == 0:
                offer(i)
        sorted_ids: List[int] = []
        while heap:
            i = heapq.heappop(heap)[3]
            n = nodes[i]
            sorted_ids.append(i)
            if n.comm_from is not None:
                q = fifo[conn_in(n)]
                q.pop(0)
                if q and q[0] in blocked.get(conn_in(n), {}):
                    heapq.heappush(heap, key(blocked[conn_in(n)].pop(q[0])))
            if n.comm_to is not None:
                conn = (n.rank, n.send_peer, n.tb.chan)
                fifo.setdefault(conn, []).append(i)
            for sx in succ_all[i]:
                indeg[sx] -= 1
                if indeg[sx] == 0:
                    offer(sx)
        if len(sorted_ids) != len(order_ids):
            stuck = [i for d in blocked.values() for i in d.values()]
            return None, min(stuck, key=lambda i: nodes[i].order) if stuck else None
        return sorted_ids, None


    # Fusion can tie a receive early in the program to a send late in it; two such transfers sharing a
    # connection may then be needed in opposite orders at its two ends.  Such a chain is moved to a
    # channel of its own and the schedule is tried again.
    separate: Dict[int, int] = {}
    while True:
        sorted_ids, stuck = attempt(separate)
        if sorted_ids is not None:
            break
        if stuck is None:
            raise CompileError("the instruction graph cannot be scheduled")
        root = find(stuck)
        if root in separate or any(n.ch is not None for n in chains[root]):
            raise CompileError("no schedule keeps every connection first-in first-out: two transfers on one "
                               "connection are needed in opposite orders at its two ends; give them different channels")
        separate[root] = len(separate)

    # ---- thread blocks and emission ----------------------------------------------------------------------
    chan_ids = sorted({n.tb.chan for n in alive if n.tb is not None})
    dense = {c: k for k, c in enumerate(chan_ids)}
    out = Program(prog.name, prog.collective, R, prog.in_chunks * F, prog.out_chunks * F, prog.inplace, prog.protocol)
    rank_tbs: List[List[_Tb]] = [[] for _ in range(R)]
    for n in sorted(alive, key=lambda n: n.order):
        if n.tb is not None and n.tb not in rank_tbs[n.rank]:
            rank_tbs[n.rank].append(n.tb)
    emitted: Dict[int, Tuple[ThreadBlock, int]] = {}
    for pos, i in enumerate(sorted_ids):
        n = nodes[i]
        if n.tb is None:
            # a local instruction may run on any thread block: take the one whose latest instruction is earliest
            if not rank_tbs[n.rank]:
                rank_tbs[n.rank].append(_Tb(n.rank))
            n.tb = min(rank_tbs[n.rank], key=lambda t: t.last_pos)
        t = n.tb
        if t.obj is None:
            t.obj = out.tb(t.rank, t.send, t.recv, dense.get(t.chan, 0))
        t.last_pos = pos
        deps = {}
        for p in n.preds:
            ptb, pstep = emitted[p]
            if ptb is not t.obj:
                deps[id(ptb)] = (ptb, max(pstep, deps.get(id(ptb), (ptb, -1))[1]))
        step = t.obj.add(n.opcode, src=n.src, dst=n.dst, count=n.count, deps=list(deps.values()))
        emitted[i] = (t.obj, step)
    return out
