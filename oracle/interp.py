"""Sequential CPU interpreter of GC3-IR (the oracle proper).  Test infrastructure.

Executes a parsed program one instruction at a time, in any order that respects
(a) the sequential order inside a thread block (Section 5, GC3-IR), (b) the
cross-thread-block dependencies (Section 5.2 synchronisation insertion and
Section 6.2 cross thread block synchronisation), (c) FIFO order on every
connection, and optionally (d) at most `slots` outstanding sends per connection
(Section 6.1, remote buffers).  Whole chunks are moved: every instruction is
element-wise, so the runtime's tiling cannot change a value.

Instruction meaning (Section 4.2):
    send   push a copy of the source chunks to the send connection
    recv   pop a message into the destination chunks
    copy   destination <- source
    reduce destination <- destination (+) source
    rrc    destination <- popped message (+) source
    rcs    destination <- popped message, and push it on
    rrcs   destination <- popped message (+) source, and push the result on
    rrs    push popped message (+) source on, no local store
"""
from __future__ import annotations

import random
from collections import Counter, deque
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import numeric
from .irtext import OProgram

POPS = {"recv", "rrc", "rcs", "rrcs", "rrs"}
PUSHES = {"send", "rcs", "rrcs", "rrs"}


class OracleError(RuntimeError):
    pass


class OracleDeadlock(OracleError):
    pass


# ---------------------------------------------------------------------------
# value stores: numeric (numpy arrays) and symbolic (multisets of input chunks)
# ---------------------------------------------------------------------------

class _NumericStore:
    def __init__(self, prog: OProgram, inputs, outputs, scratch, dtype: str):
        self.dtype = dtype
        self.prog = prog
        n_in = inputs[0].size
        if n_in % prog.in_chunks:
            raise OracleError("input length not divisible by the program's chunk count")
        self.ce = n_in // prog.in_chunks
        self.bufs = []
        for r in range(prog.ranks):
            if inputs[r].size != n_in:
                raise OracleError("ranks disagree on input size")
            out = inputs[r] if prog.inplace else outputs[r]
            if out.size != self.ce * prog.out_chunks:
                raise OracleError("output buffer has the wrong size")
            if scratch[r].size < self.ce * prog.scratch_chunks[r]:
                raise OracleError("scratch buffer too small")
            self.bufs.append({"i": inputs[r], "o": out, "s": scratch[r]})

    def read(self, r, buf, idx, count):
        return self.bufs[r][buf][idx * self.ce:(idx + count) * self.ce].copy()

    def write(self, r, buf, idx, count, val):
        self.bufs[r][buf][idx * self.ce:(idx + count) * self.ce] = val

    def add(self, a, b):
        return numeric.add(a, b, self.dtype)


class _SymbolicStore:
    """Chunks as multisets of input chunks (rank, index); None = uninitialised
    (Section 3.1: input, reduction and uninitialised chunks)."""

    def __init__(self, prog: OProgram):
        self.prog = prog
        self.bufs = []
        for r in range(prog.ranks):
            inp = [Counter({(r, j): 1}) for j in range(prog.in_chunks)]
            out = inp if prog.inplace else [None] * prog.out_chunks
            self.bufs.append({"i": inp, "o": out, "s": [None] * prog.scratch_chunks[r]})

    def read(self, r, buf, idx, count):
        vals = self.bufs[r][buf][idx:idx + count]
        if len(vals) != count:
            raise OracleError(f"rank {r}: {buf}[{idx}:{idx + count}] out of range")
        if any(v is None for v in vals):
            raise OracleError(f"rank {r}: read of uninitialised chunk {buf}[{idx}:{idx + count}]")
        return [Counter(v) for v in vals]

    def write(self, r, buf, idx, count, val):
        if idx + count > len(self.bufs[r][buf]):
            raise OracleError(f"rank {r}: {buf}[{idx}:{idx + count}] out of range")
        self.bufs[r][buf][idx:idx + count] = [Counter(v) for v in val]

    def add(self, a, b):
        return [x + y for x, y in zip(a, b)]


# ---------------------------------------------------------------------------
# the interpreter
# ---------------------------------------------------------------------------

def _execute(prog: OProgram, store, slots: Optional[int], order: str, seed: int) -> Dict[str, int]:
    R = prog.ranks
    pc = [[0] * len(prog.tbs[r]) for r in range(R)]
    depth = [[0] * len(prog.tbs[r]) for r in range(R)]   # communication depth reached by each tb
    done_depth: List[List[List[int]]] = [[[] for _ in prog.tbs[r]] for r in range(R)]
    queues: Dict[Tuple[int, int, int], deque] = {}
    rng = random.Random(seed)
    tblist = [(r, b) for r in range(R) for b in range(len(prog.tbs[r]))]
    remaining = sum(len(prog.tbs[r][b].instrs) for r, b in tblist)
    stats = {"instructions": 0, "messages": 0, "comm_steps": 0, "max_outstanding": 0}

    def runnable(r: int, b: int) -> bool:
        tb = prog.tbs[r][b]
        if pc[r][b] >= len(tb.instrs):
            return False
        ins = tb.instrs[pc[r][b]]
        for db, ds in ins.deps:
            if not (0 <= db < len(prog.tbs[r])) or not (0 <= ds < len(prog.tbs[r][db].instrs)):
                raise OracleError(f"rank {r} tb {b}: dependency on a step that does not exist")
            if pc[r][db] <= ds:
                return False
        if ins.opcode in POPS:
            if tb.recv < 0:
                raise OracleError(f"rank {r} tb {b}: {ins.opcode} without receive peer")
            if not queues.get((tb.recv, r, tb.chan)):
                return False
        if ins.opcode in PUSHES:
            if tb.send < 0:
                raise OracleError(f"rank {r} tb {b}: {ins.opcode} without send peer")
            if slots is not None and len(queues.get((r, tb.send, tb.chan), ())) >= slots:
                return False
        return True

    def step(r: int, b: int) -> None:
        tb = prog.tbs[r][b]
        ins = tb.instrs[pc[r][b]]
        op, n = ins.opcode, ins.count
        d = depth[r][b]
        for db, ds in ins.deps:
            d = max(d, done_depth[r][db][ds])
        msg = None
        if op in POPS:
            mcount, mdepth, msg = queues[(tb.recv, r, tb.chan)].popleft()
            if mcount != n:
                raise OracleError(f"rank {r} tb {b} step {pc[r][b]}: message of {mcount} chunks, "
                                  f"instruction expects {n}")
            d = max(d, mdepth)
        if op == "send":
            val = store.read(r, ins.srcbuf, ins.srcidx, n)
        elif op == "recv":
            val = msg
            store.write(r, ins.dstbuf, ins.dstidx, n, val)
        elif op == "copy":
            val = store.read(r, ins.srcbuf, ins.srcidx, n)
            store.write(r, ins.dstbuf, ins.dstidx, n, val)
        elif op == "reduce":
            val = store.add(store.read(r, ins.dstbuf, ins.dstidx, n), store.read(r, ins.srcbuf, ins.srcidx, n))
            store.write(r, ins.dstbuf, ins.dstidx, n, val)
        elif op in ("rrc", "rrcs", "rrs"):
            val = store.add(msg, store.read(r, ins.srcbuf, ins.srcidx, n))
            if op != "rrs":
                store.write(r, ins.dstbuf, ins.dstidx, n, val)
        elif op == "rcs":
            val = msg
            store.write(r, ins.dstbuf, ins.dstidx, n, val)
        else:
            raise OracleError(f"unknown opcode {op}")
        if op in PUSHES:
            q = queues.setdefault((r, tb.send, tb.chan), deque())
            q.append((n, d + 1, val))
            stats["messages"] += 1
            stats["comm_steps"] = max(stats["comm_steps"], d + 1)
            stats["max_outstanding"] = max(stats["max_outstanding"], len(q))
        depth[r][b] = d
        done_depth[r][b].append(d)
        pc[r][b] += 1
        stats["instructions"] += 1

    while remaining:
        if order == "random":
            ready = [(r, b) for r, b in tblist if runnable(r, b)]
            if not ready:
                break
            r, b = rng.choice(ready)
            step(r, b)
            remaining -= 1
        else:  # round robin: one sweep over the thread blocks, one instruction each
            progressed = False
            for r, b in tblist:
                if runnable(r, b):
                    step(r, b)
                    remaining -= 1
                    progressed = True
            if not progressed:
                break
    if remaining:
        stuck = [(r, b, pc[r][b]) for r, b in tblist if pc[r][b] < len(prog.tbs[r][b].instrs)]
        raise OracleDeadlock(f"no runnable thread block; stuck (rank, tb, step): {stuck[:8]}")
    left = {k: len(q) for k, q in queues.items() if q}
    if left:
        raise OracleError(f"messages never received on connections {sorted(left)[:8]}")
    return stats


def run_program(prog: OProgram, inputs: Sequence[np.ndarray], outputs: Optional[Sequence[np.ndarray]],
                dtype: str, scratch: Optional[Sequence[np.ndarray]] = None, slots: Optional[int] = None,
                order: str = "round_robin", seed: int = 0) -> Dict[str, int]:
    """Run `prog` on host arrays (one 1-D array per rank, numpy storage type of
    `dtype`).  In-place programs update `inputs`; others fill `outputs`.  Scratch
    is allocated here when not given.  Returns execution statistics, among them
    `comm_steps`, the length of the longest chain of dependent messages."""
    if dtype not in numeric.DTYPES:
        raise OracleError(f"unknown dtype {dtype}")
    st = numeric.STORAGE[dtype]
    for a in inputs:
        if a.dtype != st or a.ndim != 1:
            raise OracleError("input arrays must be 1-D arrays of the dtype's storage type")
    if not prog.inplace:
        if outputs is None:
            raise OracleError("out-of-place program needs output arrays")
        for a in outputs:
            if a.dtype != st or a.ndim != 1:
                raise OracleError("output arrays must be 1-D arrays of the dtype's storage type")
    ce = inputs[0].size // max(prog.in_chunks, 1)
    if scratch is None:
        scratch = [np.zeros(ce * prog.scratch_chunks[r], dtype=st) for r in range(prog.ranks)]
    store = _NumericStore(prog, inputs, outputs, scratch, dtype)
    return _execute(prog, store, slots, order, seed)


def run_symbolic(prog: OProgram, slots: Optional[int] = None, order: str = "round_robin", seed: int = 0):
    """Run `prog` on symbolic chunks.  Returns (buffers, stats): buffers[r][buf] is
    a list with one multiset (Counter of (rank, input index)) or None
    (uninitialised) per chunk, buf in 'i', 'o', 's'."""
    store = _SymbolicStore(prog)
    stats = _execute(prog, store, slots, order, seed)
    return store.bufs, stats
