"""GC3-IR program builder and text serialiser (CPU side, generator use only).

The GC3-IR is the tree the paper describes in Section 5 ("GC3-IR" paragraph):
program -> per-GPU program -> thread blocks -> sequential instruction list,
where a thread block has at most one send peer and one receive peer plus a
channel.  An instruction carries what the interpreter figure of Section 6.2
lists: opcode, source/destination buffer and chunk offset, count, the
(thread block, step) pairs it depends on, and a has-dependent flag.

The paper fixes the IR's content but no file format; the line-oriented text
below is this library's own.  Grammar (tokens separated by blanks, `#` starts a
comment, one statement per line):

    gc3ir 1
    name <token>
    collective <token>
    inplace <0|1>
    protocol <simple|ll|ll128|auto>  (Section 6.1 protocols; auto = the runtime picks by message size)
    ranks <R>
    chunks <in_chunks> <out_chunks>  (per rank)
    rank <r> scratch <n_chunks> tbs <n_tbs>      (ranks in order 0..R-1)
    tb <id> send <peer|-1> recv <peer|-1> chan <c> ops <n>   (ids 0..n_tbs-1)
    op <opcode> <srcbuf> <srcidx> <dstbuf> <dstidx> <count> <hasdep> <ndeps> {<tb> <step>}
    end

opcode is one of send recv copy reduce rrc rcs rrcs rrs; a buffer is `i`, `o`,
`s` or `-` (operand unused, index 0).  Dependencies name a thread block of the
same rank and one of its steps.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

OPCODES = ("send", "recv", "copy", "reduce", "rrc", "rcs", "rrcs", "rrs")
# which opcodes pop a message from the receive connection / push one to the send connection
POPS = {"recv", "rrc", "rcs", "rrcs", "rrs"}
PUSHES = {"send", "rcs", "rrcs", "rrs"}
USES_SRC = {"send", "copy", "reduce", "rrc", "rrcs", "rrs"}
USES_DST = {"recv", "copy", "reduce", "rrc", "rcs", "rrcs"}
BUFFERS = ("i", "o", "s")


@dataclass
class Op:
    opcode: str
    srcbuf: str = "-"
    srcidx: int = 0
    dstbuf: str = "-"
    dstidx: int = 0
    count: int = 1
    hasdep: bool = False
    deps: List[Tuple[int, int]] = field(default_factory=list)


@dataclass
class ThreadBlock:
    rank: int
    tbid: int
    send: int
    recv: int
    chan: int
    ops: List[Op] = field(default_factory=list)

    def add(self, opcode: str, src: Optional[Tuple[str, int]] = None,
            dst: Optional[Tuple[str, int]] = None, count: int = 1,
            deps: Sequence[Tuple["ThreadBlock", int]] = ()) -> int:
        """Append one instruction, return its step.  `deps` are (thread block, step)
        pairs of the same rank; the dependee gets its has-dependent flag set
        (synchronisation insertion, Section 5.2)."""
        if opcode not in OPCODES:
            raise ValueError(f"unknown opcode {opcode}")
        if opcode in PUSHES and self.send < 0:
            raise ValueError(f"{opcode} in a thread block without send peer")
        if opcode in POPS and self.recv < 0:
            raise ValueError(f"{opcode} in a thread block without receive peer")
        if (opcode in USES_SRC) != (src is not None):
            raise ValueError(f"{opcode}: source operand mismatch")
        if (opcode in USES_DST) != (dst is not None):
            raise ValueError(f"{opcode}: destination operand mismatch")
        op = Op(opcode, count=count)
        if src is not None:
            op.srcbuf, op.srcidx = src
        if dst is not None:
            op.dstbuf, op.dstidx = dst
        for tb, step in deps:
            if tb.rank != self.rank:
                raise ValueError("cross-rank dependency")
            if tb is self:
                continue  # same thread block: order is implicit
            if not (0 <= step < len(tb.ops)):
                raise ValueError("dependency on a step that does not exist yet")
            tb.ops[step].hasdep = True
            if (tb.tbid, step) not in op.deps:
                op.deps.append((tb.tbid, step))
        self.ops.append(op)
        return len(self.ops) - 1


class Program:
    """A whole GC3-IR program under construction."""

    def __init__(self, name: str, collective: str, ranks: int, in_chunks: int,
                 out_chunks: int, inplace: bool, protocol: str = "simple"):
        self.name = name
        self.collective = collective
        self.ranks = ranks
        self.in_chunks = in_chunks
        self.out_chunks = out_chunks
        self.inplace = inplace
        self.protocol = protocol
        self.tbs: List[List[ThreadBlock]] = [[] for _ in range(ranks)]
        self._by_key: Dict[Tuple[int, int, int, int], ThreadBlock] = {}

    def tb(self, rank: int, send: int = -1, recv: int = -1, chan: int = 0) -> ThreadBlock:
        """The thread block of `rank` with this (send peer, receive peer, channel),
        created on first use (Section 5.2, thread block assignment step 1)."""
        key = (rank, send, recv, chan)
        t = self._by_key.get(key)
        if t is None:
            t = ThreadBlock(rank, len(self.tbs[rank]), send, recv, chan)
            self.tbs[rank].append(t)
            self._by_key[key] = t
        return t

    def scratch_chunks(self, rank: int) -> int:
        """Scratch size is deduced from the highest scratch index used (Section 3.2)."""
        hi = 0
        for t in self.tbs[rank]:
            for op in t.ops:
                if op.srcbuf == "s":
                    hi = max(hi, op.srcidx + op.count)
                if op.dstbuf == "s":
                    hi = max(hi, op.dstidx + op.count)
        return hi

    def num_tbs(self) -> int:
        return sum(len(t) for t in self.tbs)

    def num_ops(self) -> int:
        return sum(len(t.ops) for r in self.tbs for t in r)

    def max_count(self) -> int:
        return max((op.count for r in self.tbs for t in r for op in t.ops), default=1)

    def algorithmic_chunks(self) -> int:
        """Global-memory traffic of one run in units of one chunk: per instruction
        (count x) send 2, recv 2, copy 2, reduce 3, rrc 3, rcs 3, rrcs 4, rrs 3."""
        w = {"send": 2, "recv": 2, "copy": 2, "reduce": 3, "rrc": 3, "rcs": 3, "rrcs": 4, "rrs": 3}
        return sum(w[op.opcode] * op.count for r in self.tbs for t in r for op in t.ops)

    def fifo_chunks(self) -> int:
        """The part of algorithmic_chunks() that is FIFO traffic: one chunk written per pushed and one
        read per popped message chunk."""
        return sum(op.count * ((op.opcode in PUSHES) + (op.opcode in POPS))
                   for r in self.tbs for t in r for op in t.ops)

    def to_text(self) -> str:
        out = ["gc3ir 1", f"name {self.name}", f"collective {self.collective}",
               f"inplace {int(self.inplace)}", f"protocol {self.protocol}",
               f"ranks {self.ranks}", f"chunks {self.in_chunks} {self.out_chunks}"]
        for r in range(self.ranks):
            out.append(f"rank {r} scratch {self.scratch_chunks(r)} tbs {len(self.tbs[r])}")
            for t in self.tbs[r]:
                out.append(f"tb {t.tbid} send {t.send} recv {t.recv} chan {t.chan} ops {len(t.ops)}")
                for op in t.ops:
                    deps = "".join(f" {b} {s}" for b, s in op.deps)
                    out.append(f"op {op.opcode} {op.srcbuf} {op.srcidx} {op.dstbuf} {op.dstidx} "
                               f"{op.count} {int(op.hasdep)} {len(op.deps)}{deps}")
        out.append("end")
        return "\n".join(out) + "\n"
