"""The chunk-oriented DSL of the paper (Section 3) as a traced Python API.

    with GC3Program("ring", "allreduce", ranks=R, in_chunks=R, inplace=True) as prog:
        c = chunk(rank, "input", index, count=1)       # reference to chunks currently in a buffer
        c = c.copy(rank2, "input", index2, ch=0)       # copy (remote or local), returns the new reference
        c = chunk(rank2, "input", index2).reduce(c)    # in-place reduction into the first operand
        with parallelize(N): ...                       # chunk parallelization (Section 5.1)
    ir_program = compiler.compile_program(prog)

Tracing runs the program once and records every copy / reduce (Section 4.1).  While tracing, each
location carries its symbolic content - an input chunk (rank, index), a reduction chunk (multiset of
input chunks) or uninitialised (Section 3.1) - so that reading an uninitialised chunk and using a stale
reference raise immediately (Section 3.3), and the collective's postcondition (Section 3.2) is checked
when the `with` block ends.
"""
from __future__ import annotations

from collections import Counter
from dataclasses import dataclass
from typing import Dict, List, Optional, Tuple

BUFFER_ALIASES = {"input": "i", "output": "o", "scratch": "s", "i": "i", "o": "o", "s": "s"}


class DslError(RuntimeError):
    pass


@dataclass
class TraceOp:
    kind: str                      # "copy" or "reduce"
    src: Tuple[int, str, int, int]  # rank, buffer, index, count
    dst: Tuple[int, str, int, int]
    ch: Optional[int]
    par: int                       # parallelize factor in force (1 = none)
    order: int


_current: Optional["GC3Program"] = None


def _prog() -> "GC3Program":
    if _current is None:
        raise DslError("no GC3Program is being traced")
    return _current


class GC3Program:
    def __init__(self, name: str, collective: str, ranks: int, in_chunks: int, out_chunks: Optional[int] = None,
                 inplace: bool = False, protocol: str = "simple", check: bool = True):
        self.name, self.collective, self.ranks = name, collective, ranks
        self.in_chunks = in_chunks
        self.out_chunks = in_chunks if out_chunks is None else out_chunks
        self.inplace, self.protocol, self.check = inplace, protocol, check
        if inplace and self.out_chunks != self.in_chunks:
            raise DslError("an in-place collective has equally many input and output chunks")
        self.ops: List[TraceOp] = []
        self._par = 1
        # symbolic content and version of every location
        self.content: List[Dict[str, List[Optional[Counter]]]] = []
        self.version: List[Dict[str, List[int]]] = []
        for r in range(ranks):
            inp: List[Optional[Counter]] = [Counter({(r, j): 1}) for j in range(in_chunks)]
            out = inp if inplace else [None] * self.out_chunks
            self.content.append({"i": inp, "o": out, "s": []})
            vin = [0] * in_chunks
            self.version.append({"i": vin, "o": vin if inplace else [0] * self.out_chunks, "s": []})

    # -- context management -------------------------------------------------------------------------
    def __enter__(self) -> "GC3Program":
        global _current
        if _current is not None:
            raise DslError("GC3Program blocks cannot be nested")
        _current = self
        return self

    def __exit__(self, exc_type, exc, tb) -> None:
        global _current
        _current = None
        if exc_type is None and self.check:
            self.check_postcondition()

    # -- helpers ----------------------------------------------------------------------------------------
    def _buf(self, name: str) -> str:
        if name not in BUFFER_ALIASES:
            raise DslError(f"unknown buffer {name}")
        b = BUFFER_ALIASES[name]
        return "i" if (b == "o" and self.inplace) else b

    def _grow_scratch(self, rank: int, upto: int) -> None:
        c, v = self.content[rank]["s"], self.version[rank]["s"]
        while len(c) < upto:
            c.append(None)
            v.append(0)

    def _check_range(self, rank: int, buf: str, index: int, count: int, grow: bool) -> None:
        if not (0 <= rank < self.ranks):
            raise DslError(f"rank {rank} out of range")
        if count < 1 or index < 0:
            raise DslError("bad chunk range")
        if buf == "s":
            if grow:
                self._grow_scratch(rank, index + count)   # scratch size follows the highest index used
        if index + count > len(self.content[rank][buf]):
            raise DslError(f"rank {rank}: {buf}[{index}:{index + count}] is outside the buffer")

    def scratch_chunks(self, rank: int) -> int:
        return len(self.content[rank]["s"])

    def check_postcondition(self) -> None:
        R = self.ranks
        for r in range(R):
            for j in range(self.out_chunks):
                got = self.content[r]["o"][j]
                if self.collective == "allreduce":
                    want: Optional[Counter] = Counter({(q, j): 1 for q in range(R)})
                elif self.collective == "alltoall":
                    per = self.out_chunks // R
                    want = Counter({(j // per, r * per + j % per): 1})
                elif self.collective == "alltonext":
                    want = None if r == 0 else Counter({(r - 1, j): 1})
                elif self.collective == "allgather":
                    per = self.out_chunks // R
                    want = Counter({(j // per, j % per): 1})
                elif self.collective == "reducescatter":
                    want = Counter({(q, r * self.out_chunks + j): 1 for q in range(R)})
                elif self.collective == "custom":
                    continue
                else:
                    raise DslError(f"no postcondition known for collective {self.collective}")
                if got != want:
                    raise DslError(f"postcondition violated: rank {r} output chunk {j} holds {got}, needs {want}")


class Ref:
    """Reference to `count` contiguous chunks at (rank, buffer, index) as they were when it was made."""

    def __init__(self, rank: int, buffer: str, index: int, count: int):
        p = _prog()
        self.rank, self.buffer, self.index, self.count = rank, p._buf(buffer), index, count
        p._check_range(rank, self.buffer, index, count, grow=False)
        self.versions = list(p.version[rank][self.buffer][index:index + count])

    def _use(self) -> None:
        p = _prog()
        now = p.version[self.rank][self.buffer][self.index:self.index + self.count]
        if now != self.versions:
            raise DslError(f"stale reference to rank {self.rank} {self.buffer}[{self.index}:{self.index + self.count}]")
        if any(c is None for c in p.content[self.rank][self.buffer][self.index:self.index + self.count]):
            raise DslError(f"rank {self.rank} {self.buffer}[{self.index}:{self.index + self.count}] is uninitialised")

    def copy(self, rank: int, buffer: str, index: int, ch: Optional[int] = None) -> "Ref":
        p = _prog()
        self._use()
        b = p._buf(buffer)
        p._check_range(rank, b, index, self.count, grow=True)
        if (rank, b) == (self.rank, self.buffer) and abs(index - self.index) < self.count:
            raise DslError("copy onto an overlapping range")
        src = p.content[self.rank][self.buffer]
        for k in range(self.count):
            p.content[rank][b][index + k] = Counter(src[self.index + k])
            p.version[rank][b][index + k] += 1
        p.ops.append(TraceOp("copy", (self.rank, self.buffer, self.index, self.count), (rank, b, index, self.count),
                             ch, p._par, len(p.ops)))
        return Ref(rank, b, index, self.count)

    def reduce(self, other: "Ref", ch: Optional[int] = None) -> "Ref":
        p = _prog()
        self._use()
        other._use()
        if other.count != self.count:
            raise DslError("reduce needs references of equal count")
        if (other.rank, other.buffer) == (self.rank, self.buffer) and abs(other.index - self.index) < self.count:
            raise DslError("reduce of overlapping ranges")
        dstc = p.content[self.rank][self.buffer]
        srcc = p.content[other.rank][other.buffer]
        for k in range(self.count):
            dstc[self.index + k] = dstc[self.index + k] + srcc[other.index + k]
            p.version[self.rank][self.buffer][self.index + k] += 1
        p.ops.append(TraceOp("reduce", (other.rank, other.buffer, other.index, other.count),
                             (self.rank, self.buffer, self.index, self.count), ch, p._par, len(p.ops)))
        return Ref(self.rank, self.buffer, self.index, self.count)


def chunk(rank: int, buffer: str, index: int, count: int = 1) -> Ref:
    """Reference to the chunks currently at (rank, buffer, index .. index+count)."""
    return Ref(rank, buffer, index, count)


class parallelize:
    """`with parallelize(N):` - the operations inside are replaced by N instances, each on 1/N of the
    referenced range and on channels of its own (Section 5.1)."""

    def __init__(self, n: int):
        if n < 1:
            raise DslError("parallelize factor must be positive")
        self.n = n

    def __enter__(self):
        p = _prog()
        if p._par != 1:
            raise DslError("parallelize blocks cannot be nested")
        p._par = self.n
        return self

    def __exit__(self, exc_type, exc, tb):
        _prog()._par = 1
