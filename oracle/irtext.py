"""Reader for the GC3-IR text form (oracle side; independent of the runtime's parser).

Content of the IR follows Section 5 ("GC3-IR": program -> GPU programs ->
thread blocks -> instruction lists; at most one send and one receive peer per
thread block, identified with a channel) and the instruction record of the
interpreter figure in Section 6.2 (opcode, source/destination buffer and chunk
offset, count, dependency pairs, has-dependent flag).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

OPCODES = ("send", "recv", "copy", "reduce", "rrc", "rcs", "rrcs", "rrs")


class IRError(ValueError):
    pass


@dataclass
class OInstr:
    opcode: str
    srcbuf: str
    srcidx: int
    dstbuf: str
    dstidx: int
    count: int
    hasdep: bool
    deps: List[Tuple[int, int]]


@dataclass
class OThreadBlock:
    send: int
    recv: int
    chan: int
    instrs: List[OInstr] = field(default_factory=list)


@dataclass
class OProgram:
    name: str = ""
    collective: str = ""
    inplace: bool = False
    protocol: str = ""
    ranks: int = 0
    in_chunks: int = 0
    out_chunks: int = 0
    scratch_chunks: List[int] = field(default_factory=list)
    tbs: List[List[OThreadBlock]] = field(default_factory=list)


def parse_program(text: str) -> OProgram:
    p = OProgram()
    cur_tbs = None
    cur_tb = None
    want_tbs = want_ops = 0
    ended = False
    for ln, raw in enumerate(text.splitlines(), 1):
        line = raw.split("#", 1)[0].split()
        if not line:
            continue
        if ended:
            raise IRError(f"line {ln}: text after end")
        key, a = line[0], line[1:]
        try:
            if key == "gc3ir":
                if a != ["1"]:
                    raise IRError(f"line {ln}: unsupported version")
            elif key == "name":
                p.name = a[0]
            elif key == "collective":
                p.collective = a[0]
            elif key == "inplace":
                p.inplace = bool(int(a[0]))
            elif key == "protocol":
                p.protocol = a[0]
            elif key == "ranks":
                p.ranks = int(a[0])
            elif key == "chunks":
                p.in_chunks, p.out_chunks = int(a[0]), int(a[1])
            elif key == "rank":
                if int(a[0]) != len(p.tbs) or a[1] != "scratch" or a[3] != "tbs":
                    raise IRError(f"line {ln}: bad rank statement")
                if cur_tbs is not None and (len(cur_tbs) != want_tbs or
                                            (cur_tb is not None and len(cur_tb.instrs) != want_ops)):
                    raise IRError(f"line {ln}: previous rank incomplete")
                p.scratch_chunks.append(int(a[2]))
                cur_tbs = []
                cur_tb = None
                p.tbs.append(cur_tbs)
                want_tbs = int(a[4])
            elif key == "tb":
                if cur_tbs is None or int(a[0]) != len(cur_tbs):
                    raise IRError(f"line {ln}: bad tb id")
                if cur_tb is not None and len(cur_tb.instrs) != want_ops:
                    raise IRError(f"line {ln}: previous tb incomplete")
                if a[1] != "send" or a[3] != "recv" or a[5] != "chan" or a[7] != "ops":
                    raise IRError(f"line {ln}: bad tb statement")
                cur_tb = OThreadBlock(int(a[2]), int(a[4]), int(a[6]))
                want_ops = int(a[8])
                cur_tbs.append(cur_tb)
            elif key == "op":
                if cur_tb is None:
                    raise IRError(f"line {ln}: op outside tb")
                if a[0] not in OPCODES:
                    raise IRError(f"line {ln}: unknown opcode {a[0]}")
                nd = int(a[7])
                if len(a) != 8 + 2 * nd:
                    raise IRError(f"line {ln}: bad dependency list")
                deps = [(int(a[8 + 2 * k]), int(a[9 + 2 * k])) for k in range(nd)]
                cur_tb.instrs.append(OInstr(a[0], a[1], int(a[2]), a[3], int(a[4]), int(a[5]),
                                            bool(int(a[6])), deps))
            elif key == "end":
                ended = True
            else:
                raise IRError(f"line {ln}: unknown statement {key}")
        except (IndexError, ValueError) as e:
            if isinstance(e, IRError):
                raise
            raise IRError(f"line {ln}: malformed statement") from e
    if not ended:
        raise IRError("missing end")
    if len(p.tbs) != p.ranks:
        raise IRError("rank count mismatch")
    if cur_tbs is not None and (len(cur_tbs) != want_tbs or
                                (cur_tb is not None and len(cur_tb.instrs) != want_ops)):
        raise IRError("last rank incomplete")
    return p
