"""Command line front end of the compiler: write the GC3-IR text of one of the paper's algorithms (written in
the DSL, compiled by compiler.py) or of a hand schedule to a file, for use through the C ABI.

    python -m paper_2201_11840_amd.gc3c ring_allreduce --ranks 8 --instances 8 -o ring.gc3ir
    python -m paper_2201_11840_amd.gc3c hierarchical_allreduce --nodes 2 --gpus 8 --hand -o hier.gc3ir
"""
from __future__ import annotations

import argparse
import sys

from . import dsl_programs, programs

ALGORITHMS = ("ring_allreduce", "allpairs_allreduce", "hierarchical_allreduce", "direct_alltoall",
              "twostep_alltoall", "alltonext", "ring_reduce_scatter", "ring_allgather")


def build(args) -> "programs.Program":
    src = programs if args.hand else dsl_programs
    fn = getattr(src, args.algorithm)
    if args.algorithm in ("ring_allreduce", "ring_reduce_scatter", "ring_allgather"):
        return fn(args.ranks, instances=args.instances)
    if args.algorithm in ("allpairs_allreduce", "direct_alltoall"):
        return fn(args.ranks)
    return fn(args.nodes, args.gpus)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("algorithm", choices=ALGORITHMS)
    ap.add_argument("--ranks", type=int, default=8)
    ap.add_argument("--instances", type=int, default=1, help="parallelize(N) of the whole program (Section 5.1)")
    ap.add_argument("--nodes", type=int, default=2)
    ap.add_argument("--gpus", type=int, default=8, help="ranks per node")
    ap.add_argument("--hand", action="store_true", help="the hand schedule of programs.py instead of the compiled DSL program")
    ap.add_argument("-o", "--output", default="-")
    args = ap.parse_args(argv)
    text = build(args).to_text()
    if args.output == "-":
        sys.stdout.write(text)
    else:
        with open(args.output, "w") as f:
            f.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
