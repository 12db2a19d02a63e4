"""CPU oracle for the GC3-IR interpreter.  TEST INFRASTRUCTURE ONLY.

A plain, slow, sequential interpreter of GC3-IR programs (Sections 4.2, 5 and 6
of the paper) plus the plain definitions of the collectives it is pinned to
(Section 3.2 postconditions; Sections 7.1, 7.3, 7.4).  It shares no code with
the HIP runtime and imports nothing from it.  Only the tests, the smoke check
and the benchmark's cpu_baseline leg may import this package; the product path
never does.

Parity status: every function here is pinned by a `-m "not gpu"` test
(tests/test_oracle_*.py).  The paper prints no numeric worked example, so
floating-point values are pinned through the collectives' definitions, exact
rational arithmetic for the 16-bit adds, and the fp32 summation error bound,
not through printed numbers.
"""
from .irtext import parse_program, IRError  # noqa: F401
from .interp import run_program, run_symbolic, OracleDeadlock, OracleError  # noqa: F401
from . import numeric, postcond  # noqa: F401
