"""Do the pins of tests/test_oracle_pins.py have teeth?  Each case plants ONE plausible mistake in a
private copy of the oracle's source (a dropped term, a wrong operand or index, a wrong queue
discipline, an off-by-one in a wait, a wrong rounding), swaps the copy in, and requires that at
least one of the pins fails.  Everything runs on the CPU; the real oracle is untouched and is
restored after every case.
"""
import importlib.util
import os
import sys

import numpy as np
import pytest

import oracle
import tests.test_oracle_pins as pins
from paper_2201_11840_amd import programs

ORACLE_DIR = os.path.dirname(os.path.abspath(oracle.__file__))


def _load_mutant(module: str, old: str, new: str):
    """A module object built from oracle/<module>.py with `old` replaced by `new` (exactly one place)."""
    path = os.path.join(ORACLE_DIR, module + ".py")
    src = open(path).read()
    assert src.count(old) == 1, f"mutation site not unique in {module}.py: {old!r} occurs {src.count(old)} times"
    name = f"oracle._mutant_{module}"
    spec = importlib.util.spec_from_loader(name, loader=None, origin=path)
    mod = importlib.util.module_from_spec(spec)
    mod.__package__ = "oracle"
    mod.__file__ = path
    sys.modules[name] = mod
    try:
        exec(compile(src.replace(old, new), path + "<mutant>", "exec"), mod.__dict__)
    finally:
        del sys.modules[name]
    return mod


def _pin_suite():
    """A cheap cross-section of the pins: symbolic postconditions, the walk-through, closed forms,
    exact integer AllReduce, bytewise AllToAll / AllToNext, invariance, slot-bound deadlock, fp error
    bound, 16-bit rounding."""
    for prog in (programs.ring_allreduce(4), programs.ring_allreduce(3, fuse=False), programs.ring_allreduce(4, use_rrs=True),
                 programs.hierarchical_allreduce(2, 3), programs.allpairs_allreduce(4),
                 programs.allpairs_allreduce(3, via_scratch=True),
                 programs.multichannel_ring_allreduce(4, 2), programs.direct_alltoall(4),
                 programs.twostep_alltoall(2, 3), programs.alltonext(2, 3)):
        pins.test_symbolic_postcondition(prog, 2, "round_robin")
        pins.test_symbolic_postcondition(prog, None, "random")
    pins.test_hierarchical_walkthrough_states()
    pins.test_ring_closed_forms(4)
    pins.test_parallelize_instances(4, 2)
    for dtype in ("f32", "bf16"):
        pins.test_allreduce_integer_values_exact(programs.ring_allreduce(4), dtype)
        pins.test_allreduce_integer_values_exact(programs.hierarchical_allreduce(2, 3), dtype)
        pins.test_allreduce_integer_values_exact(programs.allpairs_allreduce(4), dtype)
        pins.test_allreduce_integer_values_exact(programs.allpairs_allreduce(4, via_scratch=True), dtype)
    pins.test_alltoall_bytewise(5, "f16")
    pins.test_alltonext_bytewise(2, 2)
    pins.test_postcondition_definitions_by_hand()
    for prog in (programs.ring_reduce_scatter(4, instances=2), programs.ring_allgather(3, instances=2)):
        pins.test_symbolic_postcondition(prog, 2, "round_robin")
    pins.test_reducescatter_and_allgather_against_their_definitions(4, 2, "f32")
    pins.test_allreduce_fp32_error_bound_and_rank_agreement(programs.ring_allreduce(8, instances=2))
    pins.test_result_independent_of_order_slots_and_fusion("f32")
    pins.test_rrs_leaves_same_final_result()
    pins.test_fused_ring_needs_two_slots()
    pins.test_bad_programs_are_reported()
    pins.test_wrong_schedule_fails_postcondition()
    pins.test_16bit_add_is_correctly_rounded("bf16")
    pins.test_16bit_add_is_correctly_rounded("f16")
    pins.test_bf16_rounding_special_cases()


def test_pin_suite_passes_on_the_real_oracle():
    _pin_suite()


INTERP_MUTANTS = {
    "reduce drops the destination operand":
        ("val = store.add(store.read(r, ins.dstbuf, ins.dstidx, n), store.read(r, ins.srcbuf, ins.srcidx, n))",
         "val = store.add(store.read(r, ins.srcbuf, ins.srcidx, n), store.read(r, ins.srcbuf, ins.srcidx, n))"),
    "reduce writes the source instead of the destination":
        ("val = store.add(store.read(r, ins.dstbuf, ins.dstidx, n), store.read(r, ins.srcbuf, ins.srcidx, n))\n"
         "            store.write(r, ins.dstbuf, ins.dstidx, n, val)",
         "val = store.add(store.read(r, ins.dstbuf, ins.dstidx, n), store.read(r, ins.srcbuf, ins.srcidx, n))\n"
         "            store.write(r, ins.srcbuf, ins.srcidx, n, val)"),
    "fused receive-reduce drops the local operand":
        ("val = store.add(msg, store.read(r, ins.srcbuf, ins.srcidx, n))", "val = msg"),
    "fused receive-reduce drops the message":
        ("val = store.add(msg, store.read(r, ins.srcbuf, ins.srcidx, n))", "val = store.read(r, ins.srcbuf, ins.srcidx, n)"),
    "rrc / rrcs never store":
        ('            if op != "rrs":\n                store.write(r, ins.dstbuf, ins.dstidx, n, val)', "            pass"),
    "rcs forwards but does not store":
        ('        elif op == "rcs":\n            val = msg\n            store.write(r, ins.dstbuf, ins.dstidx, n, val)',
         '        elif op == "rcs":\n            val = msg'),
    "recv stores at the source index":
        ('        elif op == "recv":\n            val = msg\n            store.write(r, ins.dstbuf, ins.dstidx, n, val)',
         '        elif op == "recv":\n            val = msg\n            store.write(r, ins.dstbuf, ins.srcidx, n, val)'),
    "copy goes the wrong way":
        ('        elif op == "copy":\n            val = store.read(r, ins.srcbuf, ins.srcidx, n)\n            store.write(r, ins.dstbuf, ins.dstidx, n, val)',
         '        elif op == "copy":\n            val = store.read(r, ins.dstbuf, ins.dstidx, n)\n            store.write(r, ins.srcbuf, ins.srcidx, n, val)'),
    "send reads the chunk before the one named":
        ('        if op == "send":\n            val = store.read(r, ins.srcbuf, ins.srcidx, n)',
         '        if op == "send":\n            val = store.read(r, ins.srcbuf, max(ins.srcidx - 1, 0), n)'),
    "connections deliver last-in first-out":
        ("queues[(tb.recv, r, tb.chan)].popleft()", "queues[(tb.recv, r, tb.chan)].pop()"),
    "sends ignore the channel":
        ("q = queues.setdefault((r, tb.send, tb.chan), deque())", "q = queues.setdefault((r, tb.send, 0), deque())"),
    "receives listen to the send peer":
        ("mcount, mdepth, msg = queues[(tb.recv, r, tb.chan)].popleft()",
         "mcount, mdepth, msg = queues[(tb.send if tb.send >= 0 else tb.recv, r, tb.chan)].popleft()"),
    "a dependency is satisfied when its step starts, not when it is done":
        ("if pc[r][db] <= ds:", "if pc[r][db] < ds:"),
    "dependencies are ignored":
        ("if pc[r][db] <= ds:\n                return False", "if False:\n                return False"),
    "slot bound off by one":
        ("len(queues.get((r, tb.send, tb.chan), ())) >= slots", "len(queues.get((r, tb.send, tb.chan), ())) > slots"),
    "communication depth not advanced by a message":
        ("q.append((n, d + 1, val))", "q.append((n, d, val))"),
    "leftover messages go unnoticed":
        ("    if left:\n        raise OracleError", "    if False:\n        raise OracleError"),
    "deadlock goes unnoticed":
        ("    if remaining:\n        stuck =", "    if False:\n        stuck ="),
    "symbolic sum keeps only one operand":
        ("        return [x + y for x, y in zip(a, b)]", "        return [x for x, y in zip(a, b)]"),
}

NUMERIC_MUTANTS = {
    "bf16 narrowing truncates":
        ("rounded = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)",
         "rounded = (u >> np.uint32(16)).astype(np.uint16)"),
    "bf16 ties round away from zero":
        ("rounded = ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)",
         "rounded = ((u + np.uint32(0x8000)) >> np.uint32(16)).astype(np.uint16)"),
    "bf16 widening shifts by the wrong amount":
        ("return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)",
         "return (bits.astype(np.uint32) << np.uint32(15)).view(np.float32)"),
    "fp16 sum is formed in half precision twice":
        ("wide = a.astype(np.float32) + b.astype(np.float32)",
         "wide = (a + b).astype(np.float32) * np.float32(1 + 2.0 ** -11)"),
    "fp32 add subtracts":
        ("return np.add(a, b, dtype=np.float32)", "return np.subtract(a, b, dtype=np.float32)"),
}


POSTCOND_MUTANTS = {
    "allreduce postcondition forgets rank 0":
        ("row.append(Counter({(q, j): 1 for q in range(ranks)}))", "row.append(Counter({(q, j): 1 for q in range(1, ranks)}))"),
    "alltoall postcondition is not transposed":
        ("row.append(Counter({(src, r * per + k): 1}))", "row.append(Counter({(r, src * per + k): 1}))"),
    "alltonext postcondition shifts the wrong way":
        ("row.append(None if r == 0 else Counter({(r - 1, j): 1}))", "row.append(None if r == 0 else Counter({((r + 1) % ranks, j): 1}))"),
    "alltonext postcondition expects rank 0 to receive":
        ("row.append(None if r == 0 else Counter({(r - 1, j): 1}))", "row.append(Counter({((r - 1) % ranks, j): 1}))"),
    "reducescatter postcondition takes interleaved chunks":
        ("row.append(Counter({(q, r * out_chunks + j): 1 for q in range(ranks)}))", "row.append(Counter({(q, j * ranks + r): 1 for q in range(ranks)}))"),
    "allgather postcondition is rank-minor":
        ("row.append(Counter({(j // in_chunks, j % in_chunks): 1}))", "row.append(Counter({(j % ranks, j // ranks): 1}))"),
    "alltoall definition copies instead of transposing":
        ("o[j * ce:(j + 1) * ce] = inputs[j][i * ce:(i + 1) * ce]", "o[j * ce:(j + 1) * ce] = inputs[i][j * ce:(j + 1) * ce]"),
    "alltonext definition keeps the rank's own input":
        ("outs.append(inputs[i - 1].copy())", "outs.append(inputs[i].copy())"),
    "allreduce definition skips a rank":
        ("    for a in inputs:\n        acc += numeric.to_float64(a, dtype)", "    for a in inputs[1:]:\n        acc += numeric.to_float64(a, dtype)"),
    "reducescatter definition hands out the parts in reverse":
        ("return [total[r * part:(r + 1) * part].copy() for r in range(R)]", "return [total[(R - 1 - r) * part:(R - r) * part].copy() for r in range(R)]"),
    "allgather definition concatenates in reverse":
        ("cat = np.concatenate(list(inputs))", "cat = np.concatenate(list(inputs)[::-1])"),
}


IRTEXT_MUTANTS = {
    "parser swaps source and destination index":
        ("cur_tb.instrs.append(OInstr(a[0], a[1], int(a[2]), a[3], int(a[4]), int(a[5]),",
         "cur_tb.instrs.append(OInstr(a[0], a[1], int(a[4]), a[3], int(a[2]), int(a[5]),"),
    "parser swaps send and receive peer":
        ("cur_tb = OThreadBlock(int(a[2]), int(a[4]), int(a[6]))", "cur_tb = OThreadBlock(int(a[4]), int(a[2]), int(a[6]))"),
    "parser drops the channel":
        ("cur_tb = OThreadBlock(int(a[2]), int(a[4]), int(a[6]))", "cur_tb = OThreadBlock(int(a[2]), int(a[4]), 0)"),
    "parser reads a dependency as (step, thread block)":
        ("deps = [(int(a[8 + 2 * k]), int(a[9 + 2 * k])) for k in range(nd)]", "deps = [(int(a[9 + 2 * k]), int(a[8 + 2 * k])) for k in range(nd)]"),
    "parser ignores count":
        ("a[3], int(a[4]), int(a[5]),", "a[3], int(a[4]), 1,"),
    "parser swaps input and output chunk counts":
        ("p.in_chunks, p.out_chunks = int(a[0]), int(a[1])", "p.out_chunks, p.in_chunks = int(a[0]), int(a[1])"),
    "parser accepts text without end":
        ("    if not ended:\n        raise IRError(\"missing end\")\n", ""),
}


def _expect_caught(what):
    try:
        _pin_suite()
    except (AssertionError, oracle.OracleError, oracle.IRError, IndexError, KeyError, ValueError, TypeError,
            pytest.fail.Exception):        # the last one: a pin's `pytest.raises` saw no error
        return
    raise AssertionError(f"no pin noticed the planted mistake: {what}")


@pytest.mark.parametrize("what", sorted(INTERP_MUTANTS))
def test_interpreter_mistake_is_caught(what, monkeypatch):
    old, new = INTERP_MUTANTS[what]
    m = _load_mutant("interp", old, new)
    # the pins call oracle.run_program / oracle.run_symbolic; errors must stay of the real classes
    m.OracleError, m.OracleDeadlock = oracle.OracleError, oracle.OracleDeadlock
    monkeypatch.setattr(oracle, "run_program", m.run_program)
    monkeypatch.setattr(oracle, "run_symbolic", m.run_symbolic)
    _expect_caught(what)


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("what", sorted(NUMERIC_MUTANTS))
def test_numeric_mistake_is_caught(what, monkeypatch):
    old, new = NUMERIC_MUTANTS[what]
    m = _load_mutant("numeric", old, new)
    for fn in ("add", "f32_to_bf16_bits", "bf16_bits_to_f32", "to_float64"):
        monkeypatch.setattr(oracle.numeric, fn, getattr(m, fn))
    _expect_caught(what)


@pytest.mark.parametrize("what", sorted(POSTCOND_MUTANTS))
def test_postcondition_mistake_is_caught(what, monkeypatch):
    # a wrong definition of a collective makes correct programs (or the hand-written tiny cases) fail it
    old, new = POSTCOND_MUTANTS[what]
    m = _load_mutant("postcond", old, new)
    for fn in ("symbolic_expected", "check_symbolic", "allreduce_sum_f64", "alltoall_expected", "alltonext_expected",
               "reducescatter_sum_f64", "allgather_expected"):
        monkeypatch.setattr(oracle.postcond, fn, getattr(m, fn))
    _expect_caught(what)


@pytest.mark.parametrize("what", sorted(IRTEXT_MUTANTS))
def test_parser_mistake_is_caught(what, monkeypatch):
    old, new = IRTEXT_MUTANTS[what]
    m = _load_mutant("irtext", old, new)
    m.IRError = oracle.IRError
    monkeypatch.setattr(oracle, "parse_program", m.parse_program)
    monkeypatch.setattr(oracle.irtext, "parse_program", m.parse_program)
    _expect_caught(what)
