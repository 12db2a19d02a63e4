"""Host-side logic of libgc3.so, no GPU needed: exports, IR loader, validator, planner."""
import os
import re

import pytest

import oracle
from paper_2201_11840_amd import binding as B
from paper_2201_11840_amd import programs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def load(text):
    return B.gc3_program_load(text)


def status_of(fn, *a):
    try:
        fn(*a)
        return B.GC3_OK
    except B.Gc3Error as e:
        return e.status


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "gc3.h")).read()
    declared = set(re.findall(r"^(?:int|void|const char\*)\s+(gc3_[a-z_]+)\s*\(", header, flags=re.M))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name


def generated():
    out = [programs.ring_allreduce(R, instances=k, fuse=f) for R in (2, 3, 8) for k in (1, 3) for f in (True, False)]
    out += [programs.ring_allreduce(5, use_rrs=True), programs.multichannel_ring_allreduce(5, 2),
            programs.allpairs_allreduce(4), programs.allpairs_allreduce(5, via_scratch=True),
            programs.direct_alltoall(1), programs.direct_alltoall(8),
            programs.ring_reduce_scatter(8, instances=8), programs.ring_allgather(5, instances=2)]
    out += [programs.hierarchical_allreduce(N, G) for N, G in ((2, 2), (2, 3), (3, 2), (2, 8), (3, 8))]
    out += [programs.alltonext(N, G) for N, G in ((1, 1), (1, 4), (4, 1), (3, 8))]
    out += [programs.twostep_alltoall(N, G) for N, G in ((1, 4), (4, 1), (2, 3), (3, 8))]
    out += [programs.local_stream(8), programs.local_stream(3, 2, reduce=True)]
    return out


@pytest.mark.parametrize("prog", generated(), ids=lambda p: f"{p.name}_{p.num_ops()}")
def test_loader_info_matches_the_generator(prog):
    h = load(prog.to_text())
    try:
        B.gc3_program_validate(h, 2)
        i = B.gc3_program_info_get(h)
        assert (i.ranks, i.in_chunks, i.out_chunks, i.inplace) == (prog.ranks, prog.in_chunks, prog.out_chunks, int(prog.inplace))
        assert i.num_tbs == prog.num_tbs() and i.num_instructions == prog.num_ops()
        assert i.algorithmic_chunks == prog.algorithmic_chunks() and i.max_count == prog.max_count()
        conns = {(r, t.send, t.chan) for r in range(prog.ranks) for t in prog.tbs[r]
                 if any(o.opcode in ("send", "rcs", "rrcs", "rrs") for o in t.ops)}
        assert i.num_connections == len(conns)
        for r in range(prog.ranks):
            assert B.gc3_program_scratch_chunks(h, r) == prog.scratch_chunks(r)
    finally:
        B.gc3_program_free(h)


@pytest.mark.parametrize("prog", generated(), ids=lambda p: f"{p.name}_{p.num_ops()}")
@pytest.mark.parametrize("slots", [1, 2, 8])
def test_validator_deadlock_verdict_matches_the_oracle(prog, slots):
    # two independent implementations of the bounded-FIFO execution must agree
    h = load(prog.to_text())
    try:
        st = status_of(B.gc3_program_validate, h, slots)
    finally:
        B.gc3_program_free(h)
    try:
        oracle.run_symbolic(oracle.parse_program(prog.to_text()), slots=slots, order="random", seed=slots)
        want = B.GC3_OK
    except oracle.OracleDeadlock:
        want = B.GC3_ERR_DEADLOCK
    assert st == want


GOOD = ("gc3ir 1\nname t\ncollective custom\ninplace 0\nprotocol simple\nranks 2\nchunks 2 2\n"
        "rank 0 scratch 1 tbs 1\ntb 0 send 1 recv 1 chan 0 ops 2\nop send i 0 - 0 1 0 0\nop recv - 0 o 1 1 0 0\n"
        "rank 1 scratch 0 tbs 1\ntb 0 send 0 recv 0 chan 0 ops 2\nop send i 1 - 0 1 0 0\nop recv - 0 o 0 1 0 0\nend\n")


def test_good_text_loads_and_comments_are_ignored():
    for text in (GOOD, "# leading comment\n" + GOOD.replace("ranks 2", "ranks 2   # two ranks"), GOOD.replace("\n", "\r\n")):
        h = load(text)
        B.gc3_program_validate(h, 1)
        B.gc3_program_free(h)


@pytest.mark.parametrize("mutate", [
    lambda t: t.replace("gc3ir 1", "gc3ir 2"),
    lambda t: t.replace("end\n", ""),
    lambda t: t.replace("op send i 0 - 0 1 0 0", "op fly i 0 - 0 1 0 0"),
    lambda t: t.replace("op send i 0 - 0 1 0 0", "op send q 0 - 0 1 0 0"),
    lambda t: t.replace("op send i 0 - 0 1 0 0", "op send i 0 - 0 1 0 1 0"),      # dependency list too short
    lambda t: t.replace("op send i 0 - 0 1 0 0", "op send i 0 - 0 0 0 0"),        # count 0
    lambda t: t.replace("ops 2\nop send i 0", "ops 3\nop send i 0", 1),            # fewer ops than declared
    lambda t: t.replace("rank 1 scratch", "rank 2 scratch"),
    lambda t: t.replace("tb 0 send 0 recv 0", "tb 1 send 0 recv 0"),
    lambda t: t.replace("ranks 2", "ranks two"),
    lambda t: t + "name again\n",
    lambda t: t.replace("chunks 2 2\n", ""),
    lambda t: "",
])
def test_malformed_text_is_a_parse_error(mutate):
    with pytest.raises(B.Gc3Error) as e:
        load(mutate(GOOD))
    assert e.value.status == B.GC3_ERR_PARSE


def two_rank(ops0, ops1, tbs0=None, scratch=0):
    def rank(r, tbs):
        out = f"rank {r} scratch {scratch} tbs {len(tbs)}\n"
        for b, (send, recv, chan, ops) in enumerate(tbs):
            out += f"tb {b} send {send} recv {recv} chan {chan} ops {len(ops)}\n" + "".join(o + "\n" for o in ops)
        return out
    t0 = tbs0 if tbs0 is not None else [(1, 1, 0, ops0)]
    return ("gc3ir 1\nname t\ncollective custom\ninplace 0\nprotocol simple\nranks 2\nchunks 2 2\n"
            + rank(0, t0) + rank(1, [(0, 0, 0, ops1)]) + "end\n")


SEND, RECV = "op send i 0 - 0 1 0 0", "op recv - 0 o 0 1 0 0"


@pytest.mark.parametrize("text,want", [
    (two_rank([SEND], [RECV]), B.GC3_OK),
    # two thread blocks sending on one connection
    (two_rank(None, [RECV, RECV], tbs0=[(1, -1, 0, [SEND]), (1, 1, 0, [SEND])]), B.GC3_ERR_INVALID_PROGRAM),
    # send / receive size mismatch
    (two_rank(["op send i 0 - 0 2 0 0"], [RECV]), B.GC3_ERR_INVALID_PROGRAM),
    # message never received / receive never fed
    (two_rank([SEND], []), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank([], [RECV]), B.GC3_ERR_INVALID_PROGRAM),
    # dependency on a step that does not exist, on a step without has-dependent flag, on itself
    (two_rank(None, [], tbs0=[(-1, -1, 0, ["op copy i 0 o 0 1 0 1 1 5"]), (-1, -1, 1, ["op copy i 1 o 1 1 1 0"])]), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank(None, [], tbs0=[(-1, -1, 0, ["op copy i 0 o 0 1 0 1 1 0"]), (-1, -1, 1, ["op copy i 1 o 1 1 0 0"])]), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank(None, [], tbs0=[(-1, -1, 0, ["op copy i 0 o 0 1 1 1 0 0"])]), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank(None, [], tbs0=[(-1, -1, 0, ["op copy i 0 o 0 1 0 1 1 0"]), (-1, -1, 1, ["op copy i 1 o 1 1 1 0"])]), B.GC3_OK),
    # chunk index outside the buffer; scratch not declared; missing operand
    (two_rank(["op send i 2 - 0 1 0 0"], [RECV]), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank(["op send i 1 - 0 2 0 0"], ["op recv - 0 o 0 2 0 0"]), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank(["op send s 0 - 0 1 0 0"], [RECV]), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank(["op send - 0 - 0 1 0 0"], [RECV]), B.GC3_ERR_INVALID_PROGRAM),
    # send without a send peer, a rank as its own peer, peer out of range
    (two_rank(None, [RECV], tbs0=[(-1, 1, 0, [SEND])]), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank(None, [RECV], tbs0=[(0, 1, 0, [SEND])]), B.GC3_ERR_INVALID_PROGRAM),
    (two_rank(None, [RECV], tbs0=[(7, 1, 0, [SEND])]), B.GC3_ERR_INVALID_PROGRAM),
    # cyclic wait: both receive first
    (two_rank([RECV, SEND], [RECV, SEND]), B.GC3_ERR_DEADLOCK),
    # cyclic dependency between two thread blocks of one rank
    (two_rank(None, [], tbs0=[(-1, -1, 0, ["op copy i 0 o 0 1 1 1 1 0"]), (-1, -1, 1, ["op copy i 1 o 1 1 1 1 0 0"])]), B.GC3_ERR_DEADLOCK),
    # three sends before the peer receives anything: fine with 2 slots only if the peer drains
    (two_rank([SEND, SEND, SEND, RECV], [SEND, RECV, RECV, RECV]), B.GC3_OK),
])
def test_validator_cases(text, want):
    h = load(text)
    try:
        assert status_of(B.gc3_program_validate, h, 2) == want, B.gc3_last_error()
    finally:
        B.gc3_program_free(h)


def test_outstanding_sends_beyond_the_slot_count_deadlock():
    # Section 6.1: a schedule with more than s outstanding sends deadlocks
    text = two_rank([SEND, SEND, SEND, RECV, RECV, RECV], [SEND, SEND, SEND, RECV, RECV, RECV])
    h = load(text)
    try:
        assert status_of(B.gc3_program_validate, h, 2) == B.GC3_ERR_DEADLOCK
        assert status_of(B.gc3_program_validate, h, 3) == B.GC3_OK
        assert status_of(B.gc3_program_validate, h, 0) == B.GC3_ERR_ARG
        assert status_of(B.gc3_program_validate, h, 9) == B.GC3_ERR_ARG
    finally:
        B.gc3_program_free(h)


# ---- planner ---------------------------------------------------------------------------------------

def plan(prog, cus=256, resident=1792, **kw):
    h = load(prog.to_text())
    try:
        return B.gc3_program_plan(h, B.make_config(**kw), cus, resident)
    finally:
        B.gc3_program_free(h)


def test_plan_fills_the_device_without_exceeding_it():
    for prog in generated():
        i = plan(prog)
        assert 1 <= i.team_width <= 64
        assert i.active_wgs <= 4 * 256 or i.team_width == 1
        assert i.grid == i.active_wgs == i.team_width * i.wgs_per_lane   # lane-major grid, no padding
        assert (1 <= i.max_fibers_per_wg <= 32) or prog.num_tbs() == 0
        assert i.slot_bytes == prog.max_count() * i.tile_bytes
    i = plan(programs.ring_allreduce(8, instances=8))
    assert (i.team_width, i.active_wgs, i.max_fibers_per_wg) == (16, 1024, 1)     # one lane per workgroup
    assert i.fifo_bytes == 64 * 16 * 2 * 65536 and i.tile_bytes == 65536
    i = plan(programs.hierarchical_allreduce(2, 8))
    assert i.max_fibers_per_wg >= 2 and i.active_wgs == 1024     # light phases share workgroups
    assert i.fifo_bytes <= 256 << 20 and i.tile_bytes < 65536   # tile shrunk to keep the FIFOs cache sized
    i = plan(programs.alltonext(3, 8))
    assert i.active_wgs <= 1024 and i.max_fibers_per_wg >= 2      # 396 thread blocks cannot each own 4 lanes
    # workgroups of one wavefront share nothing while thread blocks x lanes fits the target (each lane of each
    # thread block then runs on the wavefront-level interpreter), and share again beyond it
    n = programs.alltonext(3, 8).num_tbs()
    i = plan(programs.alltonext(3, 8), resident=7168, wg_size=64, team_width=10, target_wgs=4096)
    assert (i.team_width, i.active_wgs, i.max_fibers_per_wg) == (10, 10 * n, 1)
    i = plan(programs.alltonext(3, 8), resident=7168, wg_size=64, team_width=16, target_wgs=4096)
    assert i.active_wgs <= 4096 and i.max_fibers_per_wg >= 2
    i = plan(programs.hierarchical_allreduce(2, 8), resident=7168, wg_size=64, team_width=64, target_wgs=4096)
    assert (i.active_wgs, i.max_fibers_per_wg) == (4096, 1)
    i = plan(programs.hierarchical_allreduce(2, 8), resident=7168, wg_size=256, team_width=64, target_wgs=4096)
    assert i.max_fibers_per_wg >= 2                                # larger workgroups keep sharing


def test_plan_respects_configuration_and_limits():
    prog = programs.ring_allreduce(8, instances=8)
    i = plan(prog, team_width=4, tile_bytes=4096, fifo_slots=2, wg_size=512)
    assert (i.team_width, i.tile_bytes, i.fifo_slots, i.wg_size) == (4, 4096, 2, 512)
    assert i.active_wgs == 64 * 4 and i.fifo_bytes == 64 * 4 * 2 * 4096
    i = plan(prog, target_wgs=128)
    assert i.active_wgs <= 128
    small = plan(prog, cus=8, resident=16)                     # a tiny device: thread blocks must share
    assert small.active_wgs <= 16 and small.max_fibers_per_wg >= 4
    for bad in (dict(fifo_slots=9), dict(tile_bytes=24), dict(tile_bytes=2 << 20), dict(wg_size=100),
                dict(team_width=257), dict(target_wgs=-1), dict(min_lane_bytes=24), dict(debug_hold=2), dict(lds_stage=2),
                dict(fifo_scope=3), dict(fifo_scope=2, lds_stage=1), dict(fifo_scope=2, protocol=2)):
        with pytest.raises(B.Gc3Error) as e:
            plan(prog, **bad)
        assert e.value.status == B.GC3_ERR_ARG
    with pytest.raises(B.Gc3Error) as e:
        plan(programs.alltonext(3, 8), team_width=256)             # 24 ranks x 256 lanes cannot be resident
    assert e.value.status == B.GC3_ERR_RESIDENCY
    with pytest.raises(B.Gc3Error) as e:
        plan(programs.ring_allreduce(4), fifo_slots=1)             # fused ring needs two slots
    assert e.value.status == B.GC3_ERR_DEADLOCK


def test_head_stride_follows_the_slack_in_the_slots():
    # a receiver announces freed slots every head_stride-th message only when the program also completes with
    # fifo_slots - head_stride + 1 slots (what a sender can then count on, Section 6.1)
    ring = programs.ring_allreduce(4)
    assert [plan(ring, fifo_slots=s).head_stride for s in (2, 3, 4, 7, 8)] == [1, 1, 2, 2, 4]

    def both_send_first(k):
        class P:
            def to_text(self):
                return two_rank([SEND] * k + [RECV] * k, [SEND] * k + [RECV] * k)
        return P()
    # k messages are in flight before anything is received: needs k slots
    assert plan(both_send_first(5), fifo_slots=8).head_stride == 4      # 5 slots are enough
    assert plan(both_send_first(6), fifo_slots=8).head_stride == 1      # would deadlock with 5
    assert plan(both_send_first(3), fifo_slots=4).head_stride == 2
    assert plan(both_send_first(4), fifo_slots=4).head_stride == 1


def test_die_scope_user_buffers_place_the_ranks_on_dies():
    # user_scope 2: the bins of a lane are ordered row by row over the ranks (rounded up to a multiple of 8, empty
    # bins as padding), so that workgroup index mod 8 = rank mod 8 in the lane-major grid
    for prog, kw in [(programs.allpairs_allreduce(8), dict(wg_size=64, team_width=4)),
                     (programs.hierarchical_allreduce(2, 3), dict(team_width=2)),
                     (programs.hierarchical_allreduce(3, 8), dict()),
                     (programs.twostep_alltoall(2, 3), dict(wg_size=64, team_width=1, target_wgs=4096))]:
        dev, die = plan(prog, **kw), plan(prog, user_scope=2, **kw)
        assert (dev.user_scope, die.user_scope) == (1, 2)
        assert die.wgs_per_lane % 8 == 0 and die.wgs_per_lane >= dev.wgs_per_lane
        assert die.grid == die.wgs_per_lane * die.team_width
        assert die.team_width == dev.team_width and die.active_wgs == dev.active_wgs     # the same bins, placed
    # 8 ranks x 7 thread blocks with workgroups of their own: 7 rows of 8, nothing to pad
    assert plan(programs.allpairs_allreduce(8), user_scope=2, wg_size=64, team_width=4).wgs_per_lane == 56
    with pytest.raises(B.Gc3Error) as e:
        plan(programs.ring_allreduce(4), user_scope=3)
    assert e.value.status == B.GC3_ERR_ARG
    # together with die-scope FIFOs the lanes are placed on dies (bin-major launch), which serves both: no reordering
    both, fifo = plan(programs.allpairs_allreduce(8), user_scope=2, fifo_scope=2), plan(programs.allpairs_allreduce(8), fifo_scope=2)
    assert both.user_scope == 2 and (both.wgs_per_lane, both.grid, both.team_width) == (fifo.wgs_per_lane, fifo.grid, fifo.team_width)


def test_tune_rejects_bad_sizes_before_touching_a_device():
    prog = B.gc3_program_load(programs.ring_allreduce(4).to_text())
    for elems, dtype, status in [(0, B.GC3_F32, B.GC3_ERR_SIZE), (66, B.GC3_F32, B.GC3_ERR_SIZE),
                                 (8, B.GC3_F32, B.GC3_ERR_SIZE), (64, 99, B.GC3_ERR_ARG)]:
        with pytest.raises(B.Gc3Error) as e:
            B.gc3_comm_tune(prog, None, elems, dtype)
        assert e.value.status == status
    B.gc3_program_free(prog)


@pytest.mark.parametrize("R,k", [(4, 1), (8, 8), (5, 2)])
def test_ring_user_buffer_traffic_closed_form(R, k):
    # with perfectly cached FIFOs a fused in-place ring AllReduce still moves (3 - 2/R) x S per rank through the
    # user buffers: R-1 reads for sends/reductions, R-1 + ... ; in chunks of S/(R k): (3R - 2) k per rank
    p = programs.ring_allreduce(R, instances=k)
    assert p.algorithmic_chunks() - p.fifo_chunks() == R * (3 * R - 2) * k
    assert p.fifo_chunks() == R * k * 2 * (2 * R - 2)       # 2R-2 messages per thread block, written once and read once


def test_residency_rule_for_runs_of_different_communicators():
    """Which runs in flight a new run must wait for (Section 6.2: every grid in flight must be wholly resident).
    Pure host logic behind gc3_comm_run's per-device ledger."""
    plan = B.gc3_residency_plan
    cap = 1792
    assert plan([], 7, 1024, cap) == []
    assert plan([(1, 1024, cap)], 1, 1024, cap) == [0]                 # same stream: ordered by the stream
    assert plan([(1, 1024, cap)], 2, 1024, cap) == [1]                 # 1024 + 1024 > 1792 on two streams
    assert plan([(1, 768, cap)], 2, 1024, cap) == [0]                  # fits beside it
    assert plan([(1, 512, cap), (2, 512, cap)], 3, 1024, cap) == [1, 0]          # oldest first, only as many as needed
    assert plan([(1, 512, cap), (3, 512, cap), (2, 512, cap)], 3, 1024, cap) == [1, 0, 0]   # own stream does not count
    assert plan([(1, 1000, cap), (2, 1000, cap)], 3, 1792, cap) == [1, 1]        # a grid that fills the device waits for all
    # different workgroup sizes: shares of the device, not workgroup counts (64-thread groups: 5120 fit)
    assert plan([(1, 2560, 5120)], 2, 1024, cap) == [1]                # 0.5 + 0.571 > 1
    assert plan([(1, 2048, 5120)], 2, 1024, cap) == [0]                # 0.4 + 0.571 <= 1
    for bad in (([(1, -1, cap)], 2, 10, cap), ([], 2, 10, 0), ([], 2, -1, cap)):
        with pytest.raises(B.Gc3Error) as e:
            plan(*bad)
        assert e.value.status == B.GC3_ERR_ARG


def test_selector_argument_checks_without_a_device():
    sel = B.gc3_selector_create()
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_selector_run(sel, 1024, B.GC3_F32)          # nothing registered
    assert e.value.status == B.GC3_ERR_SIZE
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_selector_run(sel, 1024, 99)
    assert e.value.status == B.GC3_ERR_ARG
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_selector_add(sel, None, 0, 0)
    assert e.value.status == B.GC3_ERR_ARG
    B.gc3_selector_destroy(sel)


def test_kernel_resources_of_the_built_library():
    """The compiler's report for the library that was built: no instantiation of the interpreter may spill to
    scratch memory or fall under 6 waves per SIMD (6 workgroups of 256 threads per compute unit; the planner
    aims at 4), which is how a careless change to the kernel shows first."""
    import json
    from paper_2201_11840_amd import build
    path = os.path.splitext(build.LIB_PATH)[0] + ".resources.json"
    if not os.path.exists(path):
        pytest.skip("library was built without the resource report")
    kernels = [k for k in json.load(open(path)) if "gc3_interpreter" in k["name"]]
    # 3 data types x (no dependencies, user buffers at device scope, at die scope) x (simple, LL, LDS staging, die-scope
    # FIFOs; wavefront-level simple, LL and die-scope FIFOs)
    assert len(kernels) == 3 * 3 * 7
    for k in kernels:
        assert k["scratch_bytes"] == 0, k
        assert k["occupancy"] >= 6, k
        staged = k["lds_bytes"] > 16384               # the staging area is 16 KiB on top of the interpreter's state
        assert k["vgprs"] <= 80 and k["lds_bytes"] <= (32768 if staged else 16384), k
    assert sum(k["lds_bytes"] > 16384 for k in kernels) == 9
    wave = [k for k in kernels if "gc3_interpreter_wave" in k["name"]]
    assert len(wave) == 3 * 3 * 3 and all(k["lds_bytes"] <= 2048 for k in wave)


def test_compiler_command_line_writes_loadable_programs(tmp_path):
    from paper_2201_11840_amd import gc3c
    for argv in (["ring_allreduce", "--ranks", "4", "--instances", "2"], ["ring_allreduce", "--ranks", "4", "--hand"],
                 ["allpairs_allreduce", "--ranks", "5"], ["hierarchical_allreduce", "--nodes", "2", "--gpus", "3"],
                 ["direct_alltoall", "--ranks", "3", "--hand"], ["twostep_alltoall", "--nodes", "2", "--gpus", "2"],
                 ["alltonext", "--nodes", "2", "--gpus", "3"], ["ring_reduce_scatter", "--ranks", "4"],
                 ["ring_allgather", "--ranks", "3", "--instances", "2", "--hand"]):
        out = tmp_path / "p.gc3ir"
        assert gc3c.main(argv + ["-o", str(out)]) == 0
        prog = B.gc3_program_load(out.read_text())
        B.gc3_program_validate(prog, 2)
        B.gc3_program_free(prog)


def test_c_abi_example_is_built_and_rejects_bad_usage():
    # the stand-alone C++ program is compiled against include/gc3.h and linked with the library by build()
    import subprocess
    from paper_2201_11840_amd import build
    if not os.path.exists(build.EXAMPLE_BIN):
        pytest.skip("example was not built")
    res = subprocess.run([build.EXAMPLE_BIN], capture_output=True, text=True)
    assert res.returncode == 1 and "usage" in res.stderr


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header has to compile as C99 with nothing but the standard headers
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "gc3.h"\nint main(void) { gc3_comm_config c = {0}; gc3_tune_report r; (void)r; return c.fifo_slots + (int)sizeof(gc3_comm_info) * 0; }\n')
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I", os.path.join(root, "include"), str(src)],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr


def test_loader_validator_and_planner_survive_mutated_programs(tmp_path):
    """The host part of the library (no device code) built with AddressSanitizer and UBSan and fed 20000 randomly
    damaged programs: every outcome is fine except a crash or a sanitizer report."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2201_11840_amd", "csrc")
    exe = tmp_path / "fuzz_host"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-I", os.path.join(root, "include"), "-I", csrc, os.path.join(root, "tests", "fuzz_host.cpp"),
           os.path.join(csrc, "program.cpp"), os.path.join(csrc, "plan.cpp"), "-o", str(exe)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    files = []
    for i, prog in enumerate([programs.ring_allreduce(4, instances=2), programs.hierarchical_allreduce(2, 3),
                              programs.allpairs_allreduce(4, via_scratch=True), programs.twostep_alltoall(2, 2),
                              programs.alltonext(2, 3)]):
        f = tmp_path / f"seed{i}.gc3ir"
        f.write_text(prog.to_text())
        files.append(str(f))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", LD_PRELOAD="")
    res = subprocess.run([str(exe), "20000"] + files, capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout + res.stderr[-4000:]
