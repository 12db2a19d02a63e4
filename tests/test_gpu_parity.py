"""GPU parity: the HIP interpreter (through the C ABI) against the CPU oracle, element by element.

Tolerances: copy-only and integer-valued data bit-exact; fp32 bit-exact (the reduction order is the
program's); fp16 / bf16 within 1e-3 relative (+1e-5 of the largest magnitude as an absolute floor for
sums near zero) - and, because both sides perform one correctly rounded add per hop in the same
order, they are additionally expected to agree bitwise, which is asserted too.
"""
import numpy as np
import pytest

import oracle
from oracle import numeric, postcond
from paper_2201_11840_amd import inputs, programs, workloads

pytestmark = pytest.mark.gpu


def _harness():
    from paper_2201_11840_amd import harness
    return harness


def compare(got, want, dtype, exact_only=False):
    if dtype == "f32" or exact_only:
        ub = {2: np.uint16, 4: np.uint32}[got.dtype.itemsize]
        same = np.array_equal(got.view(ub), want.view(ub))
        assert same, f"{np.count_nonzero(got.view(ub) != want.view(ub))} of {got.size} elements differ"
        return
    g64, w64 = numeric.to_float64(got, dtype), numeric.to_float64(want, dtype)
    # locations the program never writes keep the NaN sentinel: they must match bitwise; the tolerance
    # applies to the finite values
    fin = np.isfinite(w64)
    assert np.array_equal(got[~fin].view(np.uint16), want[~fin].view(np.uint16))
    scale = np.abs(w64[fin]).max() if fin.any() else 0.0
    tol = 1e-3 * np.abs(w64[fin]) + 1e-5 * scale
    assert np.all(np.abs(g64[fin] - w64[fin]) <= tol), f"max err {np.abs(g64[fin] - w64[fin]).max()}"
    same = np.array_equal(got.view(np.uint16), want.view(np.uint16))
    assert same, f"within tolerance but {np.count_nonzero(got.view(np.uint16) != want.view(np.uint16))} elements not bitwise equal"


def compare_special(got, want, dtype, exact_only=False):
    """Inputs full of corner cases (subnormals, ties, overflow, signed zeros, infinities, NaNs): every result
    that is not a NaN must match the oracle bit for bit - no tolerance, so a flush to zero, a different
    rounding of a tie, a lost sign of zero or a missed overflow all fail.  Where the oracle's result is a NaN
    the GPU's must be a NaN too; sign and payload of a NaN produced by an addition are left open by IEEE 754
    and are not compared."""
    utype = np.uint32 if dtype == "f32" else np.uint16
    gb, wb = got.view(utype), want.view(utype)
    with np.errstate(invalid="ignore"):
        g64, w64 = numeric.to_float64(got, dtype), numeric.to_float64(want, dtype)
    nan = np.isnan(w64)
    assert np.all(np.isnan(g64[nan])), f"{np.count_nonzero(~np.isnan(g64[nan]))} results should be NaN and are not"
    bad = gb[~nan] != wb[~nan]
    assert not bad.any(), (f"{np.count_nonzero(bad)} of {bad.size} non-NaN results differ, first: got "
                           f"{gb[~nan][bad][0]:#x} want {wb[~nan][bad][0]:#x}")


def run_case(prog, dtype, elems, dist="normal", seed=1234, cfg=None, repeats=1, exact_only=False, compare=None,
             expect_kernel=None, expect_die=None):
    """Run `prog` on the GPU and in the oracle on the same seeded inputs; compare every output element
    of every rank (and the inputs of out-of-place programs, which most programs leave untouched).  With an explicit
    configuration both protocols (payload + flag, and LL) are exercised unless it fixes one."""
    compare = compare or globals()["compare"]
    H = _harness()
    text = prog.to_text()
    p = oracle.parse_program(text)
    ins = inputs.make_inputs(p.ranks, elems, dtype, dist, seed)
    out_elems = elems // p.in_chunks * p.out_chunks
    outs = None if p.inplace else inputs.sentinel_outputs(p.ranks, out_elems, dtype)
    want_in = [a.copy() for a in ins]
    want_out = None if p.inplace else [a.copy() for a in outs]
    with np.errstate(over="ignore", invalid="ignore"):
        oracle.run_program(p, want_in, want_out, dtype, slots=8)
    protocols = [None]
    if cfg is not None and cfg.protocol == 0 and cfg.fifo_scope != 2:
        protocols = [1, 2]
    for proto in protocols:
        if proto is not None:
            cfg.protocol = proto
        coll = H.Collective(text, dtype, elems, cfg)
        try:
            if expect_kernel is not None:                  # the kernel variant this case is meant to exercise
                assert coll.launch.kernel == expect_kernel, (prog.name, coll.launch.kernel)
            if expect_die is not None:
                assert bool(coll.launch.die_scope) == expect_die, prog.name
            for _ in range(repeats):
                coll.upload(ins, outs)
                coll.run()
                coll.status()
                got_out = coll.download("out")
                for r in range(p.ranks):
                    compare(got_out[r], (want_in if p.inplace else want_out)[r], dtype, exact_only)
                if not p.inplace:
                    got_in = coll.download("in")
                    for r in range(p.ranks):               # untouched, or changed exactly as the oracle's were
                        assert got_in[r].tobytes() == want_in[r].tobytes()
        finally:
            coll.close()
            if proto is not None:
                cfg.protocol = 0


def small_cfg(**kw):
    H = _harness()
    base = dict(fifo_slots=2, tile_bytes=1024, team_width=3, min_lane_bytes=16)   # every lane active even on tiny chunks
    base.update(kw)
    return H.make_config(**base)


# ---- the tiny-R grid, small tiles so that every run spans several tiles and a ragged tail ----------

@pytest.mark.parametrize("R", [2, 3, 4, 5, 8])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_ring_allreduce_grid(R, dtype):
    elems = R * 2500 * (1 if dtype == "f32" else 2)       # chunk = 10000 bytes: 3 lanes, ragged tiles
    run_case(programs.ring_allreduce(R), dtype, elems, "normal", 100 + R, small_cfg())
    run_case(programs.ring_allreduce(R, fuse=False), dtype, elems, "uniform", 200 + R, small_cfg(fifo_slots=1))
    run_case(programs.ring_allreduce(R, use_rrs=True), dtype, elems, "normal", 300 + R, small_cfg(team_width=1))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_allreduce_variants(dtype):
    m = 1 if dtype == "f32" else 2
    run_case(programs.ring_allreduce(4, instances=3), dtype, 12 * 1000 * m, "normal", 1, small_cfg())
    run_case(programs.multichannel_ring_allreduce(5, 3), dtype, 5 * 1000 * m, "normal", 2, small_cfg())
    run_case(programs.allpairs_allreduce(4), dtype, 4 * 1000 * m, "normal", 3, small_cfg())
    run_case(programs.allpairs_allreduce(8), dtype, 8 * 1000 * m, "uniform", 4, small_cfg(team_width=2))
    # the local `reduce` instruction: chunks land in scratch and a thread block without peers sums them
    run_case(programs.allpairs_allreduce(4, via_scratch=True), dtype, 4 * 1000 * m, "normal", 5, small_cfg())
    run_case(programs.allpairs_allreduce(8, via_scratch=True), dtype, 8 * 1000 * m, "uniform", 6, small_cfg(team_width=2))
    run_case(programs.allpairs_allreduce(8, via_scratch=True), dtype, 8 * 65536 * m, "uniform", 7)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_reducescatter_and_allgather(dtype):
    # the two ring helpers of Section 2 as collectives of their own (rrs chain ending in an rrc; copy + rcs chain)
    m = 1 if dtype == "f32" else 2
    for R, k in ((2, 1), (5, 2), (8, 8)):
        run_case(programs.ring_reduce_scatter(R, instances=k), dtype, R * k * 500 * m, "normal", 31, small_cfg())
        run_case(programs.ring_allgather(R, instances=k), dtype, k * 700 * m, "normal", 32, small_cfg(), exact_only=True)
    run_case(programs.ring_reduce_scatter(8, instances=8), dtype, (4 << 20) // inputs.ITEMSIZE[dtype], "uniform", 33)
    run_case(programs.ring_allgather(8, instances=8), dtype, (512 << 10) // inputs.ITEMSIZE[dtype], "uniform", 34, exact_only=True)
    from paper_2201_11840_amd import dsl_programs as D
    run_case(D.ring_reduce_scatter(4, instances=2), dtype, 8 * 600 * m, "normal", 35, small_cfg())
    run_case(D.ring_allgather(5, instances=2), dtype, 2 * 600 * m, "normal", 36, small_cfg(), exact_only=True)


@pytest.mark.parametrize("N,G", [(2, 2), (2, 3), (3, 2), (2, 8), (3, 8)])
def test_hierarchical_allreduce_grid(N, G):
    # cross-thread-block semaphores, count = N aggregated chunks
    run_case(programs.hierarchical_allreduce(N, G), "bf16", N * G * 2000, "normal", 41, small_cfg())
    run_case(programs.hierarchical_allreduce(N, G, fuse=False), "f32", N * G * 1000, "uniform", 42, small_cfg(team_width=2))


@pytest.mark.parametrize("R", [1, 2, 3, 8])
def test_direct_alltoall_grid(R):
    run_case(programs.direct_alltoall(R), "f16", R * 5000, "normal", 21, small_cfg(), exact_only=True)


@pytest.mark.parametrize("N,G", [(1, 4), (4, 1), (2, 3), (3, 8)])
def test_twostep_alltoall_and_alltonext_grid(N, G):
    # 3 x 8 has 216 / 396 thread blocks: keep the grid within what the device holds at once
    wide = 1 if N * G > 8 else 3
    run_case(programs.twostep_alltoall(N, G), "f16", N * G * 1000, "normal", 22, small_cfg(team_width=wide), exact_only=True)
    run_case(programs.alltonext(N, G), "f16", G * 5000, "normal", 51, small_cfg(team_width=min(wide, 2)), exact_only=True)


# ---- programs produced by the DSL compiler (different thread-block structure, cross-phase fusion) -----

def test_compiled_programs():
    from paper_2201_11840_amd import dsl_programs as D
    run_case(D.ring_allreduce(8, instances=2), "f32", 16 * 1252, "uniform", 81, small_cfg())
    run_case(D.ring_allreduce(5, fuse=False), "bf16", 5 * 2000, "normal", 82, small_cfg(fifo_slots=1))
    run_case(D.ring_allreduce(4, use_rrs=True), "f16", 4 * 2000, "normal", 83, small_cfg())
    run_case(D.hierarchical_allreduce(2, 8), "bf16", 32 * 1000, "normal", 84, small_cfg())
    run_case(D.hierarchical_allreduce(3, 2, intra_parallel=False), "f32", 6 * 1000, "uniform", 85, small_cfg(team_width=2))
    run_case(D.allpairs_allreduce(8), "f32", 8 * 1000, "uniform", 86, small_cfg(team_width=2))
    run_case(D.allpairs_allreduce(5, via_scratch=True), "bf16", 5 * 2000, "normal", 90, small_cfg())
    run_case(D.twostep_alltoall(2, 3), "f16", 6 * 1000, "normal", 87, small_cfg(), exact_only=True)
    run_case(D.alltonext(3, 8), "f16", 8 * 2000, "normal", 88, small_cfg(team_width=1), exact_only=True)
    # default configuration, 16 MiB per rank
    run_case(D.hierarchical_allreduce(2, 8), "bf16", 8 << 20, "normal", 89)


@pytest.mark.parametrize("seed", range(12))
def test_random_compiled_programs(seed):
    # random copy / reduce programs: many peers per rank, scratch use, dependencies in all directions
    from tests.test_compiler import _random_program
    from paper_2201_11840_amd.compiler import compile_program
    p = _random_program(100 + seed, 2 + seed % 4, 3 + seed % 3, 14 + seed % 11, use_channels=False)
    ir = compile_program(p, fuse=seed % 4 != 3)
    dtype = ("f32", "f16", "bf16")[seed % 3]
    # copies of uninitialised scratch never happen (the DSL rejects them), so every value is defined;
    # outputs start from the sentinel pattern on both sides
    run_case(ir, dtype, ir.in_chunks * (1000 if dtype == "f32" else 2000), "normal", 500 + seed,
             small_cfg(fifo_slots=8, team_width=1 + seed % 3), repeats=3)


@pytest.mark.parametrize("seed", range(16))
def test_random_launch_configurations(seed):
    """Results never depend on the tunables (Section 6.1: b and s are the protocol's business): random team
    width, slot count, tile, workgroup size, workgroup target and minimum lane size, on programs with shared
    workgroups, dependencies, aggregation and scratch, with chunk sizes that leave ragged tiles and lanes."""
    H = _harness()
    rng = np.random.Generator(np.random.PCG64(9000 + seed))
    progs = [programs.hierarchical_allreduce(2, 3), programs.hierarchical_allreduce(3, 2, fuse=False),
             programs.ring_allreduce(5, instances=2), programs.multichannel_ring_allreduce(4, 3),
             programs.allpairs_allreduce(4, via_scratch=True), programs.allpairs_allreduce(5),
             programs.twostep_alltoall(2, 3), programs.alltonext(2, 4), programs.ring_allreduce(6, use_rrs=True)]
    prog = progs[seed % len(progs)]
    dtype = ("f32", "f16", "bf16")[int(rng.integers(3))]
    cfg = H.make_config(fifo_slots=int(rng.integers(2, 9)), tile_bytes=int(rng.choice([256, 1024, 4096, 16384, 65536])),
                        team_width=int(rng.choice([1, 2, 3, 5, 8, 13, 32])), wg_size=int(rng.choice([64, 128, 256, 512])),
                        target_wgs=int(rng.choice([0, 16, 100, 512])), min_lane_bytes=int(rng.choice([16, 256, 4096, 8192])),
                        fifo_scope=int(rng.choice([0, 2])))
    cfg.user_scope = int(rng.choice([0, 2]))
    unit = 16 // inputs.ITEMSIZE[dtype]
    chunk_elems = int(rng.choice([1, 3, 17, 250, 1031, 4100])) * unit          # 16 B .. 64 KiB per chunk
    exact = prog.collective != "allreduce"
    run_case(prog, dtype, prog.in_chunks * chunk_elems, "normal", 700 + seed, cfg, repeats=2, exact_only=exact)


def test_many_ranks_and_thread_blocks():
    # up to 64 virtual ranks and 1106 thread blocks, default plans (workgroups multiplex up to 16 thread blocks)
    for prog, dt in [(programs.hierarchical_allreduce(4, 8), "bf16"), (programs.hierarchical_allreduce(8, 4), "f32"),
                     (programs.twostep_alltoall(4, 8), "f16"), (programs.alltonext(8, 8), "f16"),
                     (programs.ring_allreduce(32, instances=2), "f32"), (programs.allpairs_allreduce(16), "f32"),
                     (programs.allpairs_allreduce(16, via_scratch=True), "bf16"), (programs.direct_alltoall(32), "f16")]:
        exact = prog.collective in ("alltoall", "alltonext")
        run_case(prog, dt, prog.in_chunks * 4096 // inputs.ITEMSIZE[dt], "normal", 5, None, exact_only=exact)


def test_local_instructions_without_any_connection():
    # the streaming programs bench.py uses for its device-memory ceiling: copy and reduce only, no FIFO, no flag
    for dtype in ("f32", "bf16"):
        m = 4 // inputs.ITEMSIZE[dtype]
        run_case(programs.local_stream(3, 2), dtype, 2 * 2500 * m, "normal", 1500, small_cfg(), exact_only=True)
        run_case(programs.local_stream(3, 2, reduce=True), dtype, 4 * 2500 * m, "normal", 1501, small_cfg())
        run_case(programs.local_stream(8, 8), dtype, 8 * 50000 * m, "normal", 1502, exact_only=True)
        run_case(programs.local_stream(8, 8, reduce=True), dtype, 16 * 50000 * m, "uniform", 1503)


# ---- edge cases ------------------------------------------------------------------------------------

def test_instruction_lists_longer_than_the_workgroup_cache():
    # 252 instructions per thread block: more than a workgroup keeps on chip, so they are fetched from global memory
    run_case(programs.ring_allreduce(64, fuse=False), "f32", 64 * 260, "uniform", 71, small_cfg())
    run_case(programs.ring_allreduce(64, fuse=False), "bf16", 64 * 4096, "normal", 72)


@pytest.mark.parametrize("lanes_active", [1, 2, 3])
def test_idle_lanes_take_over_fibers(lanes_active):
    # chunks too small for all 8 lanes: the workgroups of the idle lanes run part of the fiber lists
    # (both protocols, programs whose workgroups hold several thread blocks, cross-thread-block dependencies)
    H = _harness()
    cfg = lambda: H.make_config(team_width=8, min_lane_bytes=4096, tile_bytes=2048, target_wgs=64)
    cb = 4096 * lanes_active + 1024                       # bytes per chunk
    run_case(programs.hierarchical_allreduce(2, 3), "f32", 6 * cb // 4, "uniform", 61, cfg())
    run_case(programs.allpairs_allreduce(4, via_scratch=True), "bf16", 4 * cb // 2, "normal", 62, cfg())
    run_case(programs.alltonext(2, 3), "f16", 3 * cb // 2, "normal", 63, cfg(), exact_only=True)
    run_case(programs.twostep_alltoall(2, 3), "f16", 6 * cb // 2, "normal", 64, cfg(), exact_only=True)


def test_smallest_chunk_and_more_lanes_than_units():
    # chunk = 16 bytes (one unit): lanes beyond the first own nothing and must stay consistent
    run_case(programs.ring_allreduce(4), "f32", 16, "int8", 5, small_cfg(team_width=4))
    run_case(programs.hierarchical_allreduce(2, 2), "f16", 4 * 8, "int8", 6, small_cfg(team_width=5))
    run_case(programs.direct_alltoall(3), "bf16", 3 * 8 * 3, "normal", 7, small_cfg(team_width=2), exact_only=True)


def test_empty_input_is_a_noop():
    H = _harness()
    coll = H.Collective(programs.ring_allreduce(4).to_text(), "f32", 0)
    coll.run()
    coll.status()
    coll.close()
    # AllToNext on a single rank has no thread block at all: nothing is launched, the output is untouched
    coll = H.Collective(programs.alltonext(1, 1).to_text(), "f16", 64)
    coll.fill_outputs_with_sentinel()
    coll.run()
    coll.status()
    assert set(np.unique(coll.download("out")[0].view(np.uint16))) == {inputs.SENTINEL16}
    coll.close()


def test_largest_tile_and_slot_settings():
    # tile_bytes at its maximum (1 MiB), 8 slots, 512-thread workgroups
    cfg = _harness().make_config(fifo_slots=8, tile_bytes=1 << 20, team_width=1, wg_size=512)
    run_case(programs.ring_allreduce(3), "f32", 3 * (3 << 18) + 3 * 4, "uniform", 8, cfg)   # chunk = 3 MiB + 16 B
    cfg = _harness().make_config(fifo_slots=8, tile_bytes=16, team_width=1, wg_size=64)
    run_case(programs.ring_allreduce(3), "f32", 3 * 100, "uniform", 9, cfg)                 # 25 tiles of one unit


@pytest.mark.parametrize("slots", [3, 4, 5, 8])
def test_sender_far_ahead_of_the_receiver(slots):
    # One rank streams 24 messages, the other takes them one by one (and reduces half of them): the sender runs
    # into the slot limit again and again and goes on only when the receiver announces freed slots - after every
    # message, or after every 2nd / 4th when the plan allows that (4 or more slots).  Both kernels, both protocols,
    # several tiles.  The last case needs every one of its slots (both ranks send 4 or 8 before they receive).
    from paper_2201_11840_amd.ir import Program
    n = 24
    p = Program(f"stream_{n}", "custom", 2, n, n, inplace=False)
    src = p.tb(0, send=1, recv=-1, chan=0)
    dst = p.tb(1, send=-1, recv=0, chan=0)
    for k in range(n):
        src.add("send", src=("i", k))
        if k % 2:
            dst.add("rrc", src=("i", k), dst=("o", k))
        else:
            dst.add("recv", dst=("o", k))
    H = _harness()
    for wg in (64, 256):
        cfg = H.make_config(fifo_slots=slots, tile_bytes=1024, team_width=2, min_lane_bytes=16, wg_size=wg)
        run_case(p, "f32", n * (3 * 256 + 4), "uniform", 40 + slots, cfg)
    if slots in (4, 8):
        q = Program(f"exchange_{slots}", "custom", 2, slots, slots, inplace=False)
        for r in (0, 1):
            tb = q.tb(r, send=1 - r, recv=1 - r, chan=0)
            for k in range(slots):
                tb.add("send", src=("i", k))
            for k in range(slots):
                tb.add("recv", dst=("o", k))
        cfg = H.make_config(fifo_slots=slots, tile_bytes=1024, team_width=2, min_lane_bytes=16, wg_size=64)
        run_case(q, "f16", slots * (2 * 512 + 8), "normal", 50 + slots, cfg)


def test_repeated_runs_and_changing_sizes_on_one_communicator():
    # flags and semaphores only grow: a second and third run reuse them without clearing
    H = _harness()
    prog = programs.hierarchical_allreduce(2, 3)
    text = prog.to_text()
    p = oracle.parse_program(text)
    # (the second and third configuration use 3, 1, 8, 1, 8 of their 8 lanes in turn: lanes that sat out runs have
    # completed fewer of them than the others, under die-scope user buffers and die-scope FIFOs as well)
    for cfg in (small_cfg(), H.make_config(user_scope=2, team_width=8, min_lane_bytes=4096, tile_bytes=2048),
                H.make_config(fifo_scope=2, team_width=8, min_lane_bytes=4096, tile_bytes=2048)):
        coll = H.Collective(text, "f32", 6 * 12000, cfg)
        for elems in (6 * 4000, 6 * 40, 6 * 12000, 6 * 4, 6 * 12000):
            coll.resize(elems)
            ins = inputs.make_inputs(6, elems, "f32", "uniform", elems)
            want = [a.copy() for a in ins]
            oracle.run_program(p, want, None, "f32", slots=2)
            for _ in range(3):
                coll.upload(ins)
                coll.run()
                coll.status()
                for g, w in zip(coll.download(), want):
                    assert g.tobytes() == w.tobytes()
        coll.close()
    run_case(prog, "f32", 6 * 4000, "uniform", 77, small_cfg(), repeats=4)


@pytest.mark.parametrize("prog", [programs.ring_allreduce(8, instances=8), programs.hierarchical_allreduce(2, 8),
                                  programs.alltonext(3, 8)], ids=lambda p: p.name)
def test_fresh_data_every_run_on_one_communicator(prog):
    # FIFO slots are reused run after run: a receiver that saw an old copy of a slot would return
    # the previous run's data, so every run gets different inputs
    H = _harness()
    text = prog.to_text()
    p = oracle.parse_program(text)
    elems = p.in_chunks * 8192
    coll = H.Collective(text, "f32", elems)
    try:
        for it in range(6):
            ins = inputs.make_inputs(p.ranks, elems, "f32", "uniform", 9000 + 100 * it)
            outs = None if p.inplace else inputs.sentinel_outputs(p.ranks, elems // p.in_chunks * p.out_chunks, "f32")
            want_in = [a.copy() for a in ins]
            want_out = None if p.inplace else [a.copy() for a in outs]
            oracle.run_program(p, want_in, want_out, "f32", slots=coll.info.fifo_slots)
            coll.upload(ins, outs)
            coll.run()
            coll.status()
            for g, w in zip(coll.download("out"), want_in if p.inplace else want_out):
                assert g.tobytes() == w.tobytes(), f"run {it}"
    finally:
        coll.close()


def test_api_errors_without_launch():
    H = _harness()
    from paper_2201_11840_amd import binding as B
    coll = H.Collective(programs.ring_allreduce(4).to_text(), "f32", 64)
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_comm_run(coll.comm, 66, B.GC3_F32)          # not a multiple of the chunk count
    assert e.value.status == B.GC3_ERR_SIZE
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_comm_run(coll.comm, 4 * 2, B.GC3_F32)       # chunk of 8 bytes: not a 16-byte unit
    assert e.value.status == B.GC3_ERR_SIZE
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_comm_bind(coll.comm, 0, coll.inputs[0].data_ptr(), coll.inputs[1].data_ptr(), None, 0)
    assert e.value.status == B.GC3_ERR_ARG                # in-place program with a different output
    coll.close()
    prog = B.gc3_program_load(programs.direct_alltoall(2).to_text())
    comm = B.gc3_comm_create(prog)
    B.gc3_program_free(prog)
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_comm_run(comm, 64, B.GC3_F16)
    assert e.value.status == B.GC3_ERR_UNBOUND
    B.gc3_comm_destroy(comm)
    # a program that cannot be resident: 24 ranks x 256 lanes
    prog = B.gc3_program_load(programs.alltonext(3, 8).to_text())
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_comm_create(prog, H.make_config(team_width=256, wg_size=512))
    assert e.value.status == B.GC3_ERR_RESIDENCY
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_comm_create(prog, H.make_config(fifo_slots=9))
    assert e.value.status == B.GC3_ERR_ARG
    B.gc3_program_free(prog)
    prog = B.gc3_program_load(programs.ring_allreduce(4).to_text())
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_comm_create(prog, H.make_config(fifo_slots=1))     # fused ring needs two slots
    assert e.value.status == B.GC3_ERR_DEADLOCK
    B.gc3_program_free(prog)


def test_timeout_poisons_and_reset_recovers():
    # every workgroup waits (bounded by spin_limit_us) for a start word the host never sets: the run is
    # abandoned through the kernel's error path, all workgroups exit, the communicator is poisoned
    H = _harness()
    from paper_2201_11840_amd import binding as B
    prog = programs.hierarchical_allreduce(2, 3)
    text = prog.to_text()
    elems = 6 * 4096
    ins = inputs.make_inputs(6, elems, "f32", "uniform", 5)
    coll = H.Collective(text, "f32", elems, H.make_config(spin_limit_us=20000, debug_hold=1))
    coll.upload(ins)
    for _ in range(2):
        coll.run()
        with pytest.raises(B.Gc3Error) as e:
            coll.status()
        assert e.value.status == B.GC3_ERR_TIMEOUT
        with pytest.raises(B.Gc3Error) as e:
            coll.run()
        assert e.value.status == B.GC3_ERR_POISONED
        coll.reset()
    for g, a in zip(coll.download(), ins):
        assert g.tobytes() == a.tobytes()                    # nothing was moved
    coll.close()
    # the same buffers' contents through a normal communicator afterwards
    run_case(prog, "f32", elems, "uniform", 5, small_cfg())


def test_reset_restarts_the_ll_message_numbers():
    """The LL flags count on from run to run in device memory; gc3_comm_reset starts them again, so it must also wipe
    the LL slots: the first run after a reset expects exactly the flags the very first run left there, and would
    otherwise take that run's payload for its own."""
    H = _harness()
    for cfg in (dict(wg_size=64), dict(team_width=2, target_wgs=16)):       # wavefront-level and general kernel
        prog = programs.hierarchical_allreduce(2, 3)
        text = prog.to_text()
        p = oracle.parse_program(text)
        elems = 6 * 2048
        coll = H.Collective(text, "f32", elems, H.make_config(protocol=2, **cfg))
        try:
            for seed in (61, 62, 63):
                ins = inputs.make_inputs(6, elems, "f32", "normal", seed)
                want = [a.copy() for a in ins]
                oracle.run_program(p, want, None, "f32", slots=2)
                coll.upload(ins)
                coll.run()
                coll.status()
                for g, w_ in zip(coll.download(), want):
                    compare(g, w_, "f32")
                if seed != 62:
                    coll.reset()
        finally:
            coll.close()


def test_tune_measures_plans_and_the_chosen_one_is_correct():
    H = _harness()
    from paper_2201_11840_amd import binding as B
    for prog, dtype, elems in [(programs.ring_allreduce(8, instances=2), "f32", 16 * 8192),
                               (programs.hierarchical_allreduce(2, 3), "bf16", 6 * 16384),
                               (programs.alltonext(2, 3), "f16", 3 * 8192),
                               (programs.allpairs_allreduce(8), "f32", 8 * 8192)]:
        text = prog.to_text()
        p = oracle.parse_program(text)
        ins = inputs.make_inputs(p.ranks, elems, dtype, "normal", 77)
        outs = None if p.inplace else inputs.sentinel_outputs(p.ranks, elems // p.in_chunks * p.out_chunks, dtype)
        want_in = [a.copy() for a in ins]
        want_out = None if p.inplace else [a.copy() for a in outs]
        oracle.run_program(p, want_in, want_out, dtype, slots=8)
        coll = H.Collective(text, dtype, elems, tune=True)
        rep = coll.tune_report
        assert 2 <= rep.count <= B.GC3_TUNE_MAX_TRIED and 0 <= rep.best < rep.count
        tried = [rep.tried[i] for i in range(rep.count)]
        assert all(t.ms > 0 and t.grid >= t.active_wgs > 0 for t in tried)
        fastest = min(t.ms for t in tried)
        if rep.best == 0:                      # the default plan stays unless beaten by more than 2 %
            assert fastest >= 0.98 * tried[0].ms
        else:
            assert tried[rep.best].ms == fastest < 0.98 * tried[0].ms
        assert len({(t.team_width, t.grid, t.tile_bytes, t.wg_size, t.fifo_scope, t.protocol, t.min_lane_bytes, t.fifo_slots, t.user_scope)
                    for t in tried}) == rep.count   # no plan timed twice
        b = tried[rep.best]
        assert (coll.info.team_width, coll.info.grid, coll.info.tile_bytes, coll.info.wg_size) == \
            (b.team_width, b.grid, b.tile_bytes, b.wg_size)
        assert coll.cfg.fifo_scope == (2 if b.fifo_scope == 2 else 0)
        assert coll.info.protocol == b.protocol and coll.info.user_scope == b.user_scope
        coll.upload(ins, outs)
        coll.run()
        coll.status()
        for g, w in zip(coll.download("out"), want_in if p.inplace else want_out):
            compare(g, w, dtype)
        coll.close()
    # fields the caller fixes are not varied
    prog = B.gc3_program_load(programs.ring_allreduce(4).to_text())
    best, rep = B.gc3_comm_tune(prog, H.make_config(team_width=8, tile_bytes=4096), 4 * 4096, B.GC3_F32)
    assert best.team_width == 8 and best.tile_bytes == 4096
    assert all(rep.tried[i].team_width == 8 for i in range(rep.count))
    # a tuning run that fails ends the tuning with that error (forced from the host: no workgroup starts work)
    with pytest.raises(B.Gc3Error) as e:
        B.gc3_comm_tune(prog, H.make_config(spin_limit_us=20000, debug_hold=1), 4 * 4096, B.GC3_F32)
    assert e.value.status == B.GC3_ERR_TIMEOUT
    B.gc3_program_free(prog)


# ---- the benchmark configurations, default launch configuration -------------------------------------

def test_headline_under_every_plan_the_tuner_may_choose():
    # bench.py times the plan gc3_comm_tune picks; whichever it is, it is one of these
    H = _harness()
    w = workloads.ring_ar_r8x8(64)
    prog = w.build()
    text = prog.to_text()
    p = oracle.parse_program(text)
    ce = w.elems_per_rank // p.in_chunks
    ins = inputs.make_inputs(p.ranks, w.elems_per_rank, w.dtype, w.dist, w.seed)
    rng = np.random.Generator(np.random.PCG64(9))
    pos = np.unique(np.concatenate([rng.integers(0, ce, 20000), np.array([0, 1, ce - 2, ce - 1])]))
    for k in (1, 2, 3, 5, 7, 63):                       # lane boundaries of every width
        for W in (4, 8, 12, 16, 32, 64):
            b = min(((ce * 4 // W + 255) // 256 * 256 // 4) * k, ce - 1)
            pos = np.union1d(pos, np.clip(np.array([b - 1, b, b + 1]), 0, ce - 1))
    gather = lambda a: a.reshape(p.in_chunks, ce)[:, pos].reshape(-1).copy()
    want = [gather(a) for a in ins]
    oracle.run_program(p, want, None, w.dtype, slots=2)
    seen = set()
    candidates = [dict(team_width=W, target_wgs=tgt) for W in (0, 4, 8, 16, 32, 64) for tgt in (0, 512, 768)]
    # the tuner's later passes: slot tile and workgroup size of the winner
    candidates += [dict(tile_bytes=16384), dict(tile_bytes=32768), dict(wg_size=128),
                   dict(target_wgs=512, tile_bytes=32768), dict(target_wgs=512, wg_size=128),
                   dict(team_width=32, tile_bytes=16384, wg_size=128)]
    for kw in candidates:
        if True:
            coll = H.Collective(text, w.dtype, w.elems_per_rank, H.make_config(**kw))
            try:
                key = (coll.info.team_width, coll.info.grid, coll.info.tile_bytes, coll.info.wg_size)
                if key in seen:
                    continue
                seen.add(key)
                coll.upload(ins)
                coll.run()
                coll.status()
                got = coll.download("out")
            finally:
                coll.close()
            for r in range(p.ranks):
                assert gather(got[r]).tobytes() == want[r].tobytes(), f"plan {key} rank {r}"
                assert got[r].tobytes() == got[0].tobytes()
    assert len(seen) >= 14


def test_config1_ring_allreduce_r4():
    w = workloads.ring_ar_r4()
    run_case(w.build(), w.dtype, w.elems_per_rank, w.dist, w.seed, exact_only=True)
    run_case(programs.ring_allreduce(4, fuse=False), w.dtype, w.elems_per_rank, w.dist, w.seed, exact_only=True)
    # integer-valued data: also equal to the plain sum over ranks
    ins = inputs.make_inputs(4, w.elems_per_rank, "f32", "int8", w.seed)
    H = _harness()
    coll = H.Collective(w.build().to_text(), "f32", w.elems_per_rank)
    coll.upload(ins)
    coll.run()
    coll.status()
    want = postcond.allreduce_sum_f64(ins, "f32")
    for g in coll.download():
        assert np.array_equal(g.astype(np.float64), want)
    coll.close()


def test_config2_direct_alltoall_r8():
    w = workloads.direct_a2a_r8()
    run_case(w.build(), w.dtype, w.elems_per_rank, w.dist, w.seed, exact_only=True)


@pytest.mark.parametrize("mib", [1, 16, 64])
def test_config3_ring_allreduce_r8_x8(mib):
    w = workloads.ring_ar_r8x8(mib)
    run_case(w.build(), w.dtype, w.elems_per_rank, w.dist, w.seed)


def _full_size_case(w, tune=False):
    """A benchmark configuration at its stated size, default launch configuration (or, with `tune`, the plan
    gc3_comm_tune picks, as bench.py runs it), EVERY element of every rank against the oracle.  Host copies are
    dropped as soon as they have been compared."""
    H = _harness()
    prog = w.build()
    text = prog.to_text()
    p = oracle.parse_program(text)
    assert p.inplace
    ins = inputs.make_inputs(p.ranks, w.elems_per_rank, w.dtype, w.dist, w.seed)
    coll = H.Collective(text, w.dtype, w.elems_per_rank, tune=tune)
    try:
        coll.upload(ins)
        coll.run()
        coll.status()
        oracle.run_program(p, ins, None, w.dtype, slots=coll.info.fifo_slots)     # in place: `ins` now holds the results
        st = inputs.STORAGE[w.dtype]
        for r in range(p.ranks):
            got = coll.inputs[r][:coll.in_bytes].cpu().numpy().view(st)
            compare(got, ins[r], w.dtype)
            ins[r] = None
            del got
    finally:
        coll.close()


def test_config3_ring_allreduce_r8_x8_256MiB():
    _full_size_case(workloads.ring_ar_r8x8(256))


def test_config4_hierarchical_allreduce_2x8():
    run_case(workloads.hier_ar_2x8(4).build(), "bf16", workloads.hier_ar_2x8(4).elems_per_rank, "normal", 41840)
    _full_size_case(workloads.hier_ar_2x8(64))


def test_tuned_plans_at_the_stated_sizes():
    """The plans the tuner picks for the benchmark's workloads are unlike the default one (die-scope FIFOs, one
    wavefront per thread-block lane, 128 lanes, LL): the same full compare under them."""
    table = workloads.by_name()
    for name in ("ring_allreduce_r8_x8_f32_64MiB", "hier_allreduce_2x8_bf16_64MiB", "allpairs_allreduce_r8_f32_64MiB",
                 "ring_allreduce_rrs_r8_x8_f32_64MiB", "ring_allreduce_r8_x8_f32_1MiB", "ring_allreduce_r4_f32_64KiB",
                 "mc_ring_allreduce_r8_c4_f32_256KiB", "allpairs_allreduce_r8_f32_256KiB"):
        _full_size_case(table[name], tune=True)
    test_config5_alltonext_3x8(tune=True)


def test_config5_alltonext_3x8(tune=False):
    w = workloads.alltonext_3x8()
    H = _harness()
    prog = w.build()
    ins = inputs.make_inputs(24, w.elems_per_rank, w.dtype, w.dist, w.seed)
    coll = H.Collective(prog.to_text(), w.dtype, w.elems_per_rank, tune=tune)
    try:
        coll.fill_outputs_with_sentinel()
        coll.upload(ins)
        coll.run()
        coll.status()
        got = coll.download("out")
    finally:
        coll.close()
    assert set(np.unique(got[0].view(np.uint16))) == {inputs.SENTINEL16}       # rank 0 receives nothing
    for r in range(1, 24):
        assert got[r].tobytes() == ins[r - 1].tobytes()                      # out[i+1] == in[i], bytewise
    if tune:
        return
    # the oracle on a smaller buffer of the same program, element by element
    run_case(prog, w.dtype, 8 * 65536, w.dist, w.seed, exact_only=True)


# ---- every opcode on its own: smallest program in which its effect is visible ---------------------------

def _opcode_program(opcode, count):
    """Three ranks, 2*count input / output chunks, scratch where needed.  Rank 0 feeds, rank 1 runs the
    instruction under test, rank 2 drains what rank 1 forwards."""
    from paper_2201_11840_amd.ir import Program
    C = 2 * count
    p = Program(f"op_{opcode}_x{count}", "custom", 3, C, C, inplace=False)
    feed = p.tb(0, send=1, recv=-1, chan=0)
    mid = p.tb(1, send=2, recv=0, chan=0)
    drain = p.tb(2, send=-1, recv=1, chan=0)
    hi = ("i", count)                      # second half of the input
    if opcode in ("send", "recv"):
        feed.add("send", src=hi, count=count)
        mid.add("recv", dst=("o", 0), count=count)
    elif opcode == "copy":
        p.tb(1, chan=1).add("copy", src=hi, dst=("o", 0), count=count)
        p.tb(1, chan=1).add("copy", src=("o", 0), dst=("s", 1), count=count)
        p.tb(1, chan=1).add("copy", src=("s", 1), dst=("o", count), count=count)
    elif opcode == "reduce":
        t = p.tb(1, chan=1)
        t.add("copy", src=("i", 0), dst=("o", 0), count=count)
        t.add("reduce", src=hi, dst=("o", 0), count=count)
    else:
        feed.add("send", src=("i", 0), count=count)
        if opcode == "rrc":
            mid.add("rrc", src=hi, dst=("o", 0), count=count)
        elif opcode == "rcs":
            mid.add("rcs", dst=("o", count), count=count)
        elif opcode == "rrcs":
            mid.add("rrcs", src=hi, dst=("o", 0), count=count)
        elif opcode == "rrs":
            mid.add("rrs", src=hi, count=count)
        if opcode != "rrc":
            drain.add("recv", dst=("o", 0), count=count)
    return p


@pytest.mark.parametrize("opcode", ["send", "copy", "reduce", "rrc", "rcs", "rrcs", "rrs"])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_single_opcode(opcode, dtype):
    for count in (1, 3):
        prog = _opcode_program(opcode, count)
        es = inputs.ITEMSIZE[dtype]
        for chunk_bytes in (16, 4096 + 16, 3 * 1024 + 48, 70000 // 16 * 16):
            elems = 2 * count * chunk_bytes // es
            run_case(prog, dtype, elems, "normal", 300 + count, small_cfg())
        run_case(prog, dtype, 2 * count * (1 << 18) // es, "uniform", 310 + count)       # default plan, 256 KiB chunks


# ---- the corner cases of floating-point addition through every reducing instruction ------------------------

def _special_stats(prog, dtype, elems, seed):
    """What the oracle's results on the special inputs contain, to show that the cases are really met."""
    p = oracle.parse_program(prog.to_text())
    ins = inputs.make_inputs(p.ranks, elems, dtype, "special", seed)
    outs = None if p.inplace else inputs.sentinel_outputs(p.ranks, elems // p.in_chunks * p.out_chunks, dtype)
    with np.errstate(over="ignore", invalid="ignore"):
        oracle.run_program(p, ins, outs, dtype, slots=8)
        res = np.concatenate([numeric.to_float64(a, dtype) for a in (ins if p.inplace else outs)])
    _, ebits, _ = inputs.FORMAT[dtype]
    smallest_normal = 2.0 ** (2 - (1 << (ebits - 1)))
    return {"subnormal": int(np.count_nonzero((np.abs(res) < smallest_normal) & (res != 0))),
            "inf": int(np.count_nonzero(np.isinf(res))), "nan": int(np.count_nonzero(np.isnan(res))),
            "neg_zero": int(np.count_nonzero((res == 0) & np.signbit(res)))}


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("opcode", ["reduce", "rrc", "rrcs", "rrs"])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_special_values_single_opcode(opcode, dtype):
    # Section 4.2's reducing instructions on subnormals, ties, overflow, signed zeros, infinities and NaNs:
    # bitwise against the oracle for everything that is not a NaN (a flush-to-zero mode, a rounding other than
    # nearest-even or a packed add that treats a corner differently would show here and nowhere else)
    es = inputs.ITEMSIZE[dtype]
    for count, chunk_bytes, cfg in ((1, 96 * 1024 + 16, None), (2, 9 * 1024 + 48, small_cfg()), (1, 64 * 1024, small_cfg(wg_size=64))):
        prog = _opcode_program(opcode, count)
        elems = 2 * count * chunk_bytes // es
        st = _special_stats(prog, dtype, elems, 900 + count)
        assert min(st.values()) > 0, st
        run_case(prog, dtype, elems, "special", 900 + count, cfg, compare=compare_special)


@pytest.mark.filterwarnings("ignore::RuntimeWarning")
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_special_values_multi_hop(dtype):
    # several additions in a row (a ring of 4 and of 8 ranks, the hierarchical schedule with aggregated chunks,
    # All Pairs with the local reduce): intermediate subnormals, infinities and NaNs travel on through the FIFOs
    es = inputs.ITEMSIZE[dtype]
    cases = [(programs.ring_allreduce(4), 4 * 40000 // es, None),
             (programs.ring_allreduce(8, instances=2), 16 * 20000 // es * 2, None),
             (programs.ring_allreduce(5, use_rrs=True), 5 * 12000 // es, small_cfg()),
             (programs.hierarchical_allreduce(2, 3), 6 * 16016 // es, small_cfg()),
             (programs.allpairs_allreduce(4, via_scratch=True), 4 * 30000 // es, None)]
    for prog, elems, cfg in cases:
        elems -= elems % (prog.in_chunks * 16 // es)
        st = _special_stats(prog, dtype, elems, 950)
        assert st["subnormal"] > 0 and st["inf"] > 0 and st["nan"] > 0, st
        run_case(prog, dtype, elems, "special", 950, cfg, compare=compare_special)
        # all ranks of an AllReduce end with the same bits wherever the result is not a NaN: checked by the
        # element-wise comparison with the oracle, whose ranks agree by construction


# ---- the wavefront-level interpreter (64-thread workgroups that run one thread-block lane each) ------------------

@pytest.mark.parametrize("protocol", ["simple", "ll"])
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_wavefront_level_interpreter(dtype, protocol):
    """Every workgroup is one wavefront with one fiber: counters in registers, no barrier, no LDS state.  Programs
    with and without cross-thread-block dependencies, aggregated instructions, scratch buffers, many peers;
    tiny tiles with ragged tails and the default tile; 2 and 8 slots.  Thread blocks that share a workgroup in
    the plan are dealt to workgroups of their own when the chunk is small (split), which is how the hierarchical
    and All Pairs programs get here.  Under both protocols: payload + flag, and LL (every 8 bytes carry their own
    flag, Section 6.1), where the LL tile replaces the configured one.  The unfused ring (`rrc` then `send` of the
    same chunk) and the All Pairs variant with a chain of local `reduce` instructions are the cases where an
    instruction reads what the previous one of its thread block wrote."""
    H = _harness()
    from paper_2201_11840_amd import binding as B
    m = 4 // inputs.ITEMSIZE[dtype]
    ll = protocol == "ll"
    wave = lambda **kw: H.make_config(wg_size=64, protocol=2 if ll else 1, ll_max_lane_bytes=512 if ll else 0, **kw)
    kernel = B.KERNEL_WAVE_LL if ll else B.KERNEL_WAVE
    cases = [(programs.ring_allreduce(8), 8 * 2500 * m, wave(tile_bytes=1024, team_width=3, min_lane_bytes=16)),
             (programs.ring_allreduce(4, use_rrs=True), 4 * 2500 * m, wave(tile_bytes=256, team_width=2, min_lane_bytes=16, fifo_slots=8)),
             (programs.ring_allreduce(8, instances=2), 16 * 16384 * m, wave(team_width=32, min_lane_bytes=1024, target_wgs=2048)),
             (programs.ring_allreduce(8, instances=8), 64 * 32768 * m, wave(team_width=32, target_wgs=4096)),
             (programs.hierarchical_allreduce(2, 3), 6 * 2000 * m, wave(tile_bytes=1024, team_width=8, min_lane_bytes=4096)),
             (programs.hierarchical_allreduce(2, 8), 16 * 3072 * m, wave(team_width=16, min_lane_bytes=8192)),
             (programs.allpairs_allreduce(8), 8 * 3072 * m, wave(team_width=16, min_lane_bytes=8192)),
             (programs.allpairs_allreduce(4, via_scratch=True), 4 * 1000 * m, wave(tile_bytes=1024, team_width=8, min_lane_bytes=4096)),
             (programs.multichannel_ring_allreduce(5, 3), 5 * 1000 * m, wave(tile_bytes=512, team_width=8, min_lane_bytes=4096)),
             (programs.ring_allreduce(5, fuse=False), 5 * 3000 * m, wave(team_width=4, min_lane_bytes=1024)),
             (programs.allpairs_allreduce(8, via_scratch=True), 8 * 2048 * m, wave(team_width=16, min_lane_bytes=2048)),
             (programs.twostep_alltoall(2, 3), 6 * 1024 * m, wave(team_width=8, min_lane_bytes=1024)),
             (programs.local_stream(4, tbs_per_rank=2, reduce=True), 4 * 4 * 1024 * m, wave(team_width=8, min_lane_bytes=512))]
    for prog, elems, cfg in cases:
        run_case(prog, dtype, elems, "normal", 1200, cfg, repeats=2, expect_kernel=kernel)
    run_case(programs.direct_alltoall(8), dtype, 8 * 2048 * m, "normal", 1201, wave(team_width=16, min_lane_bytes=8192),
             exact_only=True, expect_kernel=kernel)
    run_case(programs.alltonext(2, 3), dtype, 3 * 2048 * m, "normal", 1202, wave(team_width=16, min_lane_bytes=8192),
             exact_only=True, expect_kernel=kernel)
    # instruction lists longer than the wavefront-level kernel keeps in LDS (124 per thread block)
    run_case(programs.ring_allreduce(32, fuse=False), dtype, 32 * 256 * m, "uniform", 1203, wave(team_width=1),
             expect_kernel=kernel)
    # special values travel through the flagged words unchanged
    run_case(programs.ring_allreduce(4), dtype, 4 * 4096 * m, "special", 1205, wave(team_width=4, min_lane_bytes=1024),
             compare=compare_special, expect_kernel=kernel)
    # and 64-thread workgroups that do hold several fibers (24 thread blocks x 2 lanes, 16 workgroups wanted) fall back
    # to the general interpreter
    run_case(programs.hierarchical_allreduce(2, 3), dtype, 6 * 20000 * m, "normal", 1204, wave(team_width=2, target_wgs=16),
             expect_kernel=B.KERNEL_LL if ll else B.KERNEL_GENERAL)


# ---- die-scope FIFOs: payload stays in the L2 of the die both ends of a connection run on -------------------------

@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_die_scope_fifos(dtype):
    """Plain stores into the slots, loads that bypass the compute unit's L1: correct only if sender and receiver of
    every connection share a die, which the planner arranges and every receiver verifies (a violation would end the run
    with GC3_ERR_PLACEMENT, i.e. fail status()).  Programs of every shape - one ring, many rings, pairs, relays,
    cross-thread-block dependencies, thread blocks sharing a workgroup - with slots far smaller than a die's L2
    (the lines are rewritten while still cached) and larger (they are evicted and fetched back)."""
    H = _harness()
    from paper_2201_11840_amd import binding as B
    m = 4 // inputs.ITEMSIZE[dtype]
    die = lambda **kw: H.make_config(fifo_scope=2, **kw)
    cases = [(programs.ring_allreduce(8), 8 * 65536 * m, die(team_width=16)),
             (programs.ring_allreduce(8, instances=8), 64 * 32768 * m, die()),
             (programs.ring_allreduce(8, instances=8), 64 * 16384 * m, die(wg_size=64, team_width=32, target_wgs=4096, min_lane_bytes=1024)),
             (programs.ring_allreduce(5, instances=3, use_rrs=True), 15 * 20000 * m, die(tile_bytes=4096, team_width=8, min_lane_bytes=2048)),
             (programs.ring_allreduce(3, fuse=False), 3 * 50000 * m, die(fifo_slots=1, tile_bytes=2048, team_width=8, min_lane_bytes=1024)),
             (programs.hierarchical_allreduce(2, 8), 16 * 131072 * m, die()),          # every lane active: no split
             (programs.hierarchical_allreduce(3, 2, fuse=False), 6 * 20000 * m, die(team_width=24, tile_bytes=8192, min_lane_bytes=512)),
             (programs.allpairs_allreduce(8), 8 * 65536 * m, die()),
             (programs.allpairs_allreduce(8), 8 * 65536 * m, die(wg_size=64, team_width=64, target_wgs=4096, min_lane_bytes=2048)),
             (programs.allpairs_allreduce(4, via_scratch=True), 4 * 30000 * m, die(team_width=8, tile_bytes=1024, min_lane_bytes=256)),
             (programs.multichannel_ring_allreduce(8, 4), 8 * 65536 * m, die(team_width=16)),
             (programs.ring_allreduce(8, instances=2), 16 * 262144 * m, die(tile_bytes=65536, fifo_slots=8, team_width=16))]
    for prog, elems, cfg in cases:
        run_case(prog, dtype, elems, "normal", 1600, cfg, repeats=3, expect_die=True)
    for prog, elems, cfg in [(programs.alltonext(3, 8), 8 * 65536 * 2, die(team_width=8)), (programs.twostep_alltoall(3, 8), 24 * 32768 * 2, die(team_width=8)),
                             (programs.direct_alltoall(8), 8 * 65536 * 2, die(team_width=16)),
                             (programs.ring_allgather(8, instances=8), 8 * 65536 * m, die(team_width=8))]:
        run_case(prog, dtype, elems, "normal", 1601, cfg, repeats=2, exact_only=True, expect_die=True)
    run_case(programs.ring_allreduce(8, instances=2), dtype, 16 * 32768 * m, "special", 1602, die(team_width=8), compare=compare_special, expect_die=True)
    # small chunks (fiber lists dealt to the idle lanes' workgroups) or a number of active lanes that is not a
    # multiple of 8: such a run uses device-scope FIFOs on the same communicator
    run_case(programs.hierarchical_allreduce(2, 3), dtype, 6 * 1024 * m, "normal", 1603, die(team_width=8), expect_die=False)
    run_case(programs.ring_allreduce(4), dtype, 4 * 40000 * m, "normal", 1604, die(team_width=12, min_lane_bytes=1024), expect_die=False)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_die_scope_user_buffers(dtype):
    """The workgroups of a rank on one die, the rank's buffers read through that die's L2 by thread blocks that wait
    on each other: correct only if the planner's placement holds, which every workgroup verifies (a violation fails
    status() with GC3_ERR_PLACEMENT).  Programs with chains of dependent thread blocks, rank counts that need
    padding, thread blocks sharing workgroups, both protocols, single and many tiles, idle lanes' workgroups in use."""
    H = _harness()
    m = 4 // inputs.ITEMSIZE[dtype]
    die = lambda **kw: H.make_config(user_scope=2, **kw)
    cases = [(programs.allpairs_allreduce(8), 8 * 1024 * m, die(wg_size=64)),
             (programs.allpairs_allreduce(8), 8 * 40000 * m, die(wg_size=64, team_width=16, tile_bytes=4096, min_lane_bytes=1024)),
             (programs.allpairs_allreduce(8, via_scratch=True), 8 * 30000 * m, die(team_width=8, tile_bytes=1024, min_lane_bytes=256)),
             (programs.allpairs_allreduce(5), 5 * 9000 * m, die(wg_size=64, team_width=3, tile_bytes=2048, min_lane_bytes=64)),
             (programs.hierarchical_allreduce(2, 8), 16 * 65536 * m, die()),
             (programs.hierarchical_allreduce(2, 3), 6 * 20000 * m, die(team_width=2, target_wgs=16, tile_bytes=4096)),
             (programs.hierarchical_allreduce(3, 2, fuse=False), 6 * 5000 * m, die(wg_size=64, team_width=8, min_lane_bytes=4096)),
             (programs.hierarchical_allreduce(3, 8), 24 * 8192 * m, die(wg_size=128))]
    for prog, elems, cfg in cases:
        run_case(prog, dtype, elems, "normal", 1700, cfg, repeats=3)
    run_case(programs.twostep_alltoall(2, 4), dtype, 8 * 20000 * m, "normal", 1701, die(team_width=4, tile_bytes=2048), repeats=2, exact_only=True)
    # together with die-scope FIFOs: lanes on dies, FIFO payload and user buffers both through the die's L2; a run with
    # a number of active lanes that is no multiple of 8 falls back to device scope for both
    for prog, elems, cfg, want_die in [(programs.allpairs_allreduce(8), 8 * 65536 * m, die(fifo_scope=2), True),
                                       (programs.allpairs_allreduce(8, via_scratch=True), 8 * 40000 * m, die(fifo_scope=2, wg_size=64, team_width=16, target_wgs=4096, min_lane_bytes=2048), True),
                                       (programs.hierarchical_allreduce(2, 8), 16 * 131072 * m, die(fifo_scope=2), True),
                                       (programs.hierarchical_allreduce(3, 2, fuse=False), 6 * 20000 * m, die(fifo_scope=2, team_width=24, tile_bytes=8192, min_lane_bytes=512), True),
                                       (programs.hierarchical_allreduce(2, 3), 6 * 1024 * m, die(fifo_scope=2, team_width=8), False)]:
        run_case(prog, dtype, elems, "normal", 1703, cfg, repeats=3, expect_die=want_die)
    run_case(programs.allpairs_allreduce(8), dtype, 8 * 4096 * m, "special", 1702, die(wg_size=64), compare=compare_special)
    from tests.test_compiler import _random_program
    from paper_2201_11840_amd.compiler import compile_program
    for seed in range(4):
        ir = compile_program(_random_program(300 + seed, 3 + seed, 3, 16, use_channels=False))
        run_case(ir, dtype, ir.in_chunks * 1000 * m, "normal", 1710 + seed, die(fifo_slots=8, tile_bytes=1024, team_width=2, min_lane_bytes=16), repeats=2)


def test_config3_and_config4_with_die_scope_fifos():
    H = _harness()
    for w in (workloads.ring_ar_r8x8(64), workloads.ring_ar_r8x8(1), workloads.hier_ar_2x8(64), workloads.alltonext_3x8(32)):
        run_case(w.build(), w.dtype, w.elems_per_rank, w.dist, w.seed, H.make_config(fifo_scope=2), repeats=2,
                 exact_only=w.build().collective == "alltonext")


# ---- FIFO payload staged through LDS (direct-to-LDS loads) --------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_lds_staged_payload_path(dtype):
    H = _harness()
    es = inputs.ITEMSIZE[dtype]
    staged = lambda **kw: H.make_config(lds_stage=1, protocol=1, **kw)
    for opcode in ("send", "rrc", "rcs", "rrcs", "rrs"):        # "send" pairs with recv: every receiving instruction
        for count, chunk_bytes in ((1, 16), (2, 3 * 1024 + 48), (1, 40000), (3, 70000 // 16 * 16)):
            prog = _opcode_program(opcode, count)
            run_case(prog, dtype, 2 * count * chunk_bytes // es, "normal", 1300 + count,
                     staged(tile_bytes=20480, team_width=2, min_lane_bytes=16))          # tiles larger than the staging area
        run_case(_opcode_program(opcode, 1), dtype, 2 * (1 << 18) // es, "uniform", 1310, staged())
        run_case(_opcode_program(opcode, 1), dtype, 2 * 50000 * 16 // es, "special", 1311, staged(wg_size=512), compare=compare_special)
    run_case(programs.hierarchical_allreduce(2, 3), dtype, 6 * 30000 // es * 4, "normal", 1320, staged(wg_size=128))
    run_case(programs.ring_allreduce(8, instances=8), dtype, (4 << 20) // es, "uniform", 1321, staged())
    run_case(programs.alltonext(2, 3), dtype, 3 * 65536, "normal", 1322, staged(wg_size=64), exact_only=True)


def test_config3_with_lds_staging():
    w = workloads.ring_ar_r8x8(16)
    run_case(w.build(), w.dtype, w.elems_per_rank, w.dist, w.seed, _harness().make_config(lds_stage=1, protocol=1))


# ---- a run recorded into a HIP graph ---------------------------------------------------------------------------

def test_captured_runs_replay_bit_exactly():
    """gc3_comm_run has constant kernel arguments (the run counters and the LL message numbers live in device
    memory), so a launch can be captured and replayed, under either protocol.  A graph of [restore inputs, run] x 10
    is replayed several times, with eager runs of the same communicator and synchronisations in between; every
    replay must give the eager (oracle-checked) result.  The restore is a copy kernel, not a memset node."""
    import torch
    H = _harness()
    for prog, dtype, elems, cfg in ((programs.ring_allreduce(8, instances=2), "f32", 16 * 8192, dict(protocol=1)),
                                    (programs.hierarchical_allreduce(2, 3), "bf16", 6 * 40000, dict(protocol=1)),
                                    # LL: general kernel (several fibers per workgroup) and wavefront-level kernel
                                    (programs.hierarchical_allreduce(2, 3), "f16", 6 * 8192, dict(protocol=2, team_width=2, target_wgs=16)),
                                    (programs.multichannel_ring_allreduce(8, 4), "f32", 8 * 2048, dict(protocol=2, wg_size=64))):
        text = prog.to_text()
        p = oracle.parse_program(text)
        ins = inputs.make_inputs(p.ranks, elems, dtype, "normal", 1400)
        want = [a.copy() for a in ins]
        oracle.run_program(p, want, None, dtype, slots=2)
        coll = H.Collective(text, dtype, elems, H.make_config(**cfg))
        try:
            coll.upload(ins)
            pristine = [t.clone() for t in coll.inputs]
            coll.run()                                         # eager reference, also the warm-up
            coll.status()
            for g, w_ in zip(coll.download(), want):
                compare(g, w_, dtype)
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.graph(graph, stream=side):
                for _ in range(10):
                    for d, s_ in zip(coll.inputs, pristine):
                        d.copy_(s_)
                    coll.run()
            for replay in range(4):
                for d in coll.inputs:
                    d.fill_(0)                                 # whatever a replay leaves must come from the replay
                graph.replay()
                torch.cuda.synchronize()
                coll.status()
                for g, w_ in zip(coll.download(), want):
                    compare(g, w_, dtype)
                # eager work of the same communicator between replays
                coll.upload(ins)
                coll.run()
                coll.status()
                for g, w_ in zip(coll.download(), want):
                    compare(g, w_, dtype)
        finally:
            coll.close()


def test_buffers_beyond_4GiB_sampled():
    """Offsets past 2^32 bytes: 2 ranks x 5 GiB fp32, two chunks of 2.5 GiB.  The buffers repeat a seeded
    64 MiB host block (so the oracle's inputs come from the shared generator); sampled positions, among them
    the last elements and both sides of the 4 GiB line, are checked against the oracle."""
    import torch
    H = _harness()
    prog = programs.ring_allreduce(2)
    text = prog.to_text()
    p = oracle.parse_program(text)
    block_elems = 16 << 20                                   # 64 MiB of fp32
    reps = 80
    elems = block_elems * reps                               # 5 GiB per rank
    blocks = inputs.make_inputs(2, block_elems, "f32", "uniform", 991)
    coll = H.Collective(text, "f32", elems)
    try:
        for r in range(2):
            dev_block = torch.from_numpy(blocks[r]).to(coll.device)
            coll.inputs[r][:coll.in_bytes].view(torch.float32).view(reps, block_elems).copy_(dev_block.expand(reps, block_elems))
        torch.cuda.synchronize()
        coll.run()
        coll.status()
        ce = elems // 2
        rng = np.random.Generator(np.random.PCG64(5))
        line = (1 << 32) // 4 - ce                           # element of chunk 1 that starts at byte 2^32
        pos = np.unique(np.concatenate([rng.integers(0, ce, 20000),
                                        np.array([0, 1, ce - 2, ce - 1, line - 1, line, line + 1])]))
        idx = torch.from_numpy(np.concatenate([pos, pos + ce])).to(coll.device)
        got = [coll.inputs[r][:coll.in_bytes].view(torch.float32)[idx].cpu().numpy() for r in range(2)]
    finally:
        coll.close()
    glob = np.concatenate([pos, pos + ce])
    small = [blocks[r][glob % block_elems].copy() for r in range(2)]
    oracle.run_program(p, small, None, "f32", slots=2)
    for r in range(2):
        assert got[r].tobytes() == small[r].tobytes()


def test_selector_picks_the_program_by_size():
    # All Pairs for small buffers, the ring above (Section 6: user-configured size ranges; Section 7.1.2)
    H = _harness()
    from paper_2201_11840_amd import binding as B
    small, large = programs.allpairs_allreduce(8), programs.ring_allreduce(8, instances=2)
    max_elems = 16 * 16384
    sel = H.Selector([(small.to_text(), 0, 64 * 1024), (large.to_text(), 64 * 1024 + 1, 0)], "f32", max_elems, tune=True)
    try:
        for elems, want_idx, prog in ((16 * 64, 0, small), (16 * 1024, 0, small), (16 * 1024 + 64, 1, large), (max_elems, 1, large)):
            ins = inputs.make_inputs(8, elems, "f32", "uniform", 400 + elems % 97)
            want = [a.copy() for a in ins]
            oracle.run_program(oracle.parse_program(prog.to_text()), want, None, "f32", slots=2)
            import torch
            for r in range(8):
                sel.inputs[r][:elems * 4].copy_(torch.from_numpy(ins[r].view(np.uint8)))
            assert sel.run(elems) == want_idx
            sel.status()
            for r in range(8):
                got = sel.inputs[r][:elems * 4].cpu().numpy().view(np.float32)
                assert got.tobytes() == want[r].tobytes()
        # a range that ends: sizes beyond it are refused
        bounded = B.gc3_selector_create()
        B.gc3_selector_add(bounded, sel.colls[0].comm, 1024, 4096)
        with pytest.raises(B.Gc3Error) as e:
            B.gc3_selector_run(bounded, 16 * 1024, B.GC3_F32)
        assert e.value.status == B.GC3_ERR_SIZE
        with pytest.raises(B.Gc3Error) as e:
            B.gc3_selector_add(bounded, sel.colls[0].comm, 10, 5)
        assert e.value.status == B.GC3_ERR_ARG
        B.gc3_selector_destroy(bounded)
    finally:
        sel.close()


def test_c_abi_from_a_stand_alone_program(tmp_path):
    """The library used without Python: a C++ program loads IR written by the compiler's command line, tunes,
    binds hipMalloc'ed buffers, runs and checks an AllReduce of integer-valued data."""
    import os
    import subprocess
    from paper_2201_11840_amd import build, gc3c
    if not os.path.exists(build.EXAMPLE_BIN):
        pytest.fail("the example binary is missing: run the build first")
    for argv, elems in ((["ring_allreduce", "--ranks", "8", "--instances", "2"], 16 * 65536),
                        (["hierarchical_allreduce", "--nodes", "2", "--gpus", "4", "--hand"], 8 * 4096),
                        (["allpairs_allreduce", "--ranks", "4"], 4 * 1000)):
        ir = tmp_path / "prog.gc3ir"
        assert gc3c.main(argv + ["-o", str(ir)]) == 0
        res = subprocess.run([build.EXAMPLE_BIN, str(ir), str(elems)], capture_output=True, text=True, timeout=120)
        assert res.returncode == 0, res.stdout + res.stderr
        assert ": OK (0 wrong)" in res.stdout
