"""Repeated full-size runs checked on the device: a rare ordering bug (a flag overtaking its payload, a
stale cache line) would show up as a run whose output differs from the verified first one."""
import numpy as np
import pytest
import torch

import oracle
from paper_2201_11840_amd import harness as H
from paper_2201_11840_amd import inputs, programs, workloads

pytestmark = pytest.mark.gpu


def _verified_first_run(w, coll, ins):
    """Upload, run once, check every element of every rank against the oracle."""
    p = oracle.parse_program(w.build().to_text())
    coll.fill_outputs_with_sentinel()
    coll.upload(ins)
    coll.run()
    coll.status()
    got = coll.download("out")
    want_in = [a.copy() for a in ins]
    want_out = None if p.inplace else inputs.sentinel_outputs(p.ranks, w.elems_per_rank // p.in_chunks * p.out_chunks, w.dtype)
    oracle.run_program(p, want_in, want_out, w.dtype, slots=coll.info.fifo_slots)
    want = want_in if p.inplace else want_out
    for r in range(p.ranks):
        assert got[r].tobytes() == want[r].tobytes(), f"rank {r}"


@pytest.mark.parametrize("w", [workloads.ring_ar_r8x8(16), workloads.hier_ar_2x8(16), workloads.alltonext_3x8(8),
                               workloads.Workload("allpairs_r8_f32_8MiB", lambda: programs.allpairs_allreduce(8),
                                                  "f32", 8 << 20, "uniform", 7)],
                         ids=lambda w: w.name)
@pytest.mark.parametrize("scope", ["device", "die"])
def test_many_runs_give_the_same_verified_result(w, scope):
    # die scope: the plan the tuner picks for the ring (one-wavefront workgroups, 4 KiB tiles: the slots of a die fit
    # its L2 and are rewritten while cached), and 256-thread workgroups with 16 lanes for the others
    prog = w.build()
    ins = inputs.make_inputs(prog.ranks, w.elems_per_rank, w.dtype, w.dist, w.seed)
    cfg = None
    if scope == "die":
        cfg = H.make_config(fifo_scope=2, wg_size=64, team_width=32, target_wgs=4096) if "ring" in w.name else \
            H.make_config(fifo_scope=2, team_width=16)
    coll = H.Collective(prog.to_text(), w.dtype, w.elems_per_rank, cfg)
    assert bool(coll.launch.die_scope) == (scope == "die")
    try:
        _verified_first_run(w, coll, ins)
        good = [t.clone() for t in coll.outputs]
        pristine = None
        if coll.inplace:
            coll.upload(ins)
            pristine = [t.clone() for t in coll.inputs]
        for it in range(150):
            if pristine is not None:
                for d, s in zip(coll.inputs, pristine):
                    d.copy_(s)
            coll.run()
            if it % 10 == 9:
                coll.status()
                for r in range(coll.ranks):
                    assert torch.equal(coll.outputs[r], good[r]), f"run {it}, rank {r}"
    finally:
        coll.close()


@pytest.mark.parametrize("name,build,dtype,nbytes,cfg", [
    ("mc_ring_r8_c4_4KiB", lambda: programs.multichannel_ring_allreduce(8, 4), "f32", 4096, dict(protocol=2, wg_size=64)),
    ("ring_r8_64KiB_8slots", lambda: programs.ring_allreduce(8), "f32", 65536,
     dict(protocol=2, wg_size=64, fifo_slots=8, min_lane_bytes=1024)),
    ("hier_2x3_96KiB_general", lambda: programs.hierarchical_allreduce(2, 3), "bf16", 6 * 16384,
     dict(protocol=2, team_width=2, target_wgs=16)),
    ("allpairs_r8_32KiB", lambda: programs.allpairs_allreduce(8), "f16", 32768, dict(protocol=2, wg_size=64)),
], ids=lambda x: x if isinstance(x, str) else "")
def test_many_ll_runs_give_the_same_verified_result(name, build, dtype, nbytes, cfg):
    """The LL protocol under repetition: its flags count on from run to run in device memory, slots are reused
    with and without head-flag polls, on the wavefront-level and on the general kernel."""
    w = workloads.Workload(name, build, dtype, nbytes, "normal", 11)
    prog = w.build()
    ins = inputs.make_inputs(prog.ranks, w.elems_per_rank, w.dtype, w.dist, w.seed)
    coll = H.Collective(prog.to_text(), w.dtype, w.elems_per_rank, H.make_config(**cfg))
    assert coll.launch.kernel in (1, 4)
    try:
        _verified_first_run(w, coll, ins)
        good = [t.clone() for t in coll.outputs]
        coll.upload(ins)
        pristine = [t.clone() for t in coll.inputs]
        for it in range(3000):
            for d, s in zip(coll.inputs, pristine):
                d.copy_(s)
            coll.run()
            if it % 100 == 99:
                coll.status()
                for r in range(coll.ranks):
                    assert torch.equal(coll.outputs[r], good[r]), f"run {it}, rank {r}"
    finally:
        coll.close()


def test_two_communicators_and_a_side_stream():
    # two communicators alive at once, launched alternately on a non-default stream
    a = workloads.ring_ar_r8x8(1)
    b = workloads.direct_a2a_r8()
    ca = H.Collective(a.build().to_text(), a.dtype, a.elems_per_rank)
    cb = H.Collective(b.build().to_text(), b.dtype, b.elems_per_rank)
    ia = inputs.make_inputs(8, a.elems_per_rank, a.dtype, a.dist, a.seed)
    ib = inputs.make_inputs(8, b.elems_per_rank, b.dtype, b.dist, b.seed)
    wa = [x.copy() for x in ia]
    oracle.run_program(oracle.parse_program(a.build().to_text()), wa, None, a.dtype, slots=2)
    wb = [np.concatenate([ib[j].reshape(8, -1)[i] for j in range(8)]) for i in range(8)]
    side = torch.cuda.Stream()
    try:
        for it in range(5):
            ca.upload(ia)
            cb.fill_outputs_with_sentinel()
            cb.upload(ib)
            with torch.cuda.stream(side):
                ca.run()
                cb.run()
            side.synchronize()
            ca.status()
            cb.status()
            for g, w_ in zip(ca.download(), wa):
                assert g.tobytes() == w_.tobytes()
            for g, w_ in zip(cb.download(), wb):
                assert g.tobytes() == w_.tobytes()
    finally:
        ca.close()
        cb.close()


def test_two_communicators_on_two_streams_share_the_device():
    """Two full-device grids (1024 workgroups each) launched back to back on two streams could not both be resident;
    the library's ledger makes the second stream wait for the first run, so both complete with oracle-exact
    results.  (The rule itself is unit-tested on the CPU; this test never lets two grids compete.)"""
    a, b = workloads.ring_ar_r8x8(16), workloads.hier_ar_2x8(16)
    ca = H.Collective(a.build().to_text(), a.dtype, a.elems_per_rank)
    cb = H.Collective(b.build().to_text(), b.dtype, b.elems_per_rank)
    assert ca.info.grid + cb.info.grid > ca.info.max_resident_wgs
    ia = inputs.make_inputs(8, a.elems_per_rank, a.dtype, a.dist, a.seed)
    ib = inputs.make_inputs(16, b.elems_per_rank, b.dtype, b.dist, b.seed)
    wa, wb = [x.copy() for x in ia], [x.copy() for x in ib]
    oracle.run_program(oracle.parse_program(a.build().to_text()), wa, None, a.dtype, slots=2)
    oracle.run_program(oracle.parse_program(b.build().to_text()), wb, None, b.dtype, slots=2)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    try:
        for it in range(4):
            ca.upload(ia)
            cb.upload(ib)
            with torch.cuda.stream(s1):
                ca.run()
            with torch.cuda.stream(s2):
                cb.run()
            s1.synchronize()
            s2.synchronize()
            ca.status()
            cb.status()
            for g, w_ in zip(ca.download(), wa):
                assert g.tobytes() == w_.tobytes(), f"ring, round {it}"
            for g, w_ in zip(cb.download(), wb):
                assert g.tobytes() == w_.tobytes(), f"hierarchical, round {it}"
        # small grids that fit side by side are not serialised and still give the right answers
        small_a = H.Collective(programs.ring_allreduce(4).to_text(), "f32", 4 * 4096, H.make_config(team_width=2))
        small_b = H.Collective(programs.allpairs_allreduce(4).to_text(), "f32", 4 * 4096, H.make_config(team_width=2))
        xa = inputs.make_inputs(4, 4 * 4096, "f32", "uniform", 3)
        ya = [x.copy() for x in xa]
        oracle.run_program(oracle.parse_program(programs.ring_allreduce(4).to_text()), ya, None, "f32", slots=2)
        yb = [x.copy() for x in xa]
        oracle.run_program(oracle.parse_program(programs.allpairs_allreduce(4).to_text()), yb, None, "f32", slots=2)
        for it in range(4):
            small_a.upload(xa)
            small_b.upload(xa)
            with torch.cuda.stream(s1):
                small_a.run()
            with torch.cuda.stream(s2):
                small_b.run()
            s1.synchronize()
            s2.synchronize()
            small_a.status()
            small_b.status()
            assert all(g.tobytes() == w_.tobytes() for g, w_ in zip(small_a.download(), ya))
            assert all(g.tobytes() == w_.tobytes() for g, w_ in zip(small_b.download(), yb))
        small_a.close()
        small_b.close()
    finally:
        ca.close()
        cb.close()
