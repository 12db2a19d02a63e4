"""gc3_run_static - the entry point for callers that cannot allocate device memory - against gc3_comm_run:
the same program on the same inputs must give the same bytes (and both must equal the oracle), call after
call on the one static device array, also when the next call is smaller or runs another program."""
import numpy as np
import pytest
import torch

import oracle
from paper_2201_11840_amd import binding as B
from paper_2201_11840_amd import harness as H
from paper_2201_11840_amd import inputs, programs

pytestmark = pytest.mark.gpu


def _static_run(prog, dtype, elems, ins, cfg=None):
    """Upload `ins` into fresh device buffers, run once through gc3_run_static, return the output arrays."""
    text = prog.to_text()
    es = inputs.ITEMSIZE[dtype]
    cb = elems // prog.in_chunks * es
    dev = torch.device("cuda:0")
    d_in = [torch.from_numpy(a.view(np.uint8).copy()).to(dev) for a in ins]
    out_bytes = cb * prog.out_chunks
    d_out = None
    if not prog.inplace:
        d_out = [torch.full((out_bytes // 2,), inputs.SENTINEL16, dtype=torch.int16, device=dev) for _ in ins]
    sc = [prog.scratch_chunks(r) for r in range(prog.ranks)]
    d_sc = [torch.empty(max(n * cb, 16), dtype=torch.uint8, device=dev) if n else None for n in sc]
    torch.cuda.synchronize()
    h = B.gc3_program_load(text)
    try:
        B.gc3_run_static(h, cfg, [t.data_ptr() for t in d_in],
                         None if d_out is None else [t.data_ptr() for t in d_out],
                         [t.data_ptr() if t is not None else None for t in d_sc] if any(sc) else None,
                         [n * cb for n in sc] if any(sc) else None,
                         elems, B.DTYPE_CODE[dtype], B.GC3_SUM, torch.cuda.current_stream().cuda_stream)
    finally:
        B.gc3_program_free(h)
    torch.cuda.synchronize()
    st = inputs.STORAGE[dtype]
    res = d_in if prog.inplace else d_out
    return [t.cpu().numpy().view(np.uint8).view(st).copy() for t in res]


def _comm_run(prog, dtype, elems, ins):
    coll = H.Collective(prog.to_text(), dtype, elems)
    try:
        coll.fill_outputs_with_sentinel()
        coll.upload(ins)
        coll.run()
        coll.status()
        return coll.download("out")
    finally:
        coll.close()


def _oracle_run(prog, dtype, elems, ins):
    p = oracle.parse_program(prog.to_text())
    want_in = [a.copy() for a in ins]
    want_out = None if p.inplace else inputs.sentinel_outputs(p.ranks, elems // p.in_chunks * p.out_chunks, dtype)
    oracle.run_program(p, want_in, want_out, dtype, slots=2)
    return want_in if p.inplace else want_out


def _check(prog, dtype, elems, seed, cfg=None):
    ins = inputs.make_inputs(prog.ranks, elems, dtype, "normal", seed)
    got = _static_run(prog, dtype, elems, ins, cfg)
    ref = _comm_run(prog, dtype, elems, ins)
    want = _oracle_run(prog, dtype, elems, ins)
    for r in range(prog.ranks):
        assert got[r].tobytes() == ref[r].tobytes(), f"rank {r}: differs from gc3_comm_run"
        assert got[r].tobytes() == want[r].tobytes(), f"rank {r}: differs from the oracle"


def test_static_entry_point_matches_the_communicator_path():
    ring = programs.ring_allreduce(8, instances=2)
    _check(ring, "f32", 16 * 65536, 1)              # 4 MiB per rank: several tiles per lane
    _check(ring, "f32", 16 * 1000, 2)               # the next call is smaller: stale flags and tables must not matter
    # other programs on the same array: cross-thread-block semaphores, scratch buffers, out-of-place outputs
    _check(programs.hierarchical_allreduce(2, 3), "bf16", 6 * 20000, 3)
    _check(programs.alltonext(2, 3), "f16", 3 * 4096, 4)
    _check(programs.allpairs_allreduce(4, via_scratch=True), "f32", 4 * 2500, 5, H.make_config(tile_bytes=1024, team_width=3, min_lane_bytes=16))
    _check(ring, "f32", 16 * 4, 6)                  # smallest chunk: one 16-byte unit
    # die-scope user buffers: the placement word is cleared with the flags before every call
    _check(programs.allpairs_allreduce(8), "f32", 8 * 3000, 8, H.make_config(user_scope=2, wg_size=64, team_width=2, tile_bytes=2048, min_lane_bytes=256))
    _check(programs.hierarchical_allreduce(2, 3), "bf16", 6 * 20000, 9, H.make_config(user_scope=2))
    # 8 slots: freed slots are announced after every 4th message only; many small tiles per lane
    _check(ring, "f32", 16 * 20000, 7, H.make_config(fifo_slots=8, tile_bytes=2048, team_width=4, min_lane_bytes=16))


def test_static_entry_point_rejects_what_does_not_fit():
    big = programs.ring_allreduce(8, instances=8)
    h = B.gc3_program_load(big.to_text())
    ptrs = [4096 * (r + 1) for r in range(8)]        # never dereferenced: every call below fails before any device work
    run = lambda cfg, elems, dt=B.GC3_F32: B.gc3_run_static(h, cfg, ptrs, None, None, None, elems, dt)
    try:
        with pytest.raises(B.Gc3Error) as e:         # 64 connections x 64 lanes x 2 slots x 64 KiB = 512 MiB of FIFOs
            run(H.make_config(team_width=64, tile_bytes=65536), 64 * 65536)
        assert e.value.status == B.GC3_ERR_SIZE and "bytes" in e.value.message
        with pytest.raises(B.Gc3Error) as e:
            run(None, 64 * 65536 + 1)                # not a multiple of the chunk count
        assert e.value.status == B.GC3_ERR_SIZE
        with pytest.raises(B.Gc3Error) as e:
            run(H.make_config(protocol=2), 64 * 65536)
        assert e.value.status == B.GC3_ERR_ARG
        with pytest.raises(B.Gc3Error) as e:
            run(None, 64 * 65536, 7)                 # unknown data type
        assert e.value.status == B.GC3_ERR_ARG
    finally:
        B.gc3_program_free(h)
    relay = programs.alltonext(2, 3)
    h = B.gc3_program_load(relay.to_text())
    try:
        with pytest.raises(B.Gc3Error) as e:         # scratch capacity too small for this chunk size
            B.gc3_run_static(h, None, [4096] * 6, [8192] * 6, [12288] * 6, [16] * 6, 3 * 4096, B.GC3_F16)
        assert e.value.status == B.GC3_ERR_SIZE
        with pytest.raises(B.Gc3Error) as e:         # out-of-place program without outputs
            B.gc3_run_static(h, None, [4096] * 6, None, [12288] * 6, [1 << 30] * 6, 3 * 4096, B.GC3_F16)
        assert e.value.status == B.GC3_ERR_ARG
    finally:
        B.gc3_program_free(h)


def test_static_entry_point_reports_an_abandoned_run_on_the_next_call():
    # every workgroup waits (bounded by spin_limit_us) for a start word nobody sets and leaves through the error
    # path; the next call reports it and does not run, the one after that is a normal run again
    ring = programs.ring_allreduce(4)
    elems = 4 * 4096
    ins = inputs.make_inputs(4, elems, "f32", "uniform", 9)
    held = _static_run(ring, "f32", elems, ins, H.make_config(spin_limit_us=20000, debug_hold=1))
    for g, a in zip(held, ins):
        assert g.tobytes() == a.tobytes()           # nothing was moved
    with pytest.raises(B.Gc3Error) as e:
        _static_run(ring, "f32", elems, ins)
    assert e.value.status == B.GC3_ERR_TIMEOUT
    _check(ring, "f32", elems, 9)
