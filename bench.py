#!/usr/bin/env python3
"""Benchmark of the GC3-IR interpreter on one MI355X.

A step is one complete run of a GC3-IR program (all ranks, all thread blocks, all instructions) over
one batch of synthetic per-rank buffers already resident in HBM.  Protocol of the paper's Section 7
(experimental setup): warm-up iterations, then the mean over the timed iterations; defaults 20 + 50.

The headline workload is the Ring AllReduce on 8 virtual ranks, parallelize = 8, fp32, 64 MiB per rank.
Because an in-place AllReduce overwrites its input, every step first restores the inputs from a
device-side copy; that restore is outside the timed window (HIP events bracket the run only).
`value` = algorithmic bytes of one run / mean event time.  A second figure, `back_to_back`, times K
launches wall-clock with no restore in between (values drift, throughput does not depend on them).

Team width, workgroup target, slot tile and workgroup size of every workload are picked by the library's
own tuner (gc3_comm_tune: a few short runs per candidate plan at set-up, before the warm-up) unless
--no-tune is given; the plan chosen and the planner's untuned figure for the headline workload are part of
the output.

Beside the headline the same JSON line carries, for every workload of the sweep: the share of its
algorithmic bytes that is FIFO traffic (which the 256 MiB memory-side cache can serve), the traffic that has
to touch the user buffers, the launch it was timed in, and the oracle timed on the host on a bounded sample
of the same workload; and `roofline_dram`: the interpreter's local copy / reduce instructions streaming
buffers far larger than that cache, i.e. what device memory itself sustains for this kernel.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak
HEADLINE = "ring_allreduce_r8_x8_f32_64MiB"
# HBM-side traffic per launch measured with rocprofv3 (FETCH_SIZE and WRITE_SIZE, two runs, each scaled by the
# same counter's reading for a plain copy of known size): one line per workload, written next to the
# summaries it comes from
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gc3_interpreter_hbm_traffic.txt")
PAPER_CONTEXT = ("the paper reports speedups only, on other hardware: up to 1.9x over NCCL's ring AllReduce "
                 "(one node, 8 x A100 with NVLink3 / NVSwitch, 32 KB - 3 MB buffers), up to 1.3x over a hand-optimised "
                 "Two-Step AllToAll (16 nodes, 256 x A100 with InfiniBand); context, not comparable to one MI355X")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


KERNEL_NAMES = ("general", "ll", "lds_staged", "wavefront", "wavefront_ll")   # gc3_launch_info.kernel


def measured_traffic():
    """workload -> bytes per launch (fetch + write), from the tracked profile data; empty when the file is missing."""
    out = {}
    if os.path.exists(TRAFFIC_FILE):
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) >= 3 and not line.lstrip().startswith("#"):
                out[f[0]] = int(float(f[1]) + float(f[2]))
    return out


def time_workload(coll, steps, warmup, pristine):
    """Returns (mean_ms, min_ms, wall_ms_back_to_back)."""
    import torch

    def restore():
        if pristine is not None:
            for dst, src in zip(coll.inputs, pristine):
                dst.copy_(src)

    for _ in range(warmup):
        restore()
        coll.run()
    coll.status()
    starts = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stops = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    torch.cuda.synchronize()
    for i in range(steps):
        restore()
        starts[i].record()
        coll.run()
        stops[i].record()
    torch.cuda.synchronize()
    coll.status()
    ms = [s.elapsed_time(e) for s, e in zip(starts, stops)]
    # back to back, wall clock, no restore
    restore()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        coll.run()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) * 1e3 / steps
    coll.status()
    return sum(ms) / len(ms), min(ms), wall


def device_inputs(coll, w, seed):
    """Fill the input buffers with seeded synthetic values on the device (timing-only workloads)."""
    import torch
    g = torch.Generator(device=coll.device)
    g.manual_seed(seed)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[w.dtype]
    for r in range(coll.ranks):
        v = coll.inputs[r][:coll.in_bytes].view(tdt)
        if w.dist == "uniform":
            v.copy_(torch.rand(v.shape, generator=g, device=coll.device, dtype=torch.float32).mul_(2).sub_(1).to(tdt))
        elif w.dist == "int8":
            v.copy_(torch.randint(-8, 9, v.shape, generator=g, device=coll.device).to(tdt))
        else:
            v.copy_(torch.randn(v.shape, generator=g, device=coll.device, dtype=torch.float32).to(tdt))
    torch.cuda.synchronize()


def oracle_baseline(w, prog, budget_s, sample_bytes_per_rank, slots):
    """The oracle as it stands (sequential numpy interpreter, one host core) on this workload or, for large
    ones, on the same program with `sample_bytes_per_rank` per rank; repeated until `budget_s` of oracle time is
    spent.  Throughput = algorithmic bytes of what was run / oracle time.  Returns (dict, last outputs, inputs used
    were the workload's own iff the sample is the full workload)."""
    import oracle
    from paper_2201_11840_amd import inputs
    p = oracle.parse_program(prog.to_text())
    es = inputs.ITEMSIZE[w.dtype]
    unit = p.in_chunks * (16 // es)                       # elements: whole chunks of whole 16-byte units
    elems = w.elems_per_rank
    full = True
    if w.bytes_per_rank > sample_bytes_per_rank:
        elems = max(unit, (sample_bytes_per_rank // es) // unit * unit)
        full = False
    ins = inputs.make_inputs(p.ranks, elems, w.dtype, w.dist, w.seed)
    out_elems = elems // p.in_chunks * p.out_chunks
    alg = prog.algorithmic_chunks() * (elems // p.in_chunks) * es
    t_total, reps, result = 0.0, 0, None
    while reps < 200 and (reps == 0 or t_total < budget_s):
        host_in = [a.copy() for a in ins]
        host_out = None if p.inplace else inputs.sentinel_outputs(p.ranks, out_elems, w.dtype)
        t0 = time.perf_counter()
        oracle.run_program(p, host_in, host_out, w.dtype, slots=slots)
        t_total += time.perf_counter() - t0
        reps += 1
        result = host_in if p.inplace else host_out
    what = f"the full workload ({w.name})" if full else \
        f"the same program on {elems * es // 1024} KiB per rank instead of {w.bytes_per_rank // 1024} KiB"
    rec = {"value": round(alg * reps / t_total / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
           "sample": f"{what}, {reps} run(s) of the sequential numpy oracle, {t_total / reps:.3f} s per run; "
                     f"host has {os.cpu_count()} logical cores",
           "seconds_per_run": round(t_total / reps, 4)}
    return rec, result, full


TUNE_LAUNCHES_PER_PLAN = 7   # gc3_comm_tune: 2 warm-up + 5 timed runs per plan ...
TUNE_EXTRA_LAUNCHES = 6      # ... and 6 more warm-up runs for the first plan


def report(w, coll, mean_ms, min_ms, wall_ms, prog, launches_before_timed=0):
    gbs = coll.algorithmic_bytes / (mean_ms * 1e-3) / 1e9
    li = coll.launch
    fifo = prog.fifo_chunks() * coll.chunk_bytes
    user = coll.algorithmic_bytes - fifo                 # has to touch the user buffers even with perfectly cached FIFOs
    rec = {"workload": w.name, "dtype": w.dtype, "ranks": coll.ranks, "bytes_per_rank": w.bytes_per_rank,
           "algorithmic_bytes": coll.algorithmic_bytes, "ms_mean": round(mean_ms, 5), "ms_min": round(min_ms, 5),
           "ms_back_to_back": round(wall_ms, 5), "aggregate_GBps": round(gbs, 1),
           "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
           "per_rank_algbw_GBps": round(w.bytes_per_rank / (mean_ms * 1e-3) / 1e9, 2),
           "fifo_fraction_of_bytes": round(fifo / coll.algorithmic_bytes, 4) if coll.algorithmic_bytes else 0.0,
           "user_buffer_bytes": user, "user_buffer_GBps": round(user / (mean_ms * 1e-3) / 1e9, 1),
           "grid": coll.info.grid, "team_width": coll.info.team_width, "wg_size": coll.info.wg_size,
           "tile_bytes": coll.info.tile_bytes, "fifo_slots": coll.info.fifo_slots,
           "fifo_MiB": round(coll.info.fifo_bytes / 2 ** 20, 1),
           "launch": {"grid": li.grid, "wg_size": li.wg_size, "active_lanes": li.active_lanes, "split": li.split,
                      "tile_bytes": li.tile_bytes, "fifo_scope": "die" if li.die_scope else "device",
                      "user_scope": "die" if coll.info.user_scope == 2 else "device",
                      "kernel": KERNEL_NAMES[li.kernel]}}
    rep = coll.tune_report
    if rep is not None:
        rec["tuned"] = {"team_width": coll.cfg.team_width, "target_wgs": coll.cfg.target_wgs,
                        "tile_bytes": coll.cfg.tile_bytes, "wg_size": coll.cfg.wg_size, "fifo_scope": coll.cfg.fifo_scope,
                        "user_scope": coll.cfg.user_scope,
                        "plans_timed": rep.count,
                        "untuned_plan_ms_in_tuner": round(rep.tried[0].ms, 5),
                        "chosen_plan_ms_in_tuner": round(rep.tried[rep.best].ms, 5)}
    rec["interpreter_launches_before_timed"] = launches_before_timed
    return rec


def graph_replay_us(c, runs_per_graph=20, replays=5):
    """Time per run when 20 runs of collective `c` are recorded once into a HIP graph and the graph is replayed:
    what is left of a latency-bound collective without the host's enqueue path."""
    import torch
    for _ in range(3):
        c.run()
    c.status()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        for _ in range(runs_per_graph):
            c.run()
    graph.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(replays):
        graph.replay()
    b.record()
    torch.cuda.synchronize()
    c.status()
    del graph
    return round(a.elapsed_time(b) * 1e3 / (replays * runs_per_graph), 2)


def size_sweep(steps, warmup, tune, cfg):
    """AllReduce on 8 ranks, fp32, per-rank sizes 4 KiB .. 256 MiB, five schedules of Section 7.1: the time per
    collective and the per-rank algorithm bandwidth S / time, to show which schedule wins at which size."""
    import torch
    from paper_2201_11840_amd import harness, programs, workloads
    algos = [("ring_x1", lambda: programs.ring_allreduce(8)),
             ("ring_x8", lambda: programs.ring_allreduce(8, instances=8)),
             ("ring_4ch", lambda: programs.multichannel_ring_allreduce(8, 4)),
             ("allpairs", lambda: programs.allpairs_allreduce(8)),
             ("allpairs_scratch", lambda: programs.allpairs_allreduce(8, via_scratch=True))]
    rows = []
    for kib in (4, 16, 64, 256, 1024, 4096, 16384, 65536, 262144):
        row = {"bytes_per_rank": kib * 1024}
        for name, build in algos:
            prog = build()
            elems = kib * 1024 // 4
            if elems % prog.in_chunks or (elems // prog.in_chunks * 4) % 16:
                row[name] = None                      # chunk would not be a whole number of 16-byte units
                continue
            w = workloads.Workload(f"{name}_{kib}KiB", build, "f32", kib * 1024, "uniform", 71840)
            c = harness.Collective(prog.to_text(), "f32", elems, cfg, tune=tune)
            device_inputs(c, w, w.seed)
            pr = [t.clone() for t in c.inputs]
            m, mn, wall = time_workload(c, steps, warmup, pr)
            li = c.launch
            row[name] = {"us": round(m * 1e3, 2), "us_back_to_back": round(wall * 1e3, 2),
                         "algbw_GBps": round(kib * 1024 / (m * 1e-3) / 1e9, 2),
                         "team_width": c.info.team_width, "grid": li.grid, "wg_size": li.wg_size,
                         "kernel": KERNEL_NAMES[li.kernel]}
            if kib <= 1024:
                row[name]["us_graph_replay"] = graph_replay_us(c)
            c.close()
            del pr, c
            torch.cuda.empty_cache()
        log("[bench] size sweep " + json.dumps(row))
        rows.append(row)
    return rows


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE)
    ap.add_argument("--no-sweep", action="store_true", help="time the headline workload only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-tune", action="store_true", help="use the planner's plan as is (no gc3_comm_tune)")
    ap.add_argument("--size-sweep", action="store_true",
                    help="also time five AllReduce schedules on 8 ranks from 4 KiB to 256 MiB per rank (adds about a minute)")
    ap.add_argument("--tile-bytes", type=int, default=0)
    ap.add_argument("--team-width", type=int, default=0)
    ap.add_argument("--fifo-slots", type=int, default=0)
    ap.add_argument("--wg-size", type=int, default=0)
    ap.add_argument("--target-wgs", type=int, default=0)
    ap.add_argument("--lds-stage", type=int, default=0)
    ap.add_argument("--fifo-scope", type=int, default=0, help="1 device scope, 2 die scope (FIFO payload stays in the dies' L2s)")
    ap.add_argument("--user-scope", type=int, default=0, help="1 device scope, 2 die scope (a rank's workgroups share a die and read its buffers through that die's L2)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU: the ranks of a GC3-IR program are virtual ranks in one "
            "MI355X's memory and no multi-GPU path exists; rerun with --gpus 1")
        return 2

    import torch
    from paper_2201_11840_amd import harness, inputs, workloads

    table = workloads.by_name()
    if args.workload not in table:
        log(f"unknown workload {args.workload}; known: {sorted(table)}")
        return 2
    cfg = harness.make_config(fifo_slots=args.fifo_slots, tile_bytes=args.tile_bytes, team_width=args.team_width,
                              wg_size=args.wg_size, target_wgs=args.target_wgs, lds_stage=args.lds_stage,
                              protocol=1 if args.lds_stage else 0, fifo_scope=args.fifo_scope, user_scope=args.user_scope)
    traffic = measured_traffic()

    # ---- headline workload: seeded host inputs (shared with the CPU baseline) ---------------------
    w = table[args.workload]
    prog = w.build()
    text = prog.to_text()
    log(f"[bench] generating inputs for {w.name}")
    ins = inputs.make_inputs(prog.ranks, w.elems_per_rank, w.dtype, w.dist, w.seed)
    tune = not args.no_tune
    untuned = None
    if tune:
        # the planner's plan as is, for reference (same protocol)
        c0 = harness.Collective(text, w.dtype, w.elems_per_rank, cfg)
        c0.upload(ins)
        pr0 = [t.clone() for t in c0.inputs] if c0.inplace else None
        m0, mn0, _ = time_workload(c0, args.steps, args.warmup, pr0)
        untuned = {"ms_mean": round(m0, 5), "aggregate_GBps": round(c0.algorithmic_bytes / (m0 * 1e-3) / 1e9, 1),
                   "team_width": c0.info.team_width, "grid": c0.info.grid}
        before = args.warmup + 2 * args.steps
        c0.close()
        del pr0, c0
        torch.cuda.empty_cache()
    else:
        before = 0
    coll = harness.Collective(text, w.dtype, w.elems_per_rank, cfg, tune=tune)
    if coll.tune_report is not None:
        before += coll.tune_report.count * TUNE_LAUNCHES_PER_PLAN + TUNE_EXTRA_LAUNCHES
    coll.fill_outputs_with_sentinel()
    coll.upload(ins)
    pristine = [t.clone() for t in coll.inputs] if coll.inplace else None
    coll.run()
    coll.status()
    gpu_out = coll.download("out")
    log(f"[bench] timing {w.name}: grid={coll.info.grid} W={coll.info.team_width}")
    mean_ms, min_ms, wall_ms = time_workload(coll, args.steps, args.warmup, pristine)
    head = report(w, coll, mean_ms, min_ms, wall_ms, prog, before + 1 + args.warmup)
    alg_bytes = coll.algorithmic_bytes
    coll.close()
    del pristine, ins
    torch.cuda.empty_cache()

    # ---- CPU baseline: the oracle as it stands, on the host cores, on the full headline workload ------
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        log("[bench] cpu baseline (oracle) ...")
        cpu, want, full = oracle_baseline(w, prog, 10.0, 1 << 62, head["fifo_slots"])
        parity = "bitwise_equal" if all(g.tobytes() == x.tobytes() for g, x in zip(gpu_out, want)) else "MISMATCH"
        head["cpu_baseline"] = cpu
        del want
    del gpu_out

    # ---- the other configurations (timing only, device-generated inputs) ---------------------------
    sweep = [head]
    dram = {}
    if not args.no_sweep:
        for w2 in workloads.all_workloads() + workloads.next_row_workloads() + workloads.dram_workloads():
            if w2.name == w.name:
                continue
            log(f"[bench] timing {w2.name}")
            prog2 = w2.build()
            c2 = harness.Collective(prog2.to_text(), w2.dtype, w2.elems_per_rank, cfg, tune=tune)
            device_inputs(c2, w2, w2.seed)
            c2.fill_outputs_with_sentinel()
            pr = [t.clone() for t in c2.inputs]      # every run finds freshly written inputs, in place or not
            m, mn, wl = time_workload(c2, args.steps, args.warmup, pr)
            before2 = (c2.tune_report.count * TUNE_LAUNCHES_PER_PLAN + TUNE_EXTRA_LAUNCHES if c2.tune_report is not None else 0) + args.warmup
            rec = report(w2, c2, m, mn, wl, prog2, before2)
            if m < 0.1:                                   # latency-bound: also without the host's enqueue path
                rec["ms_graph_replay"] = round(graph_replay_us(c2) * 1e-3, 5)
                rec["interpreter_launches_after_timed"] = args.steps + 3 + 20 * 6     # back to back; warm-up, 6 replays of 20
            slots = c2.info.fifo_slots
            c2.close()
            del pr, c2
            torch.cuda.empty_cache()
            if not args.no_cpu_baseline:
                # one oracle run on at most 8 MiB per rank of the same program (the rate barely depends on the size)
                rec["cpu_baseline"], _, _ = oracle_baseline(w2, prog2, 0.0, 8 << 20, slots)
            if w2.name in traffic:
                rec["measured_hbm_traffic_bytes"] = traffic[w2.name]
            if w2.name.startswith("local_"):
                dram[w2.name] = rec
            sweep.append(rec)

    gbs = alg_bytes / (mean_ms * 1e-3) / 1e9
    roofline_dram = None
    if dram:
        best = max(dram.values(), key=lambda r: r["aggregate_GBps"])
        roofline_dram = {"bound": "hbm", "achieved": best["aggregate_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(best["aggregate_GBps"] / HBM_PEAK_GBS, 4), "traffic": traffic.get(best["workload"]),
                         "kernel": "gc3_interpreter", "workload": best["workload"],
                         "what": "the interpreter's local copy / reduce instructions over buffers 8 to 16 times the "
                                 "256 MiB memory-side cache, no FIFO: every byte comes from and goes to DRAM",
                         "all": {k: v["aggregate_GBps"] for k, v in dram.items()}}
    out = {
        "metric": "aggregate HBM GB/s (and % of peak) executing AllReduce/AllToAll GC3-IR",
        "metric_definition": "algorithmic bytes of one run / mean kernel time; % of peak in frac_of_hbm_peak and roofline.frac",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(mean_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "f16": "f16", "bf16": "bf16"}[table[args.workload].dtype], "data": "synthetic",
        "config": {"workload": args.workload, "ranks": head["ranks"], "bytes_per_rank": head["bytes_per_rank"],
                   "grid": head["grid"], "team_width": head["team_width"], "wg_size": head["wg_size"],
                   "tile_bytes": head["tile_bytes"], "fifo_slots": head["fifo_slots"], "launch": head["launch"],
                   "plan": "chosen by gc3_comm_tune at set-up" if tune else "planner default",
                   "timing": "HIP events around each run on the launch stream; inputs restored outside the window"},
        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "per_rank_algbw_GBps": head["per_rank_algbw_GBps"],
        "untuned_plan": untuned,
        "ms_per_step_min": round(min_ms, 5),
        "ms_per_step_back_to_back_wall": round(wall_ms, 5),
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": traffic.get(args.workload),
                     "kernel": "gc3_interpreter", "algorithmic_bytes_per_launch": alg_bytes,
                     "fifo_fraction_of_bytes": head["fifo_fraction_of_bytes"],
                     "user_buffer_GBps": head["user_buffer_GBps"],
                     "note": "achieved counts every algorithmic byte; the FIFO share of them has a short reuse distance "
                             "and can be served by the 256 MiB memory-side cache, only user_buffer_GBps must reach DRAM; "
                             "roofline_dram is the same kernel with no FIFO on DRAM-resident buffers"},
        "roofline_dram": roofline_dram,
        "cpu_baseline": cpu,
        "parity_vs_oracle": parity,
        "paper_context": PAPER_CONTEXT,
        "workloads": sweep,
    }
    if args.size_sweep:
        out["allreduce_size_sweep"] = size_sweep(min(args.steps, 30), min(args.warmup, 10), tune, cfg)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
