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

Team width and workgroup target of every workload are picked by the library's own tuner (gc3_comm_tune:
a few short runs per candidate plan at set-up, before the warm-up) unless --no-tune is given; the plan
chosen and the planner's untuned figure for the headline workload are part of the output.

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

# HBM-side traffic per launch (bytes): rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (two runs), each
# scaled by the same counter's reading for this script's own 64 MiB restore copy (factors 1.9989 and
# 1.0000); the traffic does not depend on the plan.  Workloads not listed were not measured (null).
MEASURED_TRAFFIC = {"ring_allreduce_r8_x8_f32_64MiB": 3365023295, "hier_allreduce_2x8_bf16_64MiB": 7473969376,
                    "alltonext_3x8_f16_32MiB": 3443780562}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


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


TUNE_LAUNCHES_PER_PLAN = 7   # gc3_comm_tune: 2 warm-up + 5 timed runs per plan ...
TUNE_EXTRA_LAUNCHES = 6      # ... and 6 more warm-up runs for the first plan


def report(w, coll, mean_ms, min_ms, wall_ms, prog=None, launches_before_timed=0):
    gbs = coll.algorithmic_bytes / (mean_ms * 1e-3) / 1e9
    extra = {}
    if prog is not None:
        # traffic that has to touch the user buffers even with perfectly cached FIFOs
        user = coll.algorithmic_bytes - prog.fifo_chunks() * coll.chunk_bytes
        extra = {"user_buffer_bytes": user, "user_buffer_GBps": round(user / (mean_ms * 1e-3) / 1e9, 1)}
    rep = coll.tune_report
    if rep is not None:
        extra["tuned"] = {"team_width": coll.cfg.team_width, "target_wgs": coll.cfg.target_wgs,
                          "tile_bytes": coll.cfg.tile_bytes, "wg_size": coll.cfg.wg_size,
                          "plans_timed": rep.count,
                          "untuned_plan_ms_in_tuner": round(rep.tried[0].ms, 5),
                          "chosen_plan_ms_in_tuner": round(rep.tried[rep.best].ms, 5)}
    extra["interpreter_launches_before_timed"] = launches_before_timed
    return {**_report_base(w, coll, mean_ms, min_ms, wall_ms, gbs), **extra}


def _report_base(w, coll, mean_ms, min_ms, wall_ms, gbs):
    return {"workload": w.name, "dtype": w.dtype, "ranks": coll.ranks, "bytes_per_rank": w.bytes_per_rank,
            "algorithmic_bytes": coll.algorithmic_bytes, "ms_mean": round(mean_ms, 5), "ms_min": round(min_ms, 5),
            "ms_back_to_back": round(wall_ms, 5), "aggregate_GBps": round(gbs, 1),
            "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
            "per_rank_algbw_GBps": round(w.bytes_per_rank / (mean_ms * 1e-3) / 1e9, 2),
            "grid": coll.info.grid, "team_width": coll.info.team_width, "wg_size": coll.info.wg_size,
            "tile_bytes": coll.info.tile_bytes, "fifo_slots": coll.info.fifo_slots,
            "fifo_MiB": round(coll.info.fifo_bytes / 2 ** 20, 1)}


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
            m, mn, _ = time_workload(c, steps, warmup, pr)
            row[name] = {"us": round(m * 1e3, 2), "algbw_GBps": round(kib * 1024 / (m * 1e-3) / 1e9, 2),
                         "team_width": c.info.team_width, "grid": c.info.grid}
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
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU: the ranks of a GC3-IR program are virtual ranks in one "
            "MI355X's memory and no multi-GPU path exists; rerun with --gpus 1")
        return 2

    import numpy as np
    import torch
    from paper_2201_11840_amd import harness, inputs, workloads

    table = workloads.by_name()
    if args.workload not in table:
        log(f"unknown workload {args.workload}; known: {sorted(table)}")
        return 2
    cfg = harness.make_config(fifo_slots=args.fifo_slots, tile_bytes=args.tile_bytes, team_width=args.team_width,
                              wg_size=args.wg_size)

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
    del pristine
    torch.cuda.empty_cache()

    # ---- CPU baseline: the oracle as it stands, on the host cores ----------------------------------
    cpu = None
    parity = None
    if not args.no_cpu_baseline:
        import oracle
        p = oracle.parse_program(text)
        log("[bench] cpu baseline (oracle) ...")
        t_total, reps = 0.0, 0
        while reps < 200 and t_total < 10.0:          # about 10 s of oracle work
            host_in = [a.copy() for a in ins]
            host_out = None if p.inplace else inputs.sentinel_outputs(p.ranks, gpu_out[0].size, w.dtype)
            t0 = time.perf_counter()
            oracle.run_program(p, host_in, host_out, w.dtype, slots=head["fifo_slots"])
            t_total += time.perf_counter() - t0
            reps += 1
        want = host_in if p.inplace else host_out
        parity = "bitwise_equal" if all(g.tobytes() == x.tobytes() for g, x in zip(gpu_out, want)) else "MISMATCH"
        cpu = {"value": round(alg_bytes * reps / t_total / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
               "sample": f"the full workload ({w.name}), {reps} run(s) of the sequential numpy oracle, "
                         f"{t_total / reps:.2f} s per run; host has {os.cpu_count()} logical cores",
               "seconds_per_run": round(t_total / reps, 3)}
    del ins, gpu_out

    # ---- the other configurations (timing only, device-generated inputs) ---------------------------
    sweep = [head]
    if not args.no_sweep:
        for w2 in workloads.all_workloads() + workloads.next_row_workloads():
            if w2.name == w.name:
                continue
            log(f"[bench] timing {w2.name}")
            prog2 = w2.build()
            c2 = harness.Collective(prog2.to_text(), w2.dtype, w2.elems_per_rank, cfg, tune=tune)
            device_inputs(c2, w2, w2.seed)
            c2.fill_outputs_with_sentinel()
            pr = [t.clone() for t in c2.inputs] if c2.inplace else None
            m, mn, wl = time_workload(c2, args.steps, args.warmup, pr)
            before2 = (c2.tune_report.count * TUNE_LAUNCHES_PER_PLAN + TUNE_EXTRA_LAUNCHES if c2.tune_report is not None else 0) + args.warmup
            sweep.append(report(w2, c2, m, mn, wl, prog2, before2))
            c2.close()
            del pr, c2
            torch.cuda.empty_cache()

    gbs = alg_bytes / (mean_ms * 1e-3) / 1e9
    out = {
        "metric": "aggregate HBM GB/s (and % of peak) executing AllReduce/AllToAll GC3-IR",
        "metric_definition": "algorithmic bytes of one run / mean kernel time; % of peak in frac_of_hbm_peak and roofline.frac",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(mean_ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "f16": "f16", "bf16": "bf16"}[table[args.workload].dtype], "data": "synthetic",
        "config": {"workload": args.workload, "ranks": head["ranks"], "bytes_per_rank": head["bytes_per_rank"],
                   "grid": head["grid"], "team_width": head["team_width"], "wg_size": head["wg_size"],
                   "tile_bytes": head["tile_bytes"], "fifo_slots": head["fifo_slots"],
                   "plan": "chosen by gc3_comm_tune at set-up" if tune else "planner default",
                   "timing": "HIP events around each run on the launch stream; inputs restored outside the window"},
        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "per_rank_algbw_GBps": head["per_rank_algbw_GBps"],
        "untuned_plan": untuned,
        "ms_per_step_min": round(min_ms, 5),
        "ms_per_step_back_to_back_wall": round(wall_ms, 5),
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC.get(args.workload),
                     "kernel": "gc3_interpreter", "algorithmic_bytes_per_launch": alg_bytes},
        "cpu_baseline": cpu,
        "parity_vs_oracle": parity,
        "paper_context": "paper reports speedups only: up to 1.9x over NCCL ring AllReduce (8xA100 node), "
                         "up to 1.3x over hand-optimised Two-Step AllToAll (16 nodes, 256xA100); not comparable",
        "workloads": sweep,
    }
    if args.size_sweep:
        out["allreduce_size_sweep"] = size_sweep(min(args.steps, 30), min(args.warmup, 10), tune, cfg)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
