#!/usr/bin/env python3
"""Throughput of the block-decomposed Jacobi hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--no-cpu-baseline]

Workload (default C3): 2-D 5-point Jacobi, 16384 x 16384 fp64 interior, 8 x 8 tiles of
2048 x 2048 with halo exchange every iteration, boundary x^2 - y^2 on the unit square,
interior uniform in [-1, 1) (seeded, synthetic), residual norm every 10 iterations.

One STEP = one residual period of the workload = `residual_every` Jacobi iterations
(each: halo pack/unpack between all neighbouring tiles + 5-point update of every tile)
followed by one residual-norm reduction.  The default K = 20 steps is the workload's
whole schedule (200 iterations, 20 residuals).  Inputs are resident in device memory
before the clock starts; nothing is copied to the host inside the timed region.

Prints ONE JSON line.  `value` = interior points x iterations / wall time of the K timed
steps (GLUP/s: 1e9 lattice-point updates per second), everything included.
`roofline` describes the dominant kernel (the update sweep): algorithmic bytes per launch
divided by its mean launch duration, measured with HIP events around every update launch
of K timed steps, against the 8 TB/s HBM peak.  The K steps are timed twice: once clean
(`value`) and once with the events recorded (`roofline.value_with_events`; the launch durations
come from this region).
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload on this
machine's host cores (a baseline for context, not a target); the residual norms it returns are
compared with the GPU's over the same steps (`residuals_match_oracle_1e-12`), so every line
this program prints has checked its own output.  `other_workloads` carries the whole schedules of
the remaining workload shapes (C1, C2, C4, C5), measured the same way in the same run.
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

HBM_PEAK_GBS = 8000.0  # MI355X published peak

# HBM-side bytes per update launch (FETCH_SIZE + WRITE_SIZE, each scaled by what the same
# counter reads for the plain copy kernel of known size), from profiles/sweep2d_update_C3.md,
# profiles/sweep3d_update_C4.md and profiles/sweep3d_update_P1.md.  Valid only for the library's default options on that
# workload; otherwise reported as null.
MEASURED_TRAFFIC_BYTES = {"C3": 4589190778, "C4": 2412187863, "P1": 14467560021}
TRAFFIC_SOURCE = {"C3": "profiles/sweep2d_update_C3.md", "C4": "profiles/sweep3d_update_C4.md",
                  "P1": "profiles/sweep3d_update_P1.md"}

# The paper gives no absolute figure for its Jacobi proxy (Sec. VI-C); what it does state, as context only:
PAPER_CONTEXT = ("paper Sec. VI-C, Jacobi3D on a 1024x1024x768 domain: up to 40 % (strong scaling) / up to 30 % (weak "
                 "scaling) shorter run time than OpenMPI+CUDA on up to 16 nodes, each 2x Xeon Gold 6130 + 4x Tesla V100, "
                 "attributed to overlapping messages, transfers and kernels; no absolute times, rates, precision or "
                 "iteration counts are given, so there is no baseline figure for this metric")


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def algorithmic_bytes_per_update(w, esize: int, fused: bool) -> int:
    """Bytes one update launch must move: every tile reads its interior plus the face
    halo cells once and writes its interior once (16 B per point in fp64 plus the halo
    ring); with the fused halo push it also writes one copy of every inter-tile edge cell."""
    import math
    tile = [d // t for d, t in zip(w.dims, w.tiles)]
    ntiles = math.prod(w.tiles)
    interior = math.prod(tile)
    faces = sum(2 * interior // s for s in tile)          # halo cells read per tile
    total = ntiles * esize * (2 * interior + faces)
    if fused:
        pairs_cells = 0
        for d in range(len(tile)):
            pairs = (w.tiles[d] - 1) * (ntiles // w.tiles[d])
            pairs_cells += 2 * pairs * (interior // tile[d])
        total += esize * pairs_cells
    return total


class Schedule:
    """The step loop of one workload on one plan: W warm-up steps, then K timed steps from the same field."""

    def __init__(self, harness, torch, w, a, options=(), fuse_residual=True):
        self.h, self.torch, self.w, self.a = harness, torch, w, a
        self.every = w.residual_every
        self.fuse_residual = fuse_residual
        self.run = harness.JacobiRun(w.dims, w.tiles)
        for kv in options:
            k, v = kv.split("=")
            self.run.set_option(k, int(v))
        self.fused = bool(harness.B.jacobi_get_option(self.run.plan, "fused"))
        self.run.load(a)
        self.res_dev = None

    def steps(self, n: int) -> None:
        # Step i = `every` iterations, then the residual norm of the field they produced: n steps are ONE
        # jacobi_run call.  (The norm of step i's result is computed inside the first update of step i+1, in
        # the same pass over memory; only the last step needs the stand-alone reduction.)  With
        # --separate-residual: a jacobi_sweep and a residual_norm call per step.
        run, every, res_dev = self.run, self.every, self.res_dev
        if n <= 0:
            return
        if self.fuse_residual:
            fin = self.h.B.jacobi_run(run.plan, run.cur.data_ptr(), run.other().data_ptr(), n * every, every,
                                      res_dev.data_ptr(), int(self.torch.cuda.current_stream().cuda_stream))
            run.cur = run.a if fin == run.a.data_ptr() else run.b
        else:
            for i in range(n):
                run.sweep(every)
                run.residual_async(res_dev[i:i + 1])

    def timed(self, K: int, W: int, events: bool, reps: int = 1):
        """W warm-up steps, then `reps` times K timed steps, each time from the initial field (reloaded outside
        the clock).  With `events` a HIP event pair is recorded around every update launch of the timed steps
        (on the stream they run on).  Returns (seconds, residuals of the last repetition, summed launch ms, launches)."""
        import time
        torch, run, B = self.torch, self.run, self.h.B
        if self.res_dev is None or self.res_dev.numel() < max(K, W, 1):
            self.res_dev = torch.zeros(max(K, W, 1), dtype=torch.float64, device="cuda")
        run.set_option("profile", 1 if events else 0)
        self.steps(W)                              # also creates the events outside the timed region
        if events:
            B.jacobi_profile_read(run.plan)        # drop the warm-up launches from the record
        total, ms, n = 0.0, 0.0, 0
        for _ in range(reps):
            run.load(self.a)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.steps(K)
            torch.cuda.synchronize()
            total += time.perf_counter() - t0
            if events:
                m, c = B.jacobi_profile_read(run.plan)
                ms, n = ms + m, n + c
        run.set_option("profile", 0)
        return total, self.res_dev[:K].cpu().tolist(), ms, n

    def close(self):
        self.run.close()


def other_workload(harness, torch, gen, name: str) -> dict:
    """Whole schedule of one of the other workload shapes with the library's defaults: throughput (clean
    run), and the update kernel's launch duration from HIP events (second run)."""
    import math
    w = gen.WORKLOADS[name]
    a = gen.generate(w)
    sch = Schedule(harness, torch, w, a)
    try:
        K = w.iters // w.residual_every
        # launch-bound toy shapes: repeat the schedule so that the timed region is tens of milliseconds
        reps = max(1, min(50, int(2e8 // (w.points * w.iters))))
        dt, res, _, _ = sch.timed(K, 1, events=False, reps=reps)
        _, _, ms, n = sch.timed(K, 1, events=True, reps=reps)
        # algorithmic bytes of the iterations one launch advances (1 by default; on grids small enough to stay
        # on-chip one launch runs the whole call, and the figure is no longer a statement about HBM)
        iters_per_launch = w.iters * reps / max(n, 1)
        bytes_per_launch = algorithmic_bytes_per_update(w, 8, sch.fused) * iters_per_launch
        avg_ms = ms / max(n, 1)
        gbs = bytes_per_launch / (avg_ms * 1e-3) / 1e9 if n else 0.0
        return {
            "workload": f"{len(w.dims)}-D {'x'.join(map(str, w.dims))} fp64, {'x'.join(map(str, w.tiles))} tiles, "
                        f"{w.iters} iterations, residual every {w.residual_every}",
            "value": round(float(w.points) * w.iters * reps / dt / 1e9, 3),
            "unit": "GLUP/s",
            "ms_per_step": round(dt / (K * reps) * 1e3, 5),
            "ms_per_iteration": round(dt / (w.iters * reps) * 1e3, 6),
            "avg_launch_ms": round(avg_ms, 6),
            "launches_timed": n,
            "iterations_per_launch": round(iters_per_launch, 3),
            "frac": round(gbs / HBM_PEAK_GBS, 4),
            "last_residual": res[-1] if res else None,
            "passes_per_call": len(harness.B.jacobi_pass_schedule(sch.run.plan, w.residual_every)),
        }
    finally:
        sch.close()
        del a


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tblock", type=int, default=12,
                    help="depth limit of the extra temporal-blocking measurement (3-D passes advance 2 iterations)")
    ap.add_argument("--no-temporal-blocking", action="store_true",
                    help="skip the extra measurement with several iterations per pass")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the compact block with the other workload shapes")
    ap.add_argument("--tasks", default="", help="G,S: also measure the schedule executed as tasks of G tiles over "
                    "S streams (jacobi_sweep_tasks), e.g. 1,16; off by default")
    ap.add_argument("--separate-residual", action="store_true",
                    help="compute every residual with the stand-alone reduction pass")
    ap.add_argument("--option", action="append", default=[], help="key=value passed to jacobi_set_option")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on ONE GPU (tiles of one device stand in for a node's share "
              "of blocks); --gpus N with N > 1 is not supported", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import jacobi_inputs as gen
    from paper_2210_01238_amd import harness

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP library has no CPU path", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)

    w = gen.WORKLOADS[args.workload]
    every = w.residual_every
    K, W = args.steps, args.warmup

    t0 = time.perf_counter()
    a = gen.generate(w)
    t_gen = time.perf_counter() - t0
    sch = Schedule(harness, torch, w, a, args.option, fuse_residual=not args.separate_residual)
    run, fused, fuse_residual = sch.run, sch.fused, sch.fuse_residual

    # Two timed regions over the same K steps: one clean (`value`), one carrying the event pairs the
    # roofline figure is computed from (its own throughput is reported beside it: the events cost about
    # 1 % on the 0.7 ms launches of the default workload, far more on launch-bound ones).
    elapsed, residuals, _, _ = sch.timed(K, W, events=False)
    elapsed_ev, _, upd_ms, upd_n = sch.timed(K, W, events=True)
    lups = float(w.points) * every * K
    glups = lups / elapsed / 1e9
    esize = 8
    # one launch is one iteration - except on small 2-D grids, where the library runs a whole block of
    # iterations in one launch and the bytes are no longer a statement about HBM
    iters_per_launch = every * K / max(upd_n, 1)
    bytes_per_launch = int(algorithmic_bytes_per_update(w, esize, fused) * iters_per_launch)
    avg_ms = upd_ms / max(upd_n, 1)
    achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9 if upd_n else 0.0

    # optional temporal blocking (several iterations per pass over memory), reported separately
    tb = None
    if not args.no_temporal_blocking:
        run.set_option("tblock", args.tblock)
        tb_elapsed, tb_res, _, _ = sch.timed(K, W, events=False)
        _, _, tb_ms, tb_n = sch.timed(K, W, events=True)
        run.set_option("tblock", 1)
        tb = {
            "tblock": args.tblock,
            "value": round(lups / tb_elapsed / 1e9, 3),
            "unit": "GLUP/s",
            "ms_per_step": round(tb_elapsed / K * 1e3, 4),
            "avg_pass_ms": round(tb_ms / max(tb_n, 1), 5),
            "passes_timed": tb_n,
            "iterations_per_pass": round(every * K / max(tb_n, 1), 3),
            "residuals_match_single_step_1e-12": all(abs(x - y) <= 1e-12 * abs(y) for x, y in zip(tb_res, residuals)),
            "note": "same iterations, bit-identical grids; a pass advances up to `tblock` iterations (3-D: up to 4) "
                    "and reads the rim it needs from the neighbouring tiles itself instead of a halo exchange "
                    "per iteration",
        }

    # optional: the same schedule executed as per-tile tasks over several streams (the paper's execution model)
    tasks = None
    if args.tasks and fused:
        grp, nstr = (int(x) for x in args.tasks.split(","))
        res_dev = sch.res_dev

        def task_steps(n: int) -> None:
            for i in range(n):
                run.sweep_tasks(every, grp, nstr)
                run.residual_async(res_dev[i:i + 1])

        task_steps(W)
        run.load(a)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        task_steps(K)
        torch.cuda.synchronize()
        t_tasks = time.perf_counter() - t0
        t_res = res_dev[:K].cpu().tolist()
        tasks = {
            "tiles_per_task": grp,
            "streams": nstr,
            "tasks_per_iteration": -(-int(np.prod(w.tiles)) // grp),
            "value": round(lups / t_tasks / 1e9, 3),
            "unit": "GLUP/s",
            "ms_per_step": round(t_tasks / K * 1e3, 4),
            "residuals_match_single_launch_1e-12": all(abs(x - y) <= 1e-12 * abs(y) for x, y in zip(t_res, residuals)),
            "note": "same iterations, bit-identical grids; every group of tiles is a task per iteration, ordered "
                    "only by events on the tasks of the previous iteration that it reads from",
        }

    # practical ceiling: a plain streaming copy of one grid into the other (same bytes in and out)
    src_g, dst_g = run.cur, run.other()
    st = int(torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        harness.B.jacobi_stream_copy(dst_g.data_ptr(), src_g.data_ptr(), run.nbytes, st)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        harness.B.jacobi_stream_copy(dst_g.data_ptr(), src_g.data_ptr(), run.nbytes, st)
    torch.cuda.synchronize()
    copy_gbs = 2.0 * run.nbytes * 20 / (time.perf_counter() - t0) / 1e9
    sch.close()

    traffic = MEASURED_TRAFFIC_BYTES.get(w.name) if not args.option else None
    out = {
        "metric": "Jacobi GLUP/s (lattice updates/sec) + % of HBM roofline, 1 MI355X",
        "value": round(glups, 3),
        "unit": "GLUP/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(elapsed / K * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: {len(w.dims)}-D Jacobi {'x'.join(map(str, w.dims))} fp64, "
                        f"{'x'.join(map(str, w.tiles))} tiles, halo exchange every iteration, "
                        f"residual every {every} iterations",
            "iterations_per_step": every,
            "iterations_timed": every * K,
            "residual_calls_timed": K,
            "fused_halo_push": fused,
            "residual_fused_into_update": fuse_residual,
            "options": args.option,
            "last_residual": residuals[-1] if residuals else None,
            "input_generation_s": round(t_gen, 2),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": ("resident2d_kernel<double> (a block of iterations per launch: the grid stays in registers, so the "
                       "bytes counted never cross the HBM interface)") if iters_per_launch > 1.5 else
                      (("sweep2d_kernel<double, update>" if len(w.dims) == 2 else "sweep3d_kernel<double, update>")
                       + " (the launches timed include the first update of the run, which reads the neighbouring tiles' edge "
                         "cells instead of halo cells, and each step's first, which also accumulates the residual)"),
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": traffic,
            "traffic_source": (f"{TRAFFIC_SOURCE[w.name]} (rocprofv3 FETCH_SIZE + WRITE_SIZE of an earlier run of this "
                               "command, not measured in this run)") if traffic is not None else None,
            "bytes_per_launch": bytes_per_launch,
            "avg_launch_ms": round(avg_ms, 5),
            "launches_timed": upd_n,
            "iterations_per_launch": round(iters_per_launch, 3),
            "whole_step_frac": round((16.0 * glups) / HBM_PEAK_GBS, 4),
            "value_with_events": round(lups / elapsed_ev / 1e9, 3),
            "stream_copy_gbs": round(copy_gbs, 1),
        },
        "paper_context": PAPER_CONTEXT,
    }

    if tb is not None:
        out["temporal_blocking"] = tb
    if tasks is not None:
        out["task_execution"] = tasks

    if not args.no_cpu_baseline:
        import oracle
        oracle.build()
        n_steps_cpu = min(K, 16) if K > 0 else 1
        threads = oracle.num_threads()
        t0 = time.perf_counter()
        _, cpu_res = oracle.run(a, every * n_steps_cpu, every)
        t_cpu = time.perf_counter() - t0
        # the same loops on ONE thread, over a shorter sample (one step)
        oracle.set_threads(1)
        t0 = time.perf_counter()
        oracle.run(a, every, every)
        t_serial = time.perf_counter() - t0
        oracle.set_threads(threads)
        rate = float(w.points) * every * n_steps_cpu / t_cpu / 1e9
        rate_serial = float(w.points) * every / t_serial / 1e9
        match = len(cpu_res) == n_steps_cpu and all(abs(g - o) <= 1e-12 * abs(o) for g, o in zip(residuals, cpu_res))
        out["cpu_baseline"] = {
            "value": round(rate, 4),
            "unit": "GLUP/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"first {n_steps_cpu} steps ({every * n_steps_cpu} iterations + {n_steps_cpu} residual norms) "
                      f"of the same {w.name} field, full grid; update loops on all threads, residual sums serial; "
                      f"{t_cpu:.1f} s",
            "implied_host_gbs": round(16.0 * rate, 1),
            "serial": {"value": round(rate_serial, 4), "unit": "GLUP/s", "cores": 1,
                       "sample": f"first step ({every} iterations + 1 residual norm) of the same field; {t_serial:.1f} s"},
            "nproc": os.cpu_count(),
            "omp_num_threads": os.environ.get("OMP_NUM_THREADS"),
            "cpu_model": cpu_model(),
            "residuals_compared": n_steps_cpu,
        }
        out["residuals_match_oracle_1e-12"] = bool(match)
        if not match:
            print("bench.py: GPU residuals differ from the oracle's: " + repr(list(zip(residuals, cpu_res))), file=sys.stderr)
    del a

    if not args.no_other_workloads:
        out["other_workloads"] = {name: other_workload(harness, torch, gen, name)
                                  for name in ("C1", "C2", "C4", "C5") if name != w.name}
    print(json.dumps(out), flush=True)
    return 0 if out.get("residuals_match_oracle_1e-12", True) else 1


if __name__ == "__main__":
    sys.exit(main())
