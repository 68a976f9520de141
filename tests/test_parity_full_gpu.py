"""GPU parity at the full workload sizes, in the launch configuration the benchmark
times (default options).  The oracle cannot run the large grids for hundreds of
iterations in test time, so each workload is checked three ways:
  (1) the whole grid, bit for bit, after a few iterations (oracle runs the full grid);
  (2) sampled windows after ALL iterations: a Jacobi value after k iterations depends
      only on initial values within distance k, so the oracle recomputes windows around
      chosen points (tile junctions, tile edges, domain corners) exactly;
  (3) properties that hold at any size: discrete maximum principle, strictly decreasing
      residuals; and the schedule's first residual (after `residual_every` iterations, which
      the oracle can still run on the whole grid) against the oracle's.
The schedule is the benchmark's: blocks of `residual_every` iterations, each residual taken
from the first update of the next block (jacobi_sweep_residual), the last one stand-alone.
"""
import numpy as np
import pytest

import jacobi_inputs as gen
from parity_util import oracle_window

pytestmark = pytest.mark.gpu


def windows_for(w, iters, extra=12):
    """Index boxes (padded coordinates) whose exact part covers: the junction of tiles
    nearest the domain centre, the low corner of the domain, and the high corner."""
    pd = [d + 2 for d in w.dims]
    tile = [d // t for d, t in zip(w.dims, w.tiles)]
    boxes = []
    # junction: first cell of tile (T/2) in every dim is at padded index (T/2)*tile + 1
    c = [(t // 2) * s + 1 for t, s in zip(w.tiles, tile)]
    lo = [max(0, x - iters - extra) for x in c]
    hi = [min(p, x + iters + extra) for x, p in zip(c, pd)]
    boxes.append((lo, hi))
    # low corner (Dirichlet ring on every low face)
    boxes.append(([0] * w.ndim, [min(p, iters + 2 * extra + 1) for p in pd]))
    # high corner
    boxes.append(([max(0, p - iters - 2 * extra - 1) for p in pd], pd))
    return boxes


def full_size_check(H, oracle, name, few, fuse_residual=True, **options):
    import torch
    w = gen.WORKLOADS[name] if isinstance(name, str) else name
    name = w.name
    a = gen.generate(w)
    amin, amax = float(a.min()), float(a.max())
    r = H.JacobiRun(w.dims, w.tiles, **options)
    try:
        r.load(a)
        # (1) whole grid after `few` iterations
        r.sweep(few)
        ref, _ = oracle.run(a, few)
        out = r.fetch()
        assert np.array_equal(out, ref), f"{name}: grid differs after {few} iterations"
        res_few = r.residual()
        ref_res = oracle.residual(ref)
        assert abs(res_few - ref_res) <= 1e-12 * ref_res
        del ref, out
        # (2)+(3) the full schedule, as the benchmark runs it
        r.load(a)
        res = r.run(w.iters, w.residual_every, fuse_residual=fuse_residual)
        assert len(res) == w.iters // w.residual_every
        assert all(res[i + 1] < res[i] for i in range(len(res) - 1)), f"{name}: residual not decreasing"
        _, first = oracle.run(a, w.residual_every, w.residual_every)
        assert abs(res[0] - first[0]) <= 1e-12 * first[0], f"{name}: first residual {res[0]} vs oracle {first[0]}"
        g = r.fetch_device()
        inner = g[tuple(slice(1, -1) for _ in w.dims)]
        tol = 0.0 if w.ndim == 2 else 4 * np.spacing(max(abs(amin), abs(amax)))
        assert float(inner.min()) >= amin - tol and float(inner.max()) <= amax + tol
        for lo, hi in windows_for(w, w.iters):
            u, valid = oracle_window(oracle, w, lo, hi, w.iters)
            sl = tuple(slice(l + v.start, l + v.stop) for l, v in zip(lo, valid))
            got = g[sl].cpu().numpy()
            assert got.size > 0
            assert np.array_equal(got, u[valid]), f"{name}: window {lo}..{hi} differs"
        # large grids cap the workgroups per CU through an LDS request: the occupancy query must have confirmed it
        assert H.B.jacobi_get_option(r.plan, "lds_limit_failed") == 0 and H.B.jacobi_get_option(r.plan, "num_cu") > 0
    finally:
        r.close()


def test_full_C3_16384sq_8x8(H, oracle_mod):
    full_size_check(H, oracle_mod, "C3", few=3)


def test_full_C3_two_iterations_per_pass(H, oracle_mod):
    full_size_check(H, oracle_mod, "C3", few=3, tblock=2)


def test_full_C5_two_iterations_per_pass(H, oracle_mod):
    full_size_check(H, oracle_mod, "C5", few=5, tblock=2)


def test_full_C3_eight_iterations_per_pass(H, oracle_mod):
    full_size_check(H, oracle_mod, "C3", few=3, tblock=8)


def test_full_C2_eight_iterations_per_pass(H, oracle_mod):
    full_size_check(H, oracle_mod, "C2", few=10, tblock=8)


def test_full_C3_separate_exchange_and_residual_kernels(H, oracle_mod):
    full_size_check(H, oracle_mod, "C3", few=2, fuse_residual=False, fused=0)


def test_full_C5_8192sq_64x64(H, oracle_mod):
    full_size_check(H, oracle_mod, "C5", few=5)


def test_full_C4_512cube_4x4x4(H, oracle_mod):
    full_size_check(H, oracle_mod, "C4", few=4)


def test_full_C4_blocked_passes_of_three_and_two_iterations(H, oracle_mod):
    full_size_check(H, oracle_mod, "C4", few=5, tblock=3)      # 5 = 3 + 2; 10 per period = 3 + 3 + 2 + 2


def test_full_C4_two_iterations_per_pass(H, oracle_mod):
    full_size_check(H, oracle_mod, "C4", few=4, tblock=2)


def test_full_C2_4096sq_4x4(H, oracle_mod):
    full_size_check(H, oracle_mod, "C2", few=10)


def test_full_P1_paper_domain_1024x1024x768(H, oracle_mod):
    full_size_check(H, oracle_mod, "P1", few=2)


def test_full_P1_paper_domain_blocked_passes(H, oracle_mod):
    full_size_check(H, oracle_mod, "P1", few=3, tblock=8)


@pytest.mark.parametrize("name,few,group", [("C3", 3, 1), ("C4", 4, 4)])
def test_full_size_task_execution(H, oracle_mod, name, few, group):
    """The task path at full size: whole grid, bit for bit, after a few iterations."""
    w = gen.WORKLOADS[name]
    a = gen.generate(w)
    ref, _ = oracle_mod.run(a, few)
    r = H.JacobiRun(w.dims, w.tiles)
    try:
        r.load(a)
        r.sweep_tasks(few, group, 16)                 # tasks over 16 streams
        assert np.array_equal(r.fetch(), ref), f"{name}: task execution differs"
    finally:
        r.close()


@pytest.mark.parametrize("name,opts,n", [("C4", {}, 4), ("C3", dict(tblock=8), 16), ("C3", {}, 2)])
def test_full_size_sweep_in_a_hip_graph(H, name, opts, n):
    """On large grids some launches request LDS only to limit the workgroups per CU (and one kernel
    has to be allowed the larger request first).  Recorded into a HIP graph they must behave the
    same: every replay equals the eager run, bit for bit."""
    import torch
    w = gen.WORKLOADS[name]
    a = gen.generate(w)
    r = H.JacobiRun(w.dims, w.tiles, **opts)
    try:
        r.load(a)
        r.sweep(3 * n)
        eager3 = r.fetch_device().clone()
        r.load(a)
        r.sweep(2 * n)
        eager2 = r.fetch_device().clone()
        r.load(a)
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            r.sweep(n)                                # eager, on the side stream
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        src, dst = r.cur, r.other()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            fin = H.B.jacobi_sweep(r.plan, src.data_ptr(), dst.data_ptr(), n,
                                   int(torch.cuda.current_stream().cuda_stream))
        assert fin == src.data_ptr()                  # an even number of passes
        for expect in (eager2, eager3):               # two replays with eager work in between
            g.replay()
            torch.cuda.synchronize()
            got = r.fetch_device()
            torch.cuda.synchronize()
            assert torch.equal(got, expect), f"{name} {opts}: replay differs from the eager run"
    finally:
        r.close()


# Grids of more than 1 GiB - from that size on the launches limit the workgroups per CU - whose extents
# divide by nothing convenient: ragged strips, row groups, plane blocks and column segments.
LARGE_RAGGED_2D = gen.WORKLOADS["C3"].scaled((11000, 12200), (5, 4), iters=24, residual_every=8)      # tiles 2200 x 3050
LARGE_RAGGED_3D = gen.WORKLOADS["C4"].scaled((250, 520, 1060), (2, 4, 5), iters=10, residual_every=5)  # tiles 125 x 130 x 212


def test_large_ragged_2d(H, oracle_mod):
    full_size_check(H, oracle_mod, LARGE_RAGGED_2D, few=2)


def test_large_ragged_2d_blocked_passes(H, oracle_mod):
    full_size_check(H, oracle_mod, LARGE_RAGGED_2D, few=3, tblock=8)


def test_large_ragged_3d(H, oracle_mod):
    full_size_check(H, oracle_mod, LARGE_RAGGED_3D, few=2)


def test_large_ragged_3d_blocked_passes(H, oracle_mod):
    full_size_check(H, oracle_mod, LARGE_RAGGED_3D, few=3, tblock=4)


# ---- 32-bit limits: per-lane byte offsets inside a row of tiles are 32-bit in the blocked-pass kernels ----------
def whole_grid_after(H, oracle, w, few, **options):
    """Whole grid, bit for bit, after `few` iterations; returns the pass schedule that ran."""
    a = gen.generate(w)
    ref, _ = oracle.run(a, few)
    r = H.JacobiRun(w.dims, w.tiles, **options)
    try:
        sched = H.B.jacobi_pass_schedule(r.plan, few)
        r.load(a)
        del a
        r.sweep(few)
        got = r.fetch()
        assert np.array_equal(got, ref), f"{w.dims} {options}: grid differs after {few} iterations"
        res, ref_res = r.residual(), oracle.residual(ref)
        assert abs(res - ref_res) <= 1e-12 * ref_res
        return sched
    finally:
        r.close()


@pytest.mark.parametrize("options,few", [({}, 2), (dict(tblock=8), 6)])
def test_2d_grid_above_4_GiB(H, oracle_mod, options, few):
    """24576^2 fp64 = 4.8 GB per grid: every element offset beyond 2^32 bytes is exercised (single steps and
    blocked passes; a row of tiles is 1.2 GB, so the blocked kernels can address it)."""
    w = gen.WORKLOADS["C3"].scaled((24576, 24576), (4, 4), iters=few, residual_every=few)
    sched = whole_grid_after(H, oracle_mod, w, few, **options)
    assert sched == ([few] if options else [1] * few)


def test_row_of_tiles_of_2_GiB_falls_back_to_the_two_step_kernel(H, oracle_mod):
    """8192 x 65536 in 2 x 2 tiles: a row of tiles is 2.15 GB, beyond the 32-bit per-lane offsets of the pipelined
    blocked passes, so with tblock = 8 the planner must fall back to the two-step kernel (64-bit addressing) and
    single steps (the schedule says so), and the result must still be exact."""
    w = gen.WORKLOADS["C3"].scaled((8192, 65536), (2, 2), iters=5, residual_every=5)
    sched = whole_grid_after(H, oracle_mod, w, 5, tblock=8)
    assert sched == [2, 2, 1]
    # the same domain cut into lower tiles fits again: one pass of 5
    r = H.JacobiRun((8192, 65536), (4, 2), tblock=8)
    try:
        assert H.B.jacobi_pass_schedule(r.plan, 5) == [5]
    finally:
        r.close()
