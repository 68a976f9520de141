"""GPU parity of the all-iterations-in-one-launch path for small 2-D grids (option resident = 1, the
library's default): the whole jacobi_sweep call runs inside one kernel, the grid stays in registers
and the workgroups meet at a device-memory barrier every few iterations.  Same bar as everywhere:
fp64 grids bit-identical to the CPU oracle, fp32 within 1e-5*max|u|, residuals within 1e-12 / 1e-5."""
import numpy as np
import pytest

import jacobi_inputs as gen
from parity_util import random_padded
from test_parity_gpu import check, run_case

pytestmark = pytest.mark.gpu


def schedule(H, dims, tiles, iters, dtype=np.float64, **opts):
    r = H.JacobiRun(dims, tiles, dtype, **opts)
    try:
        return H.B.jacobi_pass_schedule(r.plan, iters)
    finally:
        r.close()


CASES = [
    # (interior dims, tiles, iters, residual_every)
    ((256, 256), (1, 1), 100, 100),      # the launch-bound workload shape: 7 phases on several workgroups
    ((256, 256), (4, 4), 37, 10),        # same grid cut into 16 tiles: rows and columns cross tile borders
    ((46, 256), (1, 1), 40, 8),          # one workgroup holds everything (46 rows + 2 ring rows = 16 x 3)
    ((47, 256), (1, 1), 40, 8),          # one row more: two workgroups
    ((62, 128), (1, 1), 40, 8),          # rows of 1 KiB: 4 rows per wavefront, 62 + 2 = 64
    ((63, 128), (1, 1), 40, 8),
    ((1, 2), (1, 1), 5, 1),
    ((2, 2), (1, 1), 5, 1),
    ((300, 70), (1, 1), 23, 23),         # ragged width (35 lanes), one segment
    ((300, 70), (5, 7), 23, 5),          # tiles 60 x 10
    ((96, 200), (3, 2), 13, 4),          # two segments, ragged second one, tile seam at column 100
    ((1000, 130), (8, 1), 50, 25),       # 1000 rows: ~40 workgroups
    ((700, 256), (7, 2), 33, 11),
    ((5000, 128), (4, 1), 20, 20),       # 114 workgroups at the barrier
    ((40, 36), (1, 18), 6, 2),           # tiles two columns wide
    ((36, 40), (36, 1), 6, 2),           # tiles one row high
]


@pytest.mark.parametrize("dims,tiles,iters,every", CASES)
def test_resident_fp64_bit_exact(H, oracle_mod, dims, tiles, iters, every):
    assert len(schedule(H, dims, tiles, every, resident=1)) < every or every == 1
    a = random_padded(dims, seed=sum(dims) + iters)
    check(*run_case(H, oracle_mod, a, tiles, iters, every, resident=1))


def run_in_one_call(H, a, tiles, iters, every, **opts):
    r = H.JacobiRun([n - 2 for n in a.shape], tiles, a.dtype, **opts)
    try:
        r.load(a)
        res = r.run(iters, every, fuse_residual=True)
        return r.fetch(), res
    finally:
        r.close()


@pytest.mark.parametrize("dims,tiles,iters,every", CASES)
def test_resident_run_takes_its_residuals_from_the_launches(H, oracle_mod, dims, tiles, iters, every):
    """jacobi_run on these shapes: every block of iterations is one launch that also delivers the norm of the
    grid it produced (the rows next to a workgroup's own must then still be exact after the deepest phase)."""
    a = random_padded(dims, seed=sum(dims) + iters + 1)
    ref, ref_res = oracle_mod.run(a, iters, every)
    out, res = run_in_one_call(H, a, tiles, iters, every, resident=1)
    check(out, res, ref, ref_res)
    out2, res2 = run_in_one_call(H, a, tiles, iters, every, resident=1)
    assert res2 == res and np.array_equal(out2, out)                 # same bits on every run


@pytest.mark.parametrize("opts", [
    dict(resident_depth=1), dict(resident_depth=2, resident_rows=1), dict(resident_depth=6, resident_rows=1),
    dict(resident_depth=7, resident_rows=1), dict(resident_depth=23), dict(resident_depth=31, resident_rows=2),
    dict(resident_rows=4), dict(),
])
def test_resident_run_with_every_phase_geometry(H, oracle_mod, opts):
    for dims, tiles, dtype in (((256, 256), (2, 2), np.float64), ((130, 100), (5, 5), np.float64),
                               ((300, 512), (3, 4), np.float32)):
        a = random_padded(dims, dtype=dtype, seed=21)
        ref, ref_res = oracle_mod.run(a, 46, 23)
        out, res = run_in_one_call(H, a, tiles, 46, 23, resident=1, **opts)
        check(out, res, ref, ref_res)


def test_resident_launch_carries_the_whole_ring_to_the_other_grid(H, oracle_mod):
    """The launch itself copies the Dirichlet ring (rows, columns, corners) to the grid it does not start from:
    that grid is filled with NaN first, and after an odd number of phases it holds the result."""
    import torch
    for dims, tiles, iters in (((256, 256), (1, 1), 20), ((40, 36), (4, 3), 3), ((700, 130), (7, 1), 15),
                               ((1, 2), (1, 1), 1)):
        a = random_padded(dims, seed=31)
        r = H.JacobiRun(dims, tiles, resident=1)
        try:
            assert len(H.B.jacobi_pass_schedule(r.plan, iters)) == 1
            r.load(a)
            r.other().view(torch.float64).fill_(float("nan"))
            r.sweep(iters)
            assert r.cur is r.b
            out = r.fetch()
        finally:
            r.close()
        ref, _ = oracle_mod.run(a, iters)
        assert np.array_equal(out, ref), dims


@pytest.mark.parametrize("dims,tiles,iters,every", [
    ((256, 256), (1, 1), 30, 10), ((256, 512), (2, 2), 30, 10), ((100, 300), (5, 3), 17, 17), ((40, 8), (2, 2), 9, 3),
])
def test_resident_fp32(H, oracle_mod, dims, tiles, iters, every):
    a = random_padded(dims, dtype=np.float32, seed=17)
    check(*run_case(H, oracle_mod, a, tiles, iters, every, resident=1))


@pytest.mark.parametrize("opts", [
    dict(resident_depth=1), dict(resident_depth=3, resident_rows=1), dict(resident_depth=5, resident_rows=2),
    dict(resident_depth=7, resident_rows=3), dict(resident_depth=24, resident_rows=4), dict(resident_depth=31),
    dict(resident_depth=23, resident_rows=3), dict(resident_depth=16),
    dict(resident_rows=1), dict(resident_rows=2), dict(resident_rows=3),
])
def test_resident_geometry_options_do_not_change_results(H, oracle_mod, opts):
    a = random_padded((256, 256), seed=5)
    check(*run_case(H, oracle_mod, a, (2, 2), 29, 29, resident=1, **opts))
    b = random_padded((90, 100), seed=6)
    check(*run_case(H, oracle_mod, b, (3, 5), 11, 4, resident=1, **opts))


def test_resident_c1_workload_stored_values_and_light_cone(H, oracle_mod):
    from test_oracle_pins import read_golden_c1
    w = gen.WORKLOADS["C1"]
    a = gen.generate(w)
    sched = schedule(H, w.dims, w.tiles, w.iters, resident=1)
    assert sum(sched) == w.iters and len(sched) <= 8                 # a handful of phases, not 100 passes
    out, res, ref, ref_res = run_case(H, oracle_mod, a, w.tiles, w.iters, w.residual_every, resident=1)
    check(out, res, ref, ref_res)
    gres, pts = read_golden_c1()
    assert abs(res[0] - gres) <= 1e-12 * gres
    for (i, j), v in pts.items():
        assert out[i, j] == v
    assert np.all(out[101:-1, 1:-1] == 0.0) and np.array_equal(out, out[:, ::-1])


def test_resident_lattice_fixed_point_and_fused_residual(H, oracle_mod):
    a = gen.lattice_field((130, 258), "i2-j2")
    out, res, ref, _ = run_case(H, oracle_mod, a, (4, 2), 6, 3, resident=1)
    assert np.array_equal(out, a) and res == [0.0, 0.0]
    # the residual of the field entering a call, delivered by jacobi_sweep_residual
    b = random_padded((200, 256), seed=8)
    ref, ref_res = oracle_mod.run(b, 24, 6)
    r = H.JacobiRun((200, 256), (2, 2), resident=1)
    try:
        r.load(b)
        res = r.run(24, 6, fuse_residual=True)
        out = r.fetch()
    finally:
        r.close()
    check(out, res, ref, ref_res)


def test_resident_selection_and_schedule(H):
    """Which plans take the path, read through jacobi_pass_schedule: with resident = 0 a pass per iteration."""
    assert schedule(H, (256, 256), (1, 1), 100, resident=0) == [1] * 100
    s = schedule(H, (256, 256), (1, 1), 100, resident=1)
    assert sum(s) == 100 and max(s) - min(s) <= 1 and max(s) <= 23
    assert schedule(H, (46, 256), (1, 1), 100, resident=1) == [100]                 # one workgroup: one phase
    assert schedule(H, (62, 128), (1, 1), 100, resident=1) == [100]
    assert schedule(H, (256, 258), (1, 1), 10, resident=1) == [1] * 10               # 258 columns: three segments
    assert schedule(H, (256, 516), (1, 1), 10, np.float32, resident=1) == [1] * 10
    assert schedule(H, (256, 512), (1, 1), 10, np.float32, resident=1) == [10]
    assert schedule(H, (30, 30), (1, 30), 10, resident=1) == [1] * 10                # tiles one column wide
    assert schedule(H, (16, 16, 16), (1, 1, 1), 10, resident=1) == [1] * 10          # 3-D
    assert len(schedule(H, (20000, 128), (1, 1), 10, resident=1)) == 10              # more workgroups than CUs


def test_resident_inside_a_hip_graph(H, oracle_mod):
    """The launch recorded into a HIP graph and replayed: it leaves its barrier words zeroed for the next one."""
    import torch
    w = gen.WORKLOADS["C1"]
    a = gen.generate(w)
    n = 40                                         # two phases of 20: result back in the source buffer
    r = H.JacobiRun(w.dims, w.tiles, resident=1)
    try:
        assert len(H.B.jacobi_pass_schedule(r.plan, n)) == 2
        r.load(a)
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            r.sweep(n)
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        assert np.array_equal(r.fetch(), oracle_mod.run(a, n)[0])
        src, dst = r.cur, r.other()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            fin = H.B.jacobi_sweep(r.plan, src.data_ptr(), dst.data_ptr(), n, int(torch.cuda.current_stream().cuda_stream))
        assert fin == src.data_ptr()
        for k in range(3):
            g.replay()
            torch.cuda.synchronize()
            got = r.fetch()
            torch.cuda.synchronize()
            assert np.array_equal(got, oracle_mod.run(a, 2 * n + n * k)[0]), k
    finally:
        r.close()


def test_resident_barrier_gives_up_instead_of_hanging(H, oracle_mod):
    """The grid barrier's wait is bounded.  With a spin limit of ZERO polls beyond the first, a workgroup that
    finds the others not yet arrived gives up at once: the launch must still drain, and what it then writes is
    NaN (or, if every workgroup happened to arrive in time, the right answer) - never a plausible wrong value.
    The next call, with the default limit, is correct again: the last workgroup to finish clears the barrier
    words, also after a barrier that gave up."""
    a = random_padded((256, 256), seed=9)
    ref, _ = oracle_mod.run(a, 40)
    r = H.JacobiRun((256, 256), (1, 1), resident=1, resident_spin_limit=1)
    try:
        r.load(a)
        r.sweep(40)
        out = r.fetch()
        assert np.array_equal(out, ref) or np.isnan(out[1:-1, 1:-1]).any()
        # the norm delivered by a launch that gave up is NaN as well
        r.load(a)
        res = r.run(40, 40, fuse_residual=True)
        out = r.fetch()
        ok = np.array_equal(out, ref)
        assert ok or np.isnan(out[1:-1, 1:-1]).any()
        assert np.isnan(res[0]) or (ok and abs(res[0] - oracle_mod.residual(ref)) <= 1e-12 * res[0])
        r.set_option("resident_spin_limit", 0)
        r.load(a)
        r.sweep(40)
        assert np.array_equal(r.fetch(), ref)
        r.load(a)
        res = r.run(40, 40, fuse_residual=True)
        assert np.array_equal(r.fetch(), ref) and abs(res[0] - oracle_mod.residual(ref)) <= 1e-12 * res[0]
    finally:
        r.close()
