"""Randomised GPU parity: seeded random shapes, tilings, iteration counts, residual cadences
and option combinations, each compared bit for bit (fp64) with the CPU oracle.  The case list
is fixed by the seed, so a failure names a reproducible case."""
import numpy as np
import pytest

from parity_util import random_padded
from test_parity_gpu import check, run_case

pytestmark = pytest.mark.gpu


def divisors(n):
    return [d for d in range(1, n + 1) if n % d == 0]


def make_cases(ndim, count, seed, blocked_3d=False):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(count):
        if ndim == 2:
            dims = (int(rng.integers(1, 200)), int(rng.integers(1, 700)))
        else:
            dims = (int(rng.integers(1, 24)), int(rng.integers(1, 40)), int(rng.integers(1, 300)))
        tiles = tuple(int(rng.choice(divisors(d))) for d in dims)
        iters = int(rng.integers(1, 20))
        every = int(rng.integers(1, iters + 1))
        opts = dict(fused=int(rng.integers(0, 2)),
                    rows_per_strip=int(rng.choice([0, 0, 1, 2, 3, 5, 8, 16, 33, 128])),
                    unroll=int(rng.choice([0, 0, 1, 2, 4, 8] + ([16] if ndim == 2 else []))),
                    xcd_chunk=int(rng.choice([0, 1, 2, 8, 8, 64])),
                    nontemporal=int(rng.choice([0, 1, 2])))
        if ndim == 2:
            opts["tblock"] = int(rng.choice([1, 1, 2, 3, 4, 5, 6, 7, 8, 10, 12]))
        else:
            opts["rows_per_wave"] = int(rng.choice([0, 1, 2, 4]))
            if blocked_3d:
                opts["tblock"] = int(rng.choice([2, 3, 4, 8]))
                opts["cooperative"] = int(rng.integers(0, 2))
        fuse_res = bool(rng.integers(0, 2))
        cases.append((dims, tiles, iters, every, opts, fuse_res))
    return cases


def run_random(H, oracle, case, seed):
    dims, tiles, iters, every, opts, fuse_res = case
    a = random_padded(dims, seed=seed)
    if not fuse_res:
        return check(*run_case(H, oracle, a, tiles, iters, every, **opts))
    r = H.JacobiRun(dims, tiles, **opts)
    try:
        r.load(a)
        res = r.run(iters, every, fuse_residual=True)
        out = r.fetch()
    finally:
        r.close()
    ref, ref_res = oracle.run(a, iters, every)
    check(out, res, ref, ref_res)


@pytest.mark.parametrize("n,case", list(enumerate(make_cases(2, 120, 20221001))))
def test_random_2d(H, oracle_mod, n, case):
    run_random(H, oracle_mod, case, 1000 + n)


@pytest.mark.parametrize("n,case", list(enumerate(make_cases(3, 80, 20221002))))
def test_random_3d(H, oracle_mod, n, case):
    run_random(H, oracle_mod, case, 2000 + n)


@pytest.mark.parametrize("n,case", list(enumerate(make_cases(3, 80, 20221003, blocked_3d=True))))
def test_random_3d_blocked(H, oracle_mod, n, case):
    run_random(H, oracle_mod, case, 3000 + n)


def make_task_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for n in range(count):
        if n % 2 == 0:
            dims = (int(rng.integers(1, 120)), int(rng.integers(1, 400)))
        else:
            dims = (int(rng.integers(1, 20)), int(rng.integers(1, 30)), int(rng.integers(1, 200)))
        tiles = tuple(int(rng.choice(divisors(d))) for d in dims)
        ntiles = int(np.prod(tiles))
        group = int(rng.integers(1, ntiles + 2))
        streams = int(rng.integers(1, 17))
        iters = int(rng.integers(1, 12))
        opts = dict(rows_per_strip=int(rng.choice([0, 0, 1, 3, 8, 33])), xcd_chunk=int(rng.choice([0, 1, 8])))
        cases.append((dims, tiles, group, streams, iters, opts))
    return cases


@pytest.mark.parametrize("n,case", list(enumerate(make_task_cases(60, 20221004))))
def test_random_task_execution(H, oracle_mod, n, case):
    """jacobi_sweep_tasks on random shapes, tilings, task sizes and stream counts."""
    dims, tiles, group, streams, iters, opts = case
    a = random_padded(dims, seed=4000 + n)
    r = H.JacobiRun(dims, tiles, **opts)
    try:
        r.load(a)
        r.sweep_tasks(iters, group, streams)
        out = r.fetch()
        res = [r.residual()]
    finally:
        r.close()
    ref, ref_res = oracle_mod.run(a, iters, iters)
    check(out, res, ref, ref_res)


def make_medium_cases(count, seed):
    """Shapes large enough for several strips, column segments and row groups per tile, with few tiles."""
    rng = np.random.default_rng(seed)
    cases = []
    for n in range(count):
        if n % 2 == 0:
            dims = (int(rng.integers(300, 2500)), int(rng.integers(300, 4000)))
        else:
            dims = (int(rng.integers(20, 140)), int(rng.integers(20, 200)), int(rng.integers(50, 700)))
        tiles = tuple(int(rng.choice([d for d in divisors(x) if d <= 8])) for x in dims)
        iters = int(rng.integers(1, 26))
        every = int(rng.integers(1, iters + 1))
        opts = dict(fused=int(rng.integers(0, 2)), tblock=int(rng.choice([1, 2, 3, 4, 8, 10, 12])),
                    rows_per_strip=int(rng.choice([0, 0, 0, 7, 32, 100])), unroll=int(rng.choice([0, 0, 1, 2, 4])),
                    xcd_chunk=int(rng.choice([0, 0, 1, 16])))
        if len(dims) == 3:
            opts["cooperative"] = int(rng.integers(0, 2))
            opts["rows_per_wave"] = int(rng.choice([0, 0, 1, 2, 4]))
        cases.append((dims, tiles, iters, every, opts, bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("n,case", list(enumerate(make_medium_cases(40, 20221005))))
def test_random_medium_sizes(H, oracle_mod, n, case):
    run_random(H, oracle_mod, case, 5000 + n)


def make_resident_cases(count, seed):
    """Shapes the all-iterations-in-one-launch path takes (rows of at most 2 KiB, tile widths a multiple of
    16 bytes), with random phase depths and rows per wavefront."""
    rng = np.random.default_rng(seed)
    cases = []
    for n in range(count):
        f32 = n % 4 == 3
        nv = 4 if f32 else 2
        width = nv * int(rng.integers(1, 128 + 1))
        dims = (int(rng.integers(1, 1500)), width)
        ty = int(rng.choice(divisors(dims[0])))
        tx = int(rng.choice([d for d in divisors(width) if (width // d) % nv == 0]))
        iters = int(rng.integers(1, 70))
        every = int(rng.integers(1, iters + 1))
        opts = dict(resident=1, resident_depth=int(rng.choice([0, 0, 1, 2, 5, 9, 14, 20, 31])),
                    resident_rows=int(rng.choice([0, 0, 1, 2, 3, 4])))
        cases.append((dims, (ty, tx), iters, every, opts, bool(rng.integers(0, 2)), np.float32 if f32 else np.float64))
    return cases


@pytest.mark.parametrize("n,case", list(enumerate(make_resident_cases(48, 20221006))))
def test_random_resident(H, oracle_mod, n, case):
    """jacobi_sweep calls that run as one launch: random small 2-D shapes, tilings, cadences, phase geometry."""
    dims, tiles, iters, every, opts, fuse_res, dtype = case
    r = H.JacobiRun(dims, tiles, dtype, **opts)
    try:
        assert len(H.B.jacobi_pass_schedule(r.plan, iters)) < iters or iters == 1 or opts["resident_depth"] == 1
    finally:
        r.close()
    a = random_padded(dims, dtype=dtype, seed=6000 + n)
    if not fuse_res:
        return check(*run_case(H, oracle_mod, a, tiles, iters, every, **opts))
    r = H.JacobiRun(dims, tiles, dtype, **opts)
    try:
        r.load(a)
        res = r.run(iters, every, fuse_residual=True)
        out = r.fetch()
    finally:
        r.close()
    ref, ref_res = oracle_mod.run(a, iters, every)
    check(out, res, ref, ref_res)


def make_stack_cases(count, seed):
    """2-D shapes for the stand-alone residual pass with stacked wavefronts (tiles at least a band of 8 rows high)."""
    rng = np.random.default_rng(seed)
    cases = []
    for n in range(count):
        ty, tx = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        th, tw = int(rng.integers(8, 300)), int(rng.integers(1, 500))
        cases.append(((ty * th, tx * tw), (ty, tx), int(rng.integers(1, 6)), int(rng.choice([4, 8])),
                      np.float32 if n % 3 == 2 else np.float64))
    return cases


@pytest.mark.parametrize("n,case", list(enumerate(make_stack_cases(36, 20221007))))
def test_random_stacked_residual(H, oracle_mod, n, case):
    """residual_norm through the stacked kernel after a few updates, against the oracle and against the
    unstacked kernel (same terms in another order: tolerance, not bits)."""
    dims, tiles, iters, stack, dtype = case
    a = random_padded(dims, dtype=dtype, seed=7000 + n)
    ref, ref_res = oracle_mod.run(a, iters, iters)
    r = H.JacobiRun(dims, tiles, dtype, stack=stack)
    try:
        r.load(a)
        r.sweep(iters)
        res = r.residual()
        assert r.residual() == res                      # reproducible to the bit
        out = r.fetch()
        r.set_option("stack", 1)
        plain = r.residual()
    finally:
        r.close()
    check(out, [res], ref, ref_res)
    assert abs(plain - res) <= (1e-12 if dtype == np.float64 else 1e-5) * max(abs(res), 1e-300)
