"""The seeded generator: published SplitMix64 values, window consistency, recipes."""
import numpy as np
import pytest

import jacobi_inputs as gen


def test_splitmix64_published_first_outputs():
    # SplitMix64 seeded with 0: the state advances by the golden gamma before mixing,
    # so the outputs for counters 0, gamma, 2*gamma are the sequence's first three values.
    g = 0x9E3779B97F4A7C15
    ctr = np.array([0, g, (2 * g) % 2**64], dtype=np.uint64)
    out = gen.splitmix64(ctr)
    assert [int(x) for x in out] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_uniform_range_and_moments():
    u = gen.uniform01(7, np.arange(200000, dtype=np.uint64))
    assert u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 5e-3 and abs(u.var() - 1 / 12) < 2e-3


@pytest.mark.parametrize("name,dims", [("C2", (40, 56)), ("C3", (40, 56)), ("C5", (24, 24)),
                                       ("C4", (6, 10, 12)), ("C1", (16, 16))])
def test_window_equals_slice_of_whole(name, dims):
    w = gen.WORKLOADS[name].scaled(dims, tuple(1 for _ in dims))
    full = gen.generate(w, chunk_rows=7)
    lo = [0, 3, 5][:len(dims)] if len(dims) == 3 else [3, 0]
    hi = [n + 2 - 1 for n in dims]
    win = gen.generate_window(w, lo, hi)
    sl = tuple(slice(a, b) for a, b in zip(lo, hi))
    assert np.array_equal(full[sl], win)


def test_recipes():
    w = gen.WORKLOADS["C3"].scaled((30, 30), (1, 1))
    a = gen.generate(w)
    x = np.arange(32) / 31.0
    assert np.array_equal(a[0], x * x - 0.0) and np.array_equal(a[:, 0], 0.0 - x * x)
    assert -1.0 <= a[1:-1, 1:-1].min() and a[1:-1, 1:-1].max() < 1.0 and a[1:-1, 1:-1].min() < -0.5
    w5 = gen.WORKLOADS["C5"].scaled((30, 30), (1, 1))
    b = gen.generate(w5)
    assert np.array_equal(b[-1], x + 1.0) and 0.0 <= b[1:-1, 1:-1].min()
    w4 = gen.WORKLOADS["C4"].scaled((6, 6, 6), (1, 1, 1))
    c = gen.generate(w4)
    assert np.all(c[1:-1, 1:-1, 1:-1] == 0.0) and c[0].max() > 0.5
    f32 = gen.generate(w, dtype=np.float32)
    assert f32.dtype == np.float32 and np.array_equal(f32, a.astype(np.float32))


def test_workload_table_matches_shapes():
    W = gen.WORKLOADS
    assert W["C3"].dims == (16384, 16384) and W["C3"].tiles == (8, 8) and W["C3"].iters == 200
    assert W["C4"].dims == (512,) * 3 and W["C4"].tiles == (4,) * 3
    assert W["C5"].tiles == (64, 64) and W["C5"].dims[0] // 64 == 128
    assert W["P1"].dims == (768, 1024, 1024) and W["P1"].points == 1024 * 1024 * 768
    for w in W.values():
        assert all(d % t == 0 for d, t in zip(w.dims, w.tiles))


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU; asking for more exits with a message before touching any device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="2")
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py")], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 2 and r.stdout.strip() == ""
