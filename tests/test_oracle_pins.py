"""Pins for the CPU oracle: every check here compares the oracle with something
that is NOT the oracle - a closed form, an invariant of the Jacobi iteration
for the Laplace equation, a dense-matrix brute force written independently in
numpy, or a direct linear solve.  (Paper Sec. VI-C fixes only the iteration
structure; it prints no values, so mathematics is the pin.)
"""
import numpy as np
import pytest

import jacobi_inputs as gen

RNG = np.random.default_rng(20221001)


# ---------------------------------------------------------------- helpers ---
def dense_iteration_2d(Ny, Nx, ring):
    """Independent brute force: dense matrix M and vector c with
    u_new = M u + c for the 5-point Jacobi mean, built cell by cell."""
    n = Ny * Nx
    M = np.zeros((n, n))
    c = np.zeros(n)
    idx = lambda i, j: (i - 1) * Nx + (j - 1)
    for i in range(1, Ny + 1):
        for j in range(1, Nx + 1):
            for (a, b) in ((i, j - 1), (i, j + 1), (i - 1, j), (i + 1, j)):
                if 1 <= a <= Ny and 1 <= b <= Nx:
                    M[idx(i, j), idx(a, b)] += 0.25
                else:
                    c[idx(i, j)] += 0.25 * ring[a, b]
    return M, c


def dense_iteration_3d(Nz, Ny, Nx, ring):
    n = Nz * Ny * Nx
    M = np.zeros((n, n))
    c = np.zeros(n)
    idx = lambda k, i, j: ((k - 1) * Ny + (i - 1)) * Nx + (j - 1)
    for k in range(1, Nz + 1):
        for i in range(1, Ny + 1):
            for j in range(1, Nx + 1):
                for (a, b, d) in ((k, i, j - 1), (k, i, j + 1), (k, i - 1, j), (k, i + 1, j),
                                  (k - 1, i, j), (k + 1, i, j)):
                    if 1 <= a <= Nz and 1 <= b <= Ny and 1 <= d <= Nx:
                        M[idx(k, i, j), idx(a, b, d)] += 1.0 / 6.0
                    else:
                        c[idx(k, i, j)] += ring[a, b, d] / 6.0
    return M, c


def random_padded(shape, dtype=np.float64, lo=0.0, hi=1.0):
    return np.ascontiguousarray(RNG.uniform(lo, hi, size=shape).astype(dtype))


def interior(a):
    return a[tuple(slice(1, -1) for _ in a.shape)]


# ------------------------------------------- I1: harmonic fixed points ------
@pytest.mark.parametrize("kind", ["i+j", "i2-j2"])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_lattice_harmonic_fixed_point_2d_bit_exact(oracle_mod, kind, dtype):
    a = gen.lattice_field((37, 53), kind, dtype)
    b, res = oracle_mod.run(a, 7, 1)
    assert np.array_equal(a, b)          # all partial sums are small integers, *0.25 exact
    assert res == [0.0] * 7


@pytest.mark.parametrize("kind", ["i+j+k", "i2+j2-2k2"])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_lattice_harmonic_fixed_point_3d(oracle_mod, kind, dtype):
    a = gen.lattice_field((11, 14, 19), kind, dtype)
    b = oracle_mod.sweep(a)
    assert b.dtype == a.dtype
    # exact up to the single multiplication by fl(1/6) (all sums are small integers, exact in fp32 too)
    assert np.max(np.abs(b - a)) <= 2 * np.spacing(np.max(np.abs(a)))
    assert oracle_mod.residual(a) == 0.0  # integer arithmetic, exactly zero
    # the multiplier is fl(1/6) in the WORKING precision: on a cell whose neighbour sum is 6*m the
    # result is fl(fl(1/6) * 6m), which a correctly rounded product in that precision reproduces
    s6 = interior(a) * dtype(6)
    assert np.array_equal(interior(b), (dtype(1) / dtype(6)) * s6)


def test_unit_square_harmonic_is_fixed_point_and_attractor(oracle_mod):
    # u = x^2 - y^2 and u = x + y sampled on a uniform grid have zero 5-point Laplacian
    n = 24
    w = gen.Workload("t", (n, n), (1, 1), 0, 0, "x2-y2", "random11", 9)
    x = np.arange(n + 2) / (n + 1.0)
    exact = x[None, :] ** 2 - x[:, None] ** 2
    b = oracle_mod.sweep(np.ascontiguousarray(exact))
    assert np.max(np.abs(b - exact)) < 1e-15
    # from a random interior the iteration converges to that harmonic function
    a = gen.generate(w)
    assert np.array_equal(a[0], exact[0]) and np.array_equal(a[:, -1], exact[:, -1])
    u, _ = oracle_mod.run(a, 4000)
    assert np.max(np.abs(u - exact)) < 1e-12


# ------------------------------------------- I2: discrete maximum principle -
@pytest.mark.parametrize("shape", [(20, 33), (9, 10, 12)])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_maximum_principle(oracle_mod, shape, dtype):
    a = random_padded(shape, dtype, lo=-3.0, hi=5.0)
    lo, hi = a.min(), a.max()
    tol = 0.0 if len(shape) == 2 else 2 * np.spacing(max(abs(lo), abs(hi)))
    u = a
    for _ in range(25):
        u = oracle_mod.sweep(u)
        assert interior(u).min() >= lo - tol and interior(u).max() <= hi + tol


# ------------------------------------------- I3: tiled == untiled -----------
@pytest.mark.parametrize("shape,tiles", [
    ((12, 18), (1, 1)), ((12, 18), (3, 2)), ((12, 18), (12, 18)), ((12, 18), (4, 18)),
    ((16, 16), (4, 4)), ((6, 8, 10), (2, 2, 2)), ((6, 8, 10), (6, 1, 5)), ((6, 8, 10), (1, 8, 1)),
])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_tiled_equals_untiled_bit_exact(oracle_mod, shape, tiles, dtype):
    a = random_padded(tuple(n + 2 for n in shape), dtype)
    ref, _ = oracle_mod.run(a, 9)
    til = oracle_mod.run_tiled(a, tiles, 9)
    assert np.array_equal(ref, til)


def test_tiled_rejects_non_divisible(oracle_mod):
    a = random_padded((12, 12))
    with pytest.raises(ValueError):
        oracle_mod.run_tiled(a, (3, 2), 1)


# ------------------------------------------- I4: eigenmodes -----------------
# fp32: the closed forms hold to a few fp32 roundings (2^-24 = 6e-8 each) of values of size <= 1
EIGEN_TOL = {np.float64: (1e-14, 1e-12), np.float32: (5e-7, 2e-6)}


@pytest.mark.parametrize("Ny,Nx,p,q", [(15, 22, 1, 1), (15, 22, 3, 5), (8, 8, 8, 1)])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_eigenmode_2d(oracle_mod, Ny, Nx, p, q, dtype):
    i = np.arange(Ny + 2)[:, None]
    j = np.arange(Nx + 2)[None, :]
    u = np.sin(p * np.pi * i / (Ny + 1)) * np.sin(q * np.pi * j / (Nx + 1))
    u[0] = u[-1] = 0.0
    u[:, 0] = u[:, -1] = 0.0
    u = np.ascontiguousarray(u.astype(dtype))
    lam = 0.5 * (np.cos(p * np.pi / (Ny + 1)) + np.cos(q * np.pi / (Nx + 1)))
    v = oracle_mod.sweep(u)
    tol_u, tol_r = EIGEN_TOL[dtype]
    assert v.dtype == u.dtype
    assert np.max(np.abs(interior(v) - lam * interior(u).astype(np.float64))) < tol_u
    norm = np.sqrt((Ny + 1) * (Nx + 1) / 4.0)
    assert abs(oracle_mod.residual(u) - 4.0 * (1.0 - lam) * norm) < tol_r * norm


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_eigenmode_3d(oracle_mod, dtype):
    Nz, Ny, Nx, p, q, r = 7, 9, 12, 2, 1, 3
    k = np.arange(Nz + 2)[:, None, None]
    i = np.arange(Ny + 2)[None, :, None]
    j = np.arange(Nx + 2)[None, None, :]
    u = (np.sin(p * np.pi * k / (Nz + 1)) * np.sin(q * np.pi * i / (Ny + 1))
         * np.sin(r * np.pi * j / (Nx + 1)))
    for ax in range(3):
        sl = [slice(None)] * 3
        sl[ax] = 0
        u[tuple(sl)] = 0.0
        sl[ax] = -1
        u[tuple(sl)] = 0.0
    u = np.ascontiguousarray(u.astype(dtype))
    lam = (np.cos(p * np.pi / (Nz + 1)) + np.cos(q * np.pi / (Ny + 1))
           + np.cos(r * np.pi / (Nx + 1))) / 3.0
    v = oracle_mod.sweep(u)
    tol_u, tol_r = EIGEN_TOL[dtype]
    assert v.dtype == u.dtype
    assert np.max(np.abs(interior(v) - lam * interior(u).astype(np.float64))) < tol_u
    norm = np.sqrt((Nz + 1) * (Ny + 1) * (Nx + 1) / 8.0)
    assert abs(oracle_mod.residual(u) - 6.0 * (1.0 - lam) * norm) < tol_r * norm


# ------------------------------------------- I5: brute force ----------------
# fp32 runs are compared with the fp64 dense iteration of the same (fp32-representable) data:
# every value stays within [-1, 1] and a step adds at most ~3 roundings of 6e-8, which the
# iteration (a contraction) does not amplify
DENSE_TOL = {np.float64: (1e-14, 1e-12), np.float32: (2e-6, 5e-6)}


@pytest.mark.parametrize("Ny,Nx", [(8, 8), (5, 9)])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_dense_matrix_brute_force_2d(oracle_mod, Ny, Nx, dtype):
    a = random_padded((Ny + 2, Nx + 2), dtype, lo=-1.0, hi=1.0)
    M, c = dense_iteration_2d(Ny, Nx, a.astype(np.float64))
    v = interior(a).reshape(-1).astype(np.float64)
    tol_k, tol_inf = DENSE_TOL[dtype]
    for k in range(1, 21):
        v = M @ v + c
        u, _ = oracle_mod.run(a, k)
        assert u.dtype == a.dtype
        assert np.max(np.abs(interior(u).reshape(-1) - v)) < tol_k
    # long run converges to the direct solve of (I - M) u = c
    u, _ = oracle_mod.run(a, 900)
    direct = np.linalg.solve(np.eye(Ny * Nx) - M, c)
    assert np.max(np.abs(interior(u).reshape(-1) - direct)) < tol_inf
    # residual against the dense form: sum_nbrs u - 4u = 4 (M u + c - u)
    u0 = interior(a).reshape(-1).astype(np.float64)
    dense_res = 4.0 * np.linalg.norm(M @ u0 + c - u0)
    assert abs(oracle_mod.residual(a) - dense_res) < (1e-12 if dtype is np.float64 else 2e-6) * dense_res


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_dense_matrix_brute_force_3d(oracle_mod, dtype):
    Nz, Ny, Nx = 3, 4, 5
    a = random_padded((Nz + 2, Ny + 2, Nx + 2), dtype, lo=-1.0, hi=1.0)
    M, c = dense_iteration_3d(Nz, Ny, Nx, a.astype(np.float64))
    v = interior(a).reshape(-1).astype(np.float64)
    tol_k, tol_inf = DENSE_TOL[dtype]
    for k in range(1, 13):
        v = M @ v + c
        u, _ = oracle_mod.run(a, k)
        assert u.dtype == a.dtype
        assert np.max(np.abs(interior(u).reshape(-1) - v)) < tol_k
    u, _ = oracle_mod.run(a, 400)
    direct = np.linalg.solve(np.eye(Nz * Ny * Nx) - M, c)
    assert np.max(np.abs(interior(u).reshape(-1) - direct)) < tol_inf
    # residual against the dense form: sum_nbrs u - 6u = 6 (M u + c - u)
    u0 = interior(a).reshape(-1).astype(np.float64)
    dense_res = 6.0 * np.linalg.norm(M @ u0 + c - u0)
    assert abs(oracle_mod.residual(a) - dense_res) < (1e-12 if dtype is np.float64 else 2e-6) * dense_res


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_residual_against_numpy_slices(oracle_mod, dtype):
    # neighbour sums and the subtraction in fp64 on the same data: the fp32 oracle forms its terms in
    # fp32 (a few roundings of 6e-8 on terms of size ~1), the sum of squares is fp64 / long double
    tol = 1e-13 if dtype is np.float64 else 1e-6
    a = random_padded((13, 17), dtype)
    w = a.astype(np.float64)
    r = w[1:-1, :-2] + w[1:-1, 2:] + w[:-2, 1:-1] + w[2:, 1:-1] - 4.0 * w[1:-1, 1:-1]
    ref = np.sqrt(np.sum(r * r))
    assert ref > 1.0 and abs(oracle_mod.residual(a) - ref) < tol * ref
    a = random_padded((7, 9, 11), dtype)
    w = a.astype(np.float64)
    c = w[1:-1, 1:-1, 1:-1]
    r = (w[1:-1, 1:-1, :-2] + w[1:-1, 1:-1, 2:] + w[1:-1, :-2, 1:-1] + w[1:-1, 2:, 1:-1]
         + w[:-2, 1:-1, 1:-1] + w[2:, 1:-1, 1:-1] - 6.0 * c)
    ref = np.sqrt(np.sum(r * r))
    assert ref > 1.0 and abs(oracle_mod.residual(a) - ref) < tol * ref


# ------------------------------------------- I6: C1 data ---------------------
def test_c1_light_cone_symmetry_and_first_row(oracle_mod):
    w = gen.WORKLOADS["C1"]
    a = gen.generate(w)
    assert a[0, 1:-1].min() == 1.0 and a[0, 0] == 0.0 and a[1:, :].max() == 0.0
    u1 = oracle_mod.sweep(a)
    assert np.all(u1[1, 1:-1] == 0.25) and np.all(u1[2:-1, 1:-1] == 0.0)
    for k in (5, 40, 100):
        u, _ = oracle_mod.run(a, k)
        assert np.all(u[k + 1:-1, 1:-1] == 0.0)          # nothing travels faster than 1 row/iter
        assert np.all(u[k, 1:-1] > 0.0) if k < 257 else True
        assert u[k, 128] == 0.25 ** k                    # the wave front is exactly 4^-k
        assert np.array_equal(u, u[:, ::-1])             # mirror symmetry needs (W+E) pairing


# ------------------------------------------- I7: residual --------------------
@pytest.mark.parametrize("shape", [(16, 16), (6, 7, 8)])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_residual_identity_and_monotone(oracle_mod, shape, dtype):
    if dtype is np.float32:
        # R(u) = 2d * ||sweep(u) - u||, to fp32 rounding of the terms, while R is far above that floor
        a = random_padded(tuple(n + 2 for n in shape), dtype)
        u = a
        for _ in range(6):
            nxt = oracle_mod.sweep(u)
            R = oracle_mod.residual(u)
            diff = 2 * len(shape) * np.linalg.norm((interior(nxt).astype(np.float64) - interior(u)).reshape(-1))
            assert R > 0.1 and abs(R - diff) <= 1e-5 * R
            u = nxt
        return
    d = len(shape)
    a = random_padded(tuple(n + 2 for n in shape))
    u = a
    prev = None
    for _ in range(30):
        nxt = oracle_mod.sweep(u)
        R = oracle_mod.residual(u)
        diff = 2 * d * np.linalg.norm((interior(nxt) - interior(u)).reshape(-1))
        assert abs(R - diff) <= 1e-13 * R
        if prev is not None:
            assert R < prev
        prev, u = R, nxt
    # contraction factor on a square: R_{k+1} <= cos(pi/(N+1)) R_k
    if d == 2:
        rho = np.cos(np.pi / (shape[0] + 1))
        _, res = oracle_mod.run(a, 60, 1)
        assert all(res[k + 1] <= rho * res[k] * (1 + 1e-12) for k in range(len(res) - 1))


def test_run_residual_is_of_the_grid_the_iteration_produced(oracle_mod):
    a = random_padded((14, 14))
    _, res = oracle_mod.run(a, 12, 4)
    for n, k in enumerate((4, 8, 12)):
        u, _ = oracle_mod.run(a, k)
        assert res[n] == oracle_mod.residual(u)


# ------------------------------------------- I8: linearity -------------------
@pytest.mark.parametrize("shape", [(10, 13), (5, 6, 7)])
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_scaling_by_two_is_exact(oracle_mod, shape, dtype):
    a = random_padded(tuple(n + 2 for n in shape), dtype, lo=-1, hi=1)
    u, _ = oracle_mod.run(a, 5)
    v, _ = oracle_mod.run(np.ascontiguousarray(dtype(2.0) * a), 5)
    assert v.dtype == a.dtype and np.array_equal(dtype(2.0) * u, v)


# ------------------------------------------- I9: steady state ----------------
def test_top_edge_problem_centre_is_one_quarter(oracle_mod):
    n = 15
    w = gen.Workload("t", (n, n), (1, 1), 0, 0, "top1", "zero", 0)
    u, _ = oracle_mod.run(gen.generate(w), 3000)
    assert abs(u[(n + 1) // 2, (n + 1) // 2] - 0.25) < 1e-13


# ------------------------------------------- fp32 follows fp64 ---------------
@pytest.mark.parametrize("shape", [(34, 34), (10, 12, 14)])
def test_fp32_tracks_fp64(oracle_mod, shape):
    a = random_padded(shape)
    u64, r64 = oracle_mod.run(a, 50, 10)
    u32, r32 = oracle_mod.run(a.astype(np.float32), 50, 10)
    assert u32.dtype == np.float32
    assert np.max(np.abs(u32 - u64)) < 1e-5
    # residuals well above the fp32 rounding floor (~1e-6 * sqrt(points)) agree to that floor
    floor = 1e-6 * np.sqrt(np.prod(shape))
    assert len(r32) == 5 and all(abs(x - y) < floor + 1e-5 * y for x, y in zip(r32, r64))


# ------------------------------------------- stored values --------------------
def read_golden_c1():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "c1_100iters.txt")
    res, pts = None, {}
    for line in open(path):
        if line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "residual":
            res = float.fromhex(f[1])
        elif f[0] == "u":
            pts[(int(f[1]), int(f[2]))] = float.fromhex(f[3])
    return res, pts


def test_oracle_reproduces_stored_c1_values(oracle_mod):
    w = gen.WORKLOADS["C1"]
    u, res = oracle_mod.run(gen.generate(w), w.iters, w.residual_every)
    gres, pts = read_golden_c1()
    assert res == [gres]
    for (i, j), v in pts.items():
        assert u[i, j] == v
    assert pts[(101, 5)] == 0.0 and pts[(100, 128)] == 0.25 ** 100
