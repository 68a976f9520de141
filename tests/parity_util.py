"""Helpers shared by the GPU parity tests (no arithmetic of the method here)."""
import numpy as np

import jacobi_inputs as gen


def interior(a):
    return a[tuple(slice(1, -1) for _ in a.shape)]


def random_padded(shape, dtype=np.float64, seed=1, lo=-1.0, hi=1.0):
    rng = np.random.default_rng(seed)
    return np.ascontiguousarray(rng.uniform(lo, hi, size=tuple(n + 2 for n in shape)).astype(dtype))


def oracle_window(oracle, w, lo, hi, iters, dtype=np.float64):
    """Run the oracle on the padded index box [lo, hi) of workload w and return
    (field after `iters` iterations, slices of the part that is exact).

    The outermost cells of the box are held constant by the oracle.  Where a box
    face coincides with the domain's Dirichlet ring that is correct; elsewhere the
    error it introduces travels one cell per iteration, so cells at least `iters`
    cells away from every artificial face carry exactly the value of a whole-domain
    run."""
    pd = [d + 2 for d in w.dims]
    a = gen.generate_window(w, lo, hi, dtype)
    u, _ = oracle.run(a, iters)
    valid = []
    for d in range(w.ndim):
        n = hi[d] - lo[d]
        s = 1 if lo[d] == 0 else iters
        e = n - 1 if hi[d] == pd[d] else n - iters
        assert e > s, "window too small for the iteration count"
        valid.append(slice(s, e))
    return u, tuple(valid)


def read_tile_cell(raw, lay, t, k, i, c):
    """Value of padded cell (k, i, c) of tile t in a raw grid buffer (numpy, element
    typed), following the documented layout; c = -1 / tw address the x halo arrays."""
    th, tw = lay.tile[1], lay.tile[2]
    base = t * lay.tile_stride
    if c < 0:
        return raw[base + lay.xhalo_offset + k * (th + 2) + i]
    if c == tw:
        return raw[base + lay.xhalo_offset + lay.xhalo_pitch + k * (th + 2) + i]
    return raw[base + (k * (th + 2) + i) * lay.pitch + c]
