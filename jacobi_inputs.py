"""Seeded synthetic inputs for the block-decomposed Jacobi proxy workload.

This module only *produces data*: padded global arrays (interior plus a
one-cell Dirichlet ring) for the workload shapes of the Jacobi proxy
application (paper Sec. VI-C: a regular Cartesian domain cut into cuboid
blocks, one-cell face halos, a fixed number of iterations).  It holds none of
the method's arithmetic (no stencil, no halo logic, no norm) and is the one
piece shared by the CPU oracle's tests and the GPU path's tests/bench.

Random fields are *counter based*: the value at padded global linear index g
depends only on (seed, g), so any rectangular window of a huge field can be
generated without materialising the rest.  The mixing function is the
published SplitMix64 finaliser (Steele, Lea, Flood 2014) applied to
seed * 2**32 + g; the top 53 bits scaled by 2**-53 give a double in [0, 1).

Index convention: row-major, last index (x) fastest.  A padded 2-D array has
shape (Ny + 2, Nx + 2); padded index 0 and N + 1 are the Dirichlet ring.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(x: np.ndarray) -> np.ndarray:
    """SplitMix64 output function on an array of uint64 counters (wraps mod 2**64)."""
    x = np.asarray(x, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = x + _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, g: np.ndarray) -> np.ndarray:
    """Double in [0, 1) for every padded global linear index in ``g``."""
    g = np.asarray(g, dtype=np.uint64)
    with np.errstate(over="ignore"):
        ctr = np.uint64((int(seed) << 32) & 0xFFFFFFFFFFFFFFFF) + g
    bits = splitmix64(ctr) >> np.uint64(11)
    return bits.astype(np.float64) * (1.0 / 9007199254740992.0)


@dataclass(frozen=True)
class Workload:
    """One workload shape: interior dims (slowest to fastest), tile counts per
    dim, iteration count, residual cadence and the recipe for the data."""

    name: str
    dims: Tuple[int, ...]
    tiles: Tuple[int, ...]
    iters: int
    residual_every: int
    boundary: str  # "top1", "random01", "x2-y2", "x+y"
    interior: str  # "zero", "random01", "random11"
    seed: int = 0

    @property
    def ndim(self) -> int:
        return len(self.dims)

    @property
    def points(self) -> int:
        n = 1
        for d in self.dims:
            n *= d
        return n

    def scaled(self, dims: Sequence[int], tiles: Optional[Sequence[int]] = None,
               iters: Optional[int] = None, residual_every: Optional[int] = None) -> "Workload":
        """Same recipe on a smaller (or differently tiled) domain."""
        return Workload(self.name + "-scaled", tuple(dims),
                        tuple(tiles) if tiles is not None else self.tiles,
                        self.iters if iters is None else iters,
                        self.residual_every if residual_every is None else residual_every,
                        self.boundary, self.interior, self.seed)


# The workload shapes.  C3 is the one the throughput figure is quoted on.
WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1", (256, 256), (1, 1), 100, 100, "top1", "zero", 0),
    "C2": Workload("C2", (4096, 4096), (4, 4), 1000, 100, "random01", "random01", 2),
    "C3": Workload("C3", (16384, 16384), (8, 8), 200, 10, "x2-y2", "random11", 3),
    "C4": Workload("C4", (512, 512, 512), (4, 4, 4), 100, 10, "random01", "zero", 4),
    "C5": Workload("C5", (8192, 8192), (64, 64), 500, 50, "x+y", "random01", 5),
    # the one domain size the paper states for its 3-D proxy runs (Sec. VI-C: 1024 x 1024 x 768),
    # cut into 128^3 blocks; data recipe as C4
    "P1": Workload("P1", (768, 1024, 1024), (6, 8, 8), 100, 10, "random01", "zero", 6),
}


def _window_axes(w: Workload, lo: Sequence[int], hi: Sequence[int]):
    pdims = [d + 2 for d in w.dims]
    for a, b, p in zip(lo, hi, pdims):
        if not (0 <= a < b <= p):
            raise ValueError(f"window [{a},{b}) outside padded extent {p}")
    return pdims, [np.arange(a, b, dtype=np.int64) for a, b in zip(lo, hi)]


def generate_window(w: Workload, lo: Sequence[int], hi: Sequence[int],
                    dtype=np.float64) -> np.ndarray:
    """Values of the padded global field of ``w`` on the index box
    ``lo[d] <= idx[d] < hi[d]`` (padded indices, slowest to fastest).

    Cells of the window that lie on the global Dirichlet ring get the boundary
    recipe; all others the interior recipe.  fp32 output is the rounding of the
    fp64 value.
    """
    nd = w.ndim
    pdims, axes = _window_axes(w, lo, hi)
    grids = np.meshgrid(*axes, indexing="ij", sparse=True)
    shape = tuple(len(a) for a in axes)

    # padded global linear index of every window cell
    lin = np.zeros(shape, dtype=np.uint64)
    for d in range(nd):
        lin = lin * np.uint64(pdims[d]) + grids[d].astype(np.uint64)

    on_ring = np.zeros(shape, dtype=bool)
    for d in range(nd):
        on_ring = on_ring | (grids[d] == 0) | (grids[d] == pdims[d] - 1)

    need_rand = ("random" in w.interior) or ("random" in w.boundary)
    u = uniform01(w.seed, lin) if need_rand else None

    if w.interior == "zero":
        interior = np.zeros(shape, dtype=np.float64)
    elif w.interior == "random01":
        interior = u
    elif w.interior == "random11":
        interior = 2.0 * u - 1.0
    else:
        raise ValueError(w.interior)

    if w.boundary == "top1":
        # first padded row (slowest index 0) is 1.0 except its corner cells; rest of ring 0.0
        top = grids[0] == 0
        not_corner = np.ones(shape, dtype=bool)
        for d in range(1, nd):
            not_corner = not_corner & (grids[d] != 0) & (grids[d] != pdims[d] - 1)
        ring = np.where(top & not_corner, 1.0, 0.0)
    elif w.boundary == "random01":
        ring = u
    elif w.boundary in ("x2-y2", "x+y"):
        if nd != 2:
            raise ValueError("analytic boundaries are 2-D recipes")
        # unit-square coordinates on padded indices 0..N+1
        y = grids[0].astype(np.float64) / float(pdims[0] - 1)
        x = grids[1].astype(np.float64) / float(pdims[1] - 1)
        ring = (x * x - y * y) if w.boundary == "x2-y2" else (x + y)
        ring = np.broadcast_to(ring, shape)
    else:
        raise ValueError(w.boundary)

    out = np.where(on_ring, ring, interior)
    return np.ascontiguousarray(out.astype(dtype))


def generate(w: Workload, dtype=np.float64, chunk_rows: int = 512) -> np.ndarray:
    """The whole padded global field of ``w`` (built in slabs of the slowest
    index to bound temporary memory)."""
    pdims = [d + 2 for d in w.dims]
    out = np.empty(pdims, dtype=dtype)
    if w.ndim == 3:
        chunk_rows = max(1, chunk_rows // 64)
    for a in range(0, pdims[0], chunk_rows):
        b = min(pdims[0], a + chunk_rows)
        lo = [a] + [0] * (w.ndim - 1)
        hi = [b] + pdims[1:]
        out[a:b] = generate_window(w, lo, hi, dtype)
    return out


def lattice_field(shape: Sequence[int], kind: str, dtype=np.float64) -> np.ndarray:
    """Integer-lattice polynomial fields on padded indices (used as data whose
    discrete Laplacian vanishes identically): "i+j", "i2-j2", "i+j+k",
    "i2+j2-2k2".  Index names follow array order: 2-D (i, j), 3-D (k, i, j)."""
    axes = np.meshgrid(*[np.arange(n, dtype=np.float64) for n in shape], indexing="ij")
    if kind == "i+j":
        i, j = axes
        f = i + j
    elif kind == "i2-j2":
        i, j = axes
        f = i * i - j * j
    elif kind == "i+j+k":
        k, i, j = axes
        f = i + j + k
    elif kind == "i2+j2-2k2":
        k, i, j = axes
        f = i * i + j * j - 2.0 * k * k
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(f.astype(dtype))
