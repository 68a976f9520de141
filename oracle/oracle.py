"""ctypes front end of the C oracle (``jacobi_oracle.c``).

Test infrastructure: a plain CPU reference of the Jacobi iteration of paper
Sec. VI-C (halo exchange, then update, a fixed number of times) plus the
residual norm.  All arithmetic lives in the C file; this module only builds it
with gcc, marshals numpy arrays and returns results.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# JACOBI_ORACLE_SRC: build and load another source file instead (the mutation test plants mistakes in a COPY
# of jacobi_oracle.c and checks that the pins notice each of them); the library is built next to that file.
_SRC = os.environ.get("JACOBI_ORACLE_SRC") or os.path.join(_HERE, "jacobi_oracle.c")
_LIB = (os.path.splitext(_SRC)[0] + ".so") if os.environ.get("JACOBI_ORACLE_SRC") else os.path.join(_HERE, "libjacobi_oracle.so")
_lib: Optional[ctypes.CDLL] = None

_SUF = {np.dtype(np.float64): "f64", np.dtype(np.float32): "f32"}
_CT = {np.dtype(np.float64): ctypes.c_double, np.dtype(np.float32): ctypes.c_float}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (contraction off, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        i64, p = ctypes.c_int64, ctypes.c_void_p
        for s in ("f64", "f32"):
            getattr(_lib, f"oracle_sweep2d_{s}").argtypes = [p, p, i64, i64]
            getattr(_lib, f"oracle_sweep2d_{s}").restype = None
            getattr(_lib, f"oracle_sweep3d_{s}").argtypes = [p, p, i64, i64, i64]
            getattr(_lib, f"oracle_sweep3d_{s}").restype = None
            getattr(_lib, f"oracle_residual2d_{s}").argtypes = [p, i64, i64]
            getattr(_lib, f"oracle_residual2d_{s}").restype = ctypes.c_double
            getattr(_lib, f"oracle_residual3d_{s}").argtypes = [p, i64, i64, i64]
            getattr(_lib, f"oracle_residual3d_{s}").restype = ctypes.c_double
            getattr(_lib, f"oracle_run_{s}").argtypes = [p, p, ctypes.c_int, p, i64, i64, p]
            getattr(_lib, f"oracle_run_{s}").restype = ctypes.c_int
            getattr(_lib, f"oracle_run_tiled_{s}").argtypes = [p, ctypes.c_int, p, p, i64]
            getattr(_lib, f"oracle_run_tiled_{s}").restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    """Threads the OpenMP sweep loops will use (OMP_NUM_THREADS or the CPU count)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        try:
            return max(1, int(v.split(",")[0]))
        except ValueError:
            pass
    return os.cpu_count() or 1


def set_threads(n: int) -> None:
    """Number of threads the OpenMP sweep loops use from now on (results do not depend on it)."""
    load()
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def _check(a: np.ndarray) -> Tuple[str, Tuple[int, ...]]:
    if a.dtype not in _SUF or not a.flags.c_contiguous or a.ndim not in (2, 3):
        raise ValueError("need a C-contiguous 2-D/3-D float32/float64 padded array")
    if min(a.shape) < 3:
        raise ValueError("padded array needs at least one interior point per dim")
    return _SUF[a.dtype], tuple(n - 2 for n in a.shape)


def sweep(a: np.ndarray) -> np.ndarray:
    """One Jacobi update of the padded array ``a``; ring copied unchanged."""
    suf, dims = _check(a)
    b = a.copy()
    fn = getattr(load(), f"oracle_sweep{a.ndim}d_{suf}")
    fn(a.ctypes.data, b.ctypes.data, *dims)
    return b


def residual(a: np.ndarray) -> float:
    """sqrt(sum over interior of (sum of face neighbours - 2d*u)^2)."""
    suf, dims = _check(a)
    fn = getattr(load(), f"oracle_residual{a.ndim}d_{suf}")
    return float(fn(a.ctypes.data, *dims))


def run(a: np.ndarray, iters: int, residual_every: int = 0) -> Tuple[np.ndarray, List[float]]:
    """``iters`` Jacobi iterations from padded field ``a`` on one untiled
    array.  Returns (final padded field, residuals after every
    ``residual_every``-th iteration)."""
    suf, dims = _check(a)
    A = a.copy()
    B = np.empty_like(A)
    nres = iters // residual_every if residual_every > 0 else 0
    res = np.zeros(max(nres, 1), dtype=np.float64)
    d = (ctypes.c_int64 * a.ndim)(*dims)
    which = getattr(load(), f"oracle_run_{suf}")(A.ctypes.data, B.ctypes.data, a.ndim, d,
                                                 iters, residual_every, res.ctypes.data)
    if which < 0:
        raise ValueError("oracle_run rejected its arguments")
    return (A if which == 0 else B), [float(x) for x in res[:nres]]


def run_tiled(a: np.ndarray, tiles: Sequence[int], iters: int) -> np.ndarray:
    """Same iteration on separately stored blocks with explicit halo copies."""
    suf, dims = _check(a)
    G = a.copy()
    d = (ctypes.c_int64 * a.ndim)(*dims)
    t = (ctypes.c_int64 * a.ndim)(*[int(x) for x in tiles])
    rc = getattr(load(), f"oracle_run_tiled_{suf}")(G.ctypes.data, a.ndim, d, t, iters)
    if rc != 0:
        raise ValueError("oracle_run_tiled rejected its arguments (dims % tiles != 0?)")
    return G
