"""ctypes binding of libjacobi (declared in include/jacobi.h).

Argument marshalling only: every step of the computation runs inside the HIP
library.  Function names match the C ABI.  Device memory and streams are the
caller's (e.g. ``torch.empty(...).data_ptr()`` and
``torch.cuda.current_stream().cuda_stream``); pointers are plain integers here.
There is no CPU fallback: if the library is missing, import fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libjacobi.so")

JACOBI_F64, JACOBI_F32 = 0, 1
JACOBI_OK, JACOBI_EINVAL, JACOBI_ENOTDIV, JACOBI_ENOMEM, JACOBI_EHIP = 0, 1, 2, 3, 4

EXPORTS = (
    "jacobi_create", "jacobi_prepare", "jacobi_scratch_bytes", "jacobi_destroy", "jacobi_grid_bytes", "jacobi_get_layout",
    "jacobi_scatter", "jacobi_gather", "jacobi_sweep", "jacobi_sweep_residual", "jacobi_run", "jacobi_sweep_tasks", "jacobi_task_dependencies", "jacobi_pass_schedule", "halo_exchange", "residual_norm",
    "residual_norm_host", "residual_norm_noalloc", "jacobi_set_option", "jacobi_get_option", "jacobi_profile_read",
    "jacobi_last_error", "jacobi_stream_copy",
)


class JacobiLayout(ctypes.Structure):
    _fields_ = [
        ("ndim", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("dims", ctypes.c_int64 * 3), ("tiles", ctypes.c_int64 * 3), ("tile", ctypes.c_int64 * 3),
        ("ntiles", ctypes.c_int64), ("nplanes", ctypes.c_int64), ("pitch", ctypes.c_int64),
        ("plane", ctypes.c_int64), ("xhalo_offset", ctypes.c_int64), ("xhalo_pitch", ctypes.c_int64),
        ("tile_stride", ctypes.c_int64), ("grid_bytes", ctypes.c_int64), ("xsend_offset", ctypes.c_int64),
    ]


class JacobiError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libjacobi status {code}: {text}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is not built; run `python -m paper_2210_01238_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    P = ctypes.POINTER
    lib.jacobi_create.argtypes = [P(vp), ci, P(i64), P(i64), ci]
    lib.jacobi_destroy.argtypes = [vp]
    lib.jacobi_prepare.argtypes = [vp]
    lib.jacobi_scratch_bytes.argtypes = [vp]
    lib.jacobi_scratch_bytes.restype = ctypes.c_size_t
    lib.jacobi_grid_bytes.argtypes = [vp]
    lib.jacobi_grid_bytes.restype = ctypes.c_size_t
    lib.jacobi_get_layout.argtypes = [vp, P(JacobiLayout)]
    lib.jacobi_scatter.argtypes = [vp, vp, vp, vp]
    lib.jacobi_gather.argtypes = [vp, vp, vp, vp]
    lib.jacobi_sweep.argtypes = [vp, vp, vp, ci, vp, P(vp)]
    lib.jacobi_sweep_residual.argtypes = [vp, vp, vp, ci, vp, P(vp), vp]
    lib.jacobi_run.argtypes = [vp, vp, vp, ci, ci, vp, vp, P(vp)]
    lib.jacobi_sweep_tasks.argtypes = [vp, vp, vp, ci, ci, ci, vp, P(vp)]
    lib.jacobi_task_dependencies.argtypes = [vp, ci, ci, P(ci), ci, P(ci), P(ci)]
    lib.jacobi_pass_schedule.argtypes = [vp, ci, P(ci), ci, P(ci)]
    lib.halo_exchange.argtypes = [vp, vp, vp]
    lib.residual_norm.argtypes = [vp, vp, vp, vp]
    lib.residual_norm_noalloc.argtypes = [vp, vp, vp, vp]
    lib.residual_norm_host.argtypes = [vp, vp, P(ctypes.c_double), vp]
    lib.jacobi_set_option.argtypes = [vp, ctypes.c_char_p, i64]
    lib.jacobi_get_option.argtypes = [vp, ctypes.c_char_p, P(i64)]
    lib.jacobi_profile_read.argtypes = [vp, P(ctypes.c_double), P(i64)]
    lib.jacobi_stream_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.jacobi_last_error.argtypes = []
    lib.jacobi_last_error.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("jacobi_grid_bytes", "jacobi_scratch_bytes", "jacobi_last_error"):
            getattr(lib, name).restype = ci
    return lib


lib = _load()


def jacobi_last_error() -> str:
    return lib.jacobi_last_error().decode()


def _check(rc: int) -> None:
    if rc != JACOBI_OK:
        raise JacobiError(rc, jacobi_last_error())


def jacobi_create(dims: Sequence[int], tiles: Sequence[int], dtype: int = JACOBI_F64) -> int:
    """Returns the plan handle (an integer pointer)."""
    n = len(dims)
    h = ctypes.c_void_p()
    d = (ctypes.c_int64 * max(n, 1))(*[int(x) for x in dims])
    t = (ctypes.c_int64 * max(len(tiles), 1))(*[int(x) for x in tiles])
    if len(tiles) != n:
        raise JacobiError(JACOBI_EINVAL, "dims and tiles differ in length")
    _check(lib.jacobi_create(ctypes.byref(h), n, d, t, int(dtype)))
    return h.value


def jacobi_prepare(plan: int) -> None:
    _check(lib.jacobi_prepare(plan))


def jacobi_scratch_bytes(plan: Optional[int]) -> int:
    return int(lib.jacobi_scratch_bytes(plan))


def jacobi_destroy(plan: Optional[int]) -> None:
    _check(lib.jacobi_destroy(plan))


def jacobi_grid_bytes(plan: int) -> int:
    return int(lib.jacobi_grid_bytes(plan))


def jacobi_get_layout(plan: int) -> JacobiLayout:
    lay = JacobiLayout()
    _check(lib.jacobi_get_layout(plan, ctypes.byref(lay)))
    return lay


def jacobi_scatter(plan: int, global_padded_dev: int, grid: int, stream: int = 0) -> None:
    _check(lib.jacobi_scatter(plan, global_padded_dev, grid, stream))


def jacobi_gather(plan: int, grid: int, global_padded_dev: int, stream: int = 0) -> None:
    _check(lib.jacobi_gather(plan, grid, global_padded_dev, stream))


def jacobi_sweep(plan: int, grid_in: int, grid_out: int, iters: int, stream: int = 0) -> int:
    """Returns the pointer (grid_in or grid_out) that holds the result."""
    fin = ctypes.c_void_p()
    _check(lib.jacobi_sweep(plan, grid_in, grid_out, int(iters), stream, ctypes.byref(fin)))
    return fin.value


def jacobi_sweep_tasks(plan: int, grid_in: int, grid_out: int, iters: int, tiles_per_task: int, nstreams: int,
                       stream: int = 0) -> int:
    """jacobi_sweep executed as tasks of `tiles_per_task` tiles over `nstreams` streams.
    Returns the pointer that holds the result grid."""
    fin = ctypes.c_void_p()
    _check(lib.jacobi_sweep_tasks(plan, grid_in, grid_out, int(iters), int(tiles_per_task), int(nstreams),
                                  stream, ctypes.byref(fin)))
    return fin.value


def jacobi_pass_schedule(plan: int, iters: int) -> list:
    """Iterations advanced by each pass jacobi_sweep(plan, ., ., iters) would launch."""
    n = ctypes.c_int()
    _check(lib.jacobi_pass_schedule(plan, int(iters), None, 0, ctypes.byref(n)))
    buf = (ctypes.c_int * max(n.value, 1))()
    _check(lib.jacobi_pass_schedule(plan, int(iters), buf, n.value, ctypes.byref(n)))
    return list(buf[:n.value])


def jacobi_task_dependencies(plan: int, tiles_per_task: int) -> list:
    """For every task of an iteration (groups of tiles_per_task consecutive tiles): the tasks of the previous
    iteration it depends on, as jacobi_sweep_tasks orders them."""
    n, nt = ctypes.c_int(), ctypes.c_int()
    _check(lib.jacobi_task_dependencies(plan, int(tiles_per_task), 0, None, 0, ctypes.byref(n), ctypes.byref(nt)))
    out = []
    for t in range(nt.value):
        _check(lib.jacobi_task_dependencies(plan, int(tiles_per_task), t, None, 0, ctypes.byref(n), None))
        buf = (ctypes.c_int * max(n.value, 1))()
        _check(lib.jacobi_task_dependencies(plan, int(tiles_per_task), t, buf, n.value, ctypes.byref(n), None))
        out.append(sorted(buf[:n.value]))
    return out


def jacobi_sweep_residual(plan: int, grid_in: int, grid_out: int, iters: int, residual_in_dev: int,
                          stream: int = 0) -> int:
    """jacobi_sweep that also writes residual_norm(grid_in) to the device double
    residual_in_dev.  Returns the pointer that holds the result grid."""
    fin = ctypes.c_void_p()
    _check(lib.jacobi_sweep_residual(plan, grid_in, grid_out, int(iters), stream, ctypes.byref(fin),
                                     residual_in_dev))
    return fin.value


def jacobi_run(plan: int, grid_in: int, grid_out: int, iters: int, residual_every: int, residuals_dev: Optional[int],
               stream: int = 0) -> int:
    """iters iterations with the residual norm after every residual_every-th one written to the device
    array residuals_dev.  Returns the pointer that holds the result grid."""
    fin = ctypes.c_void_p()
    _check(lib.jacobi_run(plan, grid_in, grid_out, int(iters), int(residual_every), residuals_dev, stream,
                          ctypes.byref(fin)))
    return fin.value


def halo_exchange(plan: int, grid: int, stream: int = 0) -> None:
    _check(lib.halo_exchange(plan, grid, stream))


def residual_norm(plan: int, grid: int, result_dev: int, stream: int = 0) -> None:
    _check(lib.residual_norm(plan, grid, result_dev, stream))


NOALLOC_MAX_PARTIALS = 131072   # JACOBI_NOALLOC_MAX_PARTIALS of include/jacobi.h


def residual_norm_noalloc(plan: int, grid: int, result_dev: int, stream: int = 0) -> None:
    """residual_norm whose scratch is a fixed array inside the library: allocates nothing."""
    _check(lib.residual_norm_noalloc(plan, grid, result_dev, stream))


def residual_norm_host(plan: int, grid: int, stream: int = 0) -> float:
    out = ctypes.c_double()
    _check(lib.residual_norm_host(plan, grid, ctypes.byref(out), stream))
    return out.value


def jacobi_set_option(plan: int, key: str, value: int) -> None:
    _check(lib.jacobi_set_option(plan, key.encode(), int(value)))


def jacobi_get_option(plan: int, key: str) -> int:
    v = ctypes.c_int64()
    _check(lib.jacobi_get_option(plan, key.encode(), ctypes.byref(v)))
    return v.value


def jacobi_profile_read(plan: int) -> Tuple[float, int]:
    ms, n = ctypes.c_double(), ctypes.c_int64()
    _check(lib.jacobi_profile_read(plan, ctypes.byref(ms), ctypes.byref(n)))
    return ms.value, n.value


def jacobi_stream_copy(dst: int, src: int, nbytes: int, stream: int = 0) -> None:
    _check(lib.jacobi_stream_copy(dst, src, nbytes, stream))
