"""MI355X-native Jacobi relaxation on a block-decomposed grid (the data-parallel
hot path of the Jacobi proxy application, paper Sec. VI-C): hand-written HIP
kernels behind the C ABI of include/jacobi.h, plus a thin ctypes binding.

The binding (and with it the shared library) is loaded on first use of any API
name, so that ``paper_2210_01238_amd.build`` can be imported to compile the
library before it exists.  There is no fallback: using the API without a built
library raises ImportError.
"""
import importlib

_API = (
    "JacobiError", "JacobiLayout", "jacobi_create", "jacobi_prepare", "jacobi_scratch_bytes", "jacobi_destroy", "jacobi_grid_bytes",
    "jacobi_get_layout", "jacobi_scatter", "jacobi_gather", "jacobi_sweep", "jacobi_sweep_residual", "jacobi_run", "jacobi_sweep_tasks",
    "jacobi_task_dependencies", "jacobi_pass_schedule", "halo_exchange",
    "residual_norm", "residual_norm_host", "residual_norm_noalloc", "jacobi_set_option", "jacobi_get_option",
    "jacobi_profile_read", "jacobi_last_error", "jacobi_stream_copy", "JACOBI_F64", "JACOBI_F32",
    "EXPORTS", "LIB_PATH",
)
__all__ = list(_API) + ["binding", "harness", "build"]


def __getattr__(name):
    if name in _API:
        return getattr(importlib.import_module(".binding", __name__), name)
    if name in ("binding", "harness", "build"):
        return importlib.import_module("." + name, __name__)
    raise AttributeError(name)
