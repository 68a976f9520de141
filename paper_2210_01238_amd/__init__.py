"""MI355X-native Jacobi relaxation on a block-decomposed grid (the data-parallel
hot path of the Jacobi proxy application, paper Sec. VI-C): hand-written HIP
kernels behind the C ABI of include/jacobi.h, plus this thin ctypes binding."""
from .binding import *  # noqa: F401,F403
from .binding import (JacobiError, JacobiLayout, jacobi_create, jacobi_destroy,  # noqa: F401
                      jacobi_grid_bytes, jacobi_get_layout, jacobi_scatter, jacobi_gather,
                      jacobi_sweep, halo_exchange, residual_norm, residual_norm_host,
                      jacobi_set_option, jacobi_get_option, jacobi_profile_read,
                      jacobi_last_error, JACOBI_F64, JACOBI_F32, EXPORTS, LIB_PATH)
