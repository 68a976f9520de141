"""CPU oracle for the block-decomposed Jacobi proxy computation (paper Sec. VI-C).

Test infrastructure only: imported by the tests, the smoke check and the
benchmark's CPU-baseline leg.  The GPU library never touches it.
"""
from .oracle import (build, run, run_tiled, sweep, residual, load,  # noqa: F401
                     num_threads, set_threads)
