import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle_mod():
    import oracle
    oracle.build()
    return oracle


@pytest.fixture(scope="session")
def H():
    """The harness module, for GPU tests.  The parity suites were written against the launch-per-pass
    kernels and keep testing those on their (mostly small) shapes: plans made through the harness in a test
    session get option resident = 0 unless a test asks for it; the all-iterations-in-one-launch path for small
    2-D grids, which the library would otherwise pick for many of these shapes, has its own suite
    (test_resident_gpu.py) that passes resident = 1."""
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2210_01238_amd import harness
    harness.DEFAULT_OPTIONS["resident"] = 0
    return harness
