"""residual_norm_noalloc - the entry point for callers that cannot allocate device memory - against
residual_norm (same kernels, same summation order: the two must agree bit for bit) and against the
CPU oracle (1e-12 relative for fp64 grids, 1e-5 for fp32), called through the C ABI.  Two calls in a
row share the library's one static scratch array; the second uses a smaller input, so it must not be
disturbed by what the first left behind."""
import ctypes

import numpy as np
import pytest

from parity_util import random_padded


def both_norms(H, raw, a, tiles):
    """(residual_norm, residual_norm_noalloc) of the field `a`, through the raw C ABI."""
    import torch
    dims = [n - 2 for n in a.shape]
    r = H.JacobiRun(dims, tiles, a.dtype)
    try:
        r.load(a)
        out = torch.full((2,), -1.0, dtype=torch.float64, device="cuda")
        st = ctypes.c_void_p(int(torch.cuda.current_stream().cuda_stream))
        plan, grid = ctypes.c_void_p(r.plan), ctypes.c_void_p(r.cur.data_ptr())
        # the new entry point first, on a plan that has NOT been through residual_norm: it must not depend on
        # the plan's own scratch
        rc = raw.residual_norm_noalloc(plan, grid, ctypes.c_void_p(out[1:2].data_ptr()), st)
        assert rc == 0, H.B.jacobi_last_error()
        rc = raw.residual_norm(plan, grid, ctypes.c_void_p(out[0:1].data_ptr()), st)
        assert rc == 0, H.B.jacobi_last_error()
        torch.cuda.synchronize()
        return out.cpu().tolist()
    finally:
        r.close()


@pytest.mark.gpu
def test_noalloc_residual_matches_residual_norm_twice_in_a_row(H, oracle_mod):
    raw = ctypes.CDLL(H.B.LIB_PATH)
    for f in (raw.residual_norm, raw.residual_norm_noalloc):
        f.argtypes = [ctypes.c_void_p] * 4
        f.restype = ctypes.c_int
    # first a grid of several tiles with ragged rows (4608 workgroups), then a much smaller 3-D one
    # (fewer partial sums than the first call left in the array), then fp32
    cases = [(random_padded((768, 1100), seed=11), (3, 2), 1e-12),
             (random_padded((24, 20, 36), seed=12), (2, 2, 3), 1e-12),
             (random_padded((40, 300), dtype=np.float32, seed=13), (2, 3), 1e-5)]
    for a, tiles, rtol in cases:
        plain, noalloc = both_norms(H, raw, a, tiles)
        ref = oracle_mod.residual(a)
        assert noalloc == plain, (a.shape, plain, noalloc)           # same kernels, same order: same bits
        assert abs(noalloc - ref) <= rtol * ref, (a.shape, noalloc, ref)


@pytest.mark.gpu
def test_noalloc_residual_inside_a_hip_graph_on_an_unprepared_plan(H, oracle_mod):
    """The case the entry point exists for: recorded into a HIP graph on a plan that never ran
    jacobi_prepare (residual_norm itself would have to allocate there).  Between the replays another,
    smaller plan's call overwrites the start of the shared array: nothing in it has to survive."""
    import torch
    a = random_padded((256, 384), seed=21)
    b = random_padded((16, 16, 24), seed=22)
    ref_a, ref_b = oracle_mod.residual(a), oracle_mod.residual(b)
    plan = H.B.jacobi_create((256, 384), (2, 3))          # never prepared: only the no-alloc call touches it
    grid = torch.empty(H.B.jacobi_grid_bytes(plan), dtype=torch.uint8, device="cuda")
    other = H.JacobiRun((16, 16, 24), (2, 2, 2))
    filler = H.JacobiRun((256, 384), (2, 3))              # same layout; used to scatter `a` into `grid`
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    try:
        other.load(b)
        g_dev = torch.from_numpy(a).cuda()
        H.B.jacobi_scatter(filler.plan, g_dev.data_ptr(), grid.data_ptr(), int(torch.cuda.current_stream().cuda_stream))
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            # a device's first call looks up the array's address: outside the capture
            H.B.residual_norm_noalloc(plan, grid.data_ptr(), out[0:1].data_ptr(), int(s.cuda_stream))
        torch.cuda.synchronize()
        eager = out[0].item()
        assert abs(eager - ref_a) <= 1e-12 * ref_a
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            H.B.residual_norm_noalloc(plan, grid.data_ptr(), out[0:1].data_ptr(), int(torch.cuda.current_stream().cuda_stream))
        for k in range(3):
            out.zero_()
            H.B.residual_norm_noalloc(other.plan, other.cur.data_ptr(), out[1:2].data_ptr(),
                                      int(torch.cuda.current_stream().cuda_stream))
            torch.cuda.synchronize()
            assert abs(out[1].item() - ref_b) <= 1e-12 * ref_b, k
            graph.replay()
            torch.cuda.synchronize()
            assert out[0].item() == eager, (k, out[0].item(), eager)
    finally:
        torch.cuda.synchronize()
        other.close()
        filler.close()
        H.B.jacobi_destroy(plan)


def test_noalloc_residual_rejects_plans_beyond_its_scratch_without_a_device():
    """Size and argument checks come before any device call."""
    import paper_2210_01238_amd as J
    big = J.jacobi_create((32768, 32768), (8, 8))         # 131072 one-workgroup groups of 16-row strips x 4 = too many
    try:
        J.jacobi_set_option(big, "rows_per_strip", 1)
        with pytest.raises(J.JacobiError) as e:
            J.residual_norm_noalloc(big, 256, 512)
        assert e.value.code == J.binding.JACOBI_EINVAL and "131072" in str(e.value)
        for bad in (lambda: J.residual_norm_noalloc(big, 0, 512), lambda: J.residual_norm_noalloc(big, 256, 0),
                    lambda: J.residual_norm_noalloc(big, 264, 512), lambda: J.residual_norm_noalloc(None, 256, 512)):
            with pytest.raises(J.JacobiError) as e:
                bad()
            assert e.value.code == J.binding.JACOBI_EINVAL
    finally:
        J.jacobi_destroy(big)
