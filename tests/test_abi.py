"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header
declares, computes the documented layout, and reports argument errors before any
device call (so these run on a machine without a GPU)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def J():
    import paper_2210_01238_amd as J
    return J


def declared_functions():
    text = open(os.path.join(ROOT, "include", "jacobi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(\w+)\s*\([^;{]*\)\s*;", text)))


def test_header_and_exports_agree(J):
    decl = declared_functions()
    assert sorted(J.EXPORTS) == decl
    raw = ctypes.CDLL(J.LIB_PATH)
    for name in decl:
        assert hasattr(raw, name), name


def test_header_is_plain_c_and_the_library_links_from_c(J, tmp_path):
    """include/jacobi.h compiled as strict C99 by gcc, a small C program linked against the built library and
    run: plan creation, layout, options, pass planning and argument errors, none of which touches a device."""
    import subprocess
    src = os.path.join(ROOT, "tests", "c_client", "client.c")
    exe = str(tmp_path / "client")
    libdir = os.path.dirname(J.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    src, "-o", exe, "-L", libdir, "-l:" + os.path.basename(J.LIB_PATH), "-Wl,-rpath," + libdir],
                   check=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0 and out.stdout.strip().endswith("c client ok"), out.stdout + out.stderr


def test_core_entry_points_present(J):
    for name in ("jacobi_create", "jacobi_sweep", "halo_exchange", "residual_norm"):
        assert name in J.EXPORTS


def test_layout_2d(J):
    p = J.jacobi_create((16384, 16384), (8, 8), J.JACOBI_F64)
    L = J.jacobi_get_layout(p)
    assert (L.ndim, L.ntiles, L.nplanes) == (2, 64, 1)
    assert list(L.tile) == [1, 2048, 2048] and list(L.tiles) == [1, 8, 8]
    assert L.pitch == 2048 and L.plane == 2050 * 2048 and L.xhalo_offset == L.plane
    assert L.xhalo_pitch % 16 == 0 and L.xhalo_pitch >= 2050
    assert L.xsend_offset == L.xhalo_offset + 2 * L.xhalo_pitch and L.tile_stride == L.xsend_offset + 2 * L.xhalo_pitch
    assert L.grid_bytes == 64 * L.tile_stride * 8 == J.jacobi_grid_bytes(p)
    assert (L.pitch * 8) % 128 == 0 and (L.tile_stride * 8) % 128 == 0
    J.jacobi_destroy(p)


def test_layout_ragged_and_f32_and_3d(J):
    p = J.jacobi_create((30, 100), (3, 4), J.JACOBI_F32)
    L = J.jacobi_get_layout(p)
    assert list(L.tile) == [1, 10, 25] and L.pitch == 32 and L.dtype == J.JACOBI_F32
    assert L.grid_bytes == 12 * L.tile_stride * 4
    J.jacobi_destroy(p)
    p = J.jacobi_create((512, 512, 512), (4, 4, 4), J.JACOBI_F64)
    L = J.jacobi_get_layout(p)
    assert L.nplanes == 130 and L.plane == 130 * 128 and L.xhalo_offset == 130 * L.plane
    assert L.xhalo_pitch >= 130 * 130
    J.jacobi_destroy(p)


@pytest.mark.parametrize("dims,tiles,dtype,code", [
    ((10, 10), (3, 2), 0, 2), ((0, 10), (1, 1), 0, 1), ((10, 10), (0, 1), 0, 1),
    ((10, 10), (1, 1), 7, 1), ((10,), (1,), 0, 1), ((4, 4, 4, 4), (1, 1, 1, 1), 0, 1),
    ((-5, 10), (1, 1), 0, 1), ((8, 8, 9), (2, 2, 2), 1, 2),
    ((1, 20000, 20000), (1, 1, 1), 0, 1),       # a plane of a 3-D tile must stay below 2 GiB
])
def test_create_rejects(J, dims, tiles, dtype, code):
    with pytest.raises(J.JacobiError) as e:
        J.jacobi_create(dims, tiles, dtype)
    assert e.value.code == code and J.jacobi_last_error() != ""


def test_null_and_argument_errors_without_device(J):
    raw = J.binding.lib
    assert raw.jacobi_create(None, 2, None, None, 0) == J.binding.JACOBI_EINVAL
    h = ctypes.c_void_p()
    d = (ctypes.c_int64 * 2)(8, 8)
    assert raw.jacobi_create(ctypes.byref(h), 2, d, None, 0) == 1 and not h.value
    p = J.jacobi_create((8, 8), (2, 2))
    # argument validation happens before any HIP call
    nb = J.jacobi_grid_bytes(p)
    for call in (lambda: J.jacobi_sweep(p, 0, 256, 1), lambda: J.jacobi_sweep(p, 256, 256, 1),
                 lambda: J.jacobi_sweep(p, 256, 256 + 8, 1),               # misaligned
                 lambda: J.jacobi_sweep(p, 4096, 4096 + nb - 16, 1),       # overlapping
                 lambda: J.halo_exchange(p, 264), lambda: J.residual_norm(p, 264, 256),
                 lambda: J.jacobi_sweep(p, 256, 256 + nb, -1), lambda: J.halo_exchange(p, 0),
                 lambda: J.jacobi_run(p, 256, 256 + nb, 4, 2, None), lambda: J.jacobi_run(p, 256, 256 + nb, -1, 2, 768),
                 lambda: J.jacobi_run(p, 256, 256 + nb, 4, -1, 768), lambda: J.jacobi_run(p, 256, 256, 4, 2, 768),
                 lambda: J.jacobi_run(p, 0, 256, 4, 2, 768),
                 lambda: J.jacobi_sweep_residual(p, 256, 256 + nb, 0, 768), lambda: J.jacobi_sweep_residual(p, 256, 256 + nb, 1, 0),
                 lambda: J.residual_norm(p, 0, 256), lambda: J.residual_norm(p, 256, 0),
                 lambda: J.jacobi_scatter(p, 0, 256), lambda: J.jacobi_gather(p, 256, 0),
                 lambda: J.jacobi_set_option(p, "no_such_option", 1),
                 lambda: J.jacobi_set_option(p, "fused", 2), lambda: J.jacobi_set_option(p, "nontemporal", 3),
                 lambda: J.jacobi_set_option(p, "tblock", 0), lambda: J.jacobi_set_option(p, "tblock", 13),
                 lambda: J.jacobi_set_option(p, "unroll", 3),
                 lambda: J.jacobi_set_option(p, "rows_per_strip", 5000),
                 lambda: J.jacobi_get_option(p, "bogus")):
        with pytest.raises(J.JacobiError) as e:
            call()
        assert e.value.code == 1
    assert J.jacobi_sweep(p, 256, 256 + nb, 0) == 256     # zero iterations: no-op, result in `in`
    assert J.jacobi_run(p, 256, 256 + nb, 0, 2, None) == 256
    J.jacobi_set_option(p, "fused", 0)
    assert J.jacobi_get_option(p, "fused") == 0
    assert J.jacobi_grid_bytes(None) == 0
    J.jacobi_destroy(p)
    J.jacobi_destroy(None)


def test_pass_schedule_host_logic(J):
    """The pass planner (host only): iterations spread evenly over the fewest passes the depth allows."""
    def sched(dims, tiles, dtype, iters, **opts):
        p = J.jacobi_create(dims, tiles, dtype)
        opts.setdefault("resident", 0)          # the launch-per-pass planner; the one-launch path is checked below
        for k, v in opts.items():
            J.jacobi_set_option(p, k, v)
        try:
            return J.jacobi_pass_schedule(p, iters)
        finally:
            J.jacobi_destroy(p)
    assert sched((64, 64), (2, 2), 0, 7) == [1] * 7                       # default: one iteration per pass
    assert sched((64, 64), (2, 2), 0, 0) == []
    assert sched((64, 64), (2, 2), 0, 10, tblock=8) == [5, 5]             # not 8 + 2
    assert sched((64, 64), (2, 2), 0, 17, tblock=8) == [6, 6, 5]
    assert sched((64, 64), (2, 2), 0, 9, tblock=2) == [2, 2, 2, 2, 1]
    assert sched((64, 64), (2, 2), 0, 3, tblock=8) == [3]
    # passes of 8 or more iterations cost the same per iteration: as many passes as fit at >= 8 each
    assert sched((64, 64), (2, 2), 0, 10, tblock=12) == [10]
    assert sched((64, 64), (2, 2), 0, 13, tblock=12) == [7, 6]
    assert sched((64, 64), (2, 2), 0, 17, tblock=12) == [9, 8]
    assert sched((64, 64), (2, 2), 0, 20, tblock=12) == [10, 10]
    assert sched((64, 64), (2, 2), 0, 50, tblock=12) == [9, 9, 8, 8, 8, 8]
    assert sched((64, 64), (2, 2), 0, 100, tblock=12) == [9] * 4 + [8] * 8
    assert sched((64, 64), (8, 8), 0, 24, tblock=12) == [8, 8, 8]          # tile height 8 limits the depth
    # grids of 1 GiB and more: passes of 10 or more
    assert sched((16384, 16384), (8, 8), 0, 50, tblock=12) == [10] * 5
    assert sched((16384, 16384), (8, 8), 0, 100, tblock=12) == [10] * 10
    assert sched((16384, 16384), (8, 8), 0, 24, tblock=12) == [12, 12]
    assert sched((16384, 16384), (8, 8), 0, 17, tblock=12) == [9, 8]
    assert sched((16384, 16384), (8, 8), 0, 10, tblock=8) == [5, 5]
    assert sched((64, 64), (16, 16), 0, 10, tblock=12) == [4, 3, 3]        # tile height 4
    assert sched((40, 36), (1, 36), 0, 6, tblock=8) == [1] * 6            # tiles one column wide: single steps
    assert sched((12, 63), (4, 1), 0, 8, tblock=8) == [2, 2, 2, 2]        # odd width, height 3: two-step kernel only
    # 3-D: fp64 up to 4 iterations per pass, fp32 up to 3
    assert sched((32, 32, 32), (2, 2, 2), 0, 10, tblock=8) == [4, 3, 3]
    assert sched((32, 32, 32), (2, 2, 2), 1, 10, tblock=8) == [3, 3, 2, 2]
    assert sched((32, 32, 32), (2, 2, 2), 0, 10, tblock=8, cooperative=0) == [3, 3, 2, 2]
    assert sched((32, 32, 32), (2, 2, 2), 1, 10, tblock=8, cooperative=0) == [2] * 5
    assert sched((32, 32, 33), (2, 2, 1), 0, 5, tblock=8) == [1] * 5      # odd tile width: single steps
    assert sched((6, 32, 32), (3, 2, 2), 0, 9, tblock=4) == [2, 2, 2, 2, 1]   # tile depth 2 limits the pass depth
    # small 2-D grids (rows of at most 2 KiB, tile width a multiple of 16 bytes): all iterations in one launch,
    # cut into equally deep phases of at most 20 (option resident_depth) iterations - fewer if the rows would
    # then need more workgroups than the device has CUs; a grid whose rows (plus the two ring rows) fit one
    # workgroup's 16 wavefronts x 3 rows (4 for rows of at most 1 KiB) needs a single phase
    assert sched((256, 256), (1, 1), 0, 100, resident=1) == [20] * 5
    assert sched((256, 256), (4, 4), 0, 100, resident=1, tblock=8) == [20] * 5
    assert sched((256, 256), (1, 1), 0, 100, resident=1, resident_depth=31) == [20] * 5     # 48 rows held: at most 23 deep
    assert sched((256, 256), (1, 1), 0, 100, resident=1, resident_depth=6) == [6] * 15 + [5] * 2
    assert sched((256, 256), (1, 1), 0, 10, resident=1) == [10]
    assert sched((46, 256), (1, 1), 0, 1000, resident=1) == [1000]
    assert sched((47, 256), (1, 1), 0, 100, resident=1) == [20] * 5
    assert sched((62, 128), (1, 1), 0, 1000, resident=1) == [1000]
    assert sched((63, 128), (1, 1), 0, 100, resident=1) == [20] * 5
    assert sched((46, 256), (1, 1), 0, 100, resident=1, resident_rows=2) == [15, 15] + [14] * 5   # 32 rows held: two workgroups
    assert sched((4096, 256), (1, 1), 0, 100, resident=1) == [15, 15] + [14] * 5     # 18 owned rows each: 228 workgroups
    assert sched((8000, 256), (1, 1), 0, 100, resident=1) == [8] * 9 + [7] * 4
    assert sched((12000, 256), (1, 1), 0, 5, resident=1) == [1] * 5          # more workgroups than CUs at any depth
    assert sched((256, 258), (1, 1), 0, 5, resident=1) == [1] * 5           # three vectors per lane: not taken
    assert sched((256, 512), (1, 1), 1, 5, resident=1) == [5]               # fp32: 512 columns are two vectors per lane
    assert sched((256, 254), (1, 127), 0, 5, resident=1) == [5]             # tiles two columns wide
    assert sched((64, 63), (1, 1), 0, 5, resident=1) == [1] * 5             # odd tile width
    assert sched((16, 16, 16), (1, 1, 1), 0, 5, resident=1) == [1] * 5      # 3-D
    p = J.jacobi_create((8, 8), (1, 1))
    raw = J.binding.lib
    n = ctypes.c_int()
    assert raw.jacobi_pass_schedule(p, 3, None, 0, None) == 1
    assert raw.jacobi_pass_schedule(p, -1, None, 0, ctypes.byref(n)) == 1
    assert raw.jacobi_pass_schedule(p, 3, None, 2, ctypes.byref(n)) == 1
    buf = (ctypes.c_int * 2)(7, 7)
    J.jacobi_set_option(p, "resident", 0)
    assert raw.jacobi_pass_schedule(p, 5, buf, 2, ctypes.byref(n)) == 0 and n.value == 5 and list(buf) == [1, 1]
    J.jacobi_destroy(p)


def test_scratch_size_covers_every_option_setting(J):
    """jacobi_scratch_bytes (host only): one double per workgroup of the finest-grained residual launch
    (strips of one row or plane, one row per wavefront; 2-D: at least the 1024 the all-iterations-in-one-launch
    kernel may use), plus the host-result slot and 16 bytes of barrier words; independent of the
    option values, so jacobi_prepare's allocation never has to grow."""
    def nbytes(dims, tiles, dtype=0, **opts):
        p = J.jacobi_create(dims, tiles, dtype)
        for k, v in opts.items():
            J.jacobi_set_option(p, k, v)
        try:
            return J.jacobi_scratch_bytes(p)
        finally:
            J.jacobi_destroy(p)
    # 16384^2 as 8 x 8 tiles, 4 strips per workgroup.  Single steps: 64 tiles x 16 column segments x 2048
    # one-row strips; the deepest blocked passes cut a whole row of tiles into segments of 104 owned columns
    # (52 of 64 lanes): 8 rows of tiles x ceil(16384 / 104) = 158 segments x 2048 strips, which is more
    assert nbytes((16384, 16384), (8, 8)) == 8 * (8 * 158 * 2048 // 4 + 1) + 16
    assert nbytes((16384, 16384), (8, 8), tblock=12, rows_per_strip=64) == nbytes((16384, 16384), (8, 8))
    # 512^3 as 4 x 4 x 4 tiles of 128^3: 64 tiles x 128 rows x 128 planes x 1 segment
    assert nbytes((512, 512, 512), (4, 4, 4)) == 8 * (64 * 128 * 128 // 4 + 1) + 16
    assert nbytes((512, 512, 512), (4, 4, 4), rows_per_wave=4, cooperative=0) == nbytes((512, 512, 512), (4, 4, 4))
    # fp32 rows of 128 cells use 8-byte lanes only with 4 rows per wavefront; finest is still 1 row per strip
    assert nbytes((512, 512, 512), (4, 4, 4), 1) == 8 * (64 * 128 * 128 // 4 + 1) + 16
    # small 2-D plans: the one-launch kernel's per-workgroup sums (at most 1024 workgroups)
    assert nbytes((1, 1), (1, 1)) == 8 * (1024 + 1) + 16
    assert nbytes((1, 1, 1), (1, 1, 1)) == 32
    assert J.jacobi_scratch_bytes(None) == 0
    with pytest.raises(J.JacobiError):
        J.jacobi_prepare(None)


def test_workgroup_limit_request_arithmetic(J):
    """The LDS request that caps the workgroups per CU (host arithmetic; the launch confirms its effect with the
    occupancy query).  How many 256-thread workgroups share a 160 KiB CU for a given request was measured
    (and is what the occupancy calculator reports): up to 20000 bytes 8, 26000 6, 32000 5, 40000 4,
    49152-53589 3, 65536-81000 2, 100000 and more 1.  The requests must lie well inside the range for n."""
    p = J.jacobi_create((16384, 16384), (8, 8))
    try:
        assert J.jacobi_get_option(p, "lds_request_1") == 0 and J.jacobi_get_option(p, "lds_request_2") == 0   # size unknown
        assert J.jacobi_get_option(p, "num_cu") == 256 and J.jacobi_get_option(p, "lds_limit_failed") == 0
        J.jacobi_set_option(p, "cu_lds", 163840)
        one, two = J.jacobi_get_option(p, "lds_request_1"), J.jacobi_get_option(p, "lds_request_2")
        assert one == 163840 - 4096 and 100000 <= one <= 163840
        assert two == 81920 - 4096 and 65536 <= two <= 81000
        J.jacobi_set_option(p, "cu_lds", 65536)            # a 64 KiB CU: one workgroup takes (nearly) all of it
        assert J.jacobi_get_option(p, "lds_request_1") == 65536 - 4096
        for bad in (lambda: J.jacobi_set_option(p, "lds_limit_failed", 0), lambda: J.jacobi_set_option(p, "num_cu", 8),
                    lambda: J.jacobi_set_option(p, "cu_lds", -1), lambda: J.jacobi_set_option(p, "cu_lds", 1 << 21)):
            with pytest.raises(J.JacobiError):
                bad()
        J.jacobi_set_option(p, "cu_lds", 1000)             # below 64 KiB: no limits
        assert J.jacobi_get_option(p, "lds_request_1") == 0
    finally:
        J.jacobi_destroy(p)


def access_sets(dims, tiles, task_tiles):
    """Cells (as padded global indices) a task of tiles `task_tiles` READS from the grid the previous iteration
    wrote - every interior cell of its tiles and the face-neighbour cells beyond them that lie inside the
    domain - and the cells it WRITES: its tiles' interiors."""
    import itertools
    tile = [d // t for d, t in zip(dims, tiles)]
    reads, writes = set(), set()
    for t in task_tiles:
        idx = list(np.unravel_index(t, tiles))
        lo = [i * s + 1 for i, s in zip(idx, tile)]
        for cell in itertools.product(*[range(l, l + s) for l, s in zip(lo, tile)]):
            writes.add(cell)
            reads.add(cell)
            for d in range(len(dims)):
                for step in (-1, 1):
                    nb = list(cell); nb[d] += step
                    if 1 <= nb[d] <= dims[d]:
                        reads.add(tuple(nb))
    return reads, writes


@pytest.mark.parametrize("dims,tiles,group", [
    ((8, 12), (4, 3), 1), ((8, 12), (4, 3), 2), ((8, 12), (4, 3), 5), ((8, 12), (4, 3), 12), ((8, 12), (4, 3), 100),
    ((6, 6), (1, 6), 1), ((6, 6), (6, 1), 4), ((5, 5), (1, 1), 1),
    ((4, 6, 4), (2, 3, 2), 1), ((4, 6, 4), (2, 3, 2), 3), ((4, 6, 4), (2, 3, 2), 7), ((2, 2, 6), (1, 1, 3), 2),
])
def test_task_dependencies_follow_from_read_and_write_sets(J, dims, tiles, group):
    """The dependency lists jacobi_sweep_tasks uses against lists derived here from what the tasks touch: task a
    of iteration k+1 depends on task b of iteration k exactly if a reads a cell that b writes (paper Sec. IV-A)."""
    p = J.jacobi_create(dims, tiles)
    try:
        got = J.jacobi_task_dependencies(p, group)
    finally:
        J.jacobi_destroy(p)
    ntiles = int(np.prod(tiles))
    g = min(group, ntiles)
    tasks = [list(range(s, min(s + g, ntiles))) for s in range(0, ntiles, g)]
    sets = [access_sets(dims, tiles, tt) for tt in tasks]
    want = [sorted(b for b in range(len(tasks)) if sets[a][0] & sets[b][1]) for a in range(len(tasks))]
    assert got == want
    # the relation is symmetric (face adjacency) and reflexive, so the same edges cover write-after-read on the ping-pong grids
    for a, deps in enumerate(got):
        assert a in deps and all(a in got[b] for b in deps)


def test_task_dependencies_argument_errors(J):
    p = J.jacobi_create((8, 12), (4, 3))
    try:
        n, nt = ctypes.c_int(), ctypes.c_int()
        raw = J.binding.lib
        assert raw.jacobi_task_dependencies(p, 2, 0, None, 0, ctypes.byref(n), ctypes.byref(nt)) == 0 and nt.value == 6
        assert raw.jacobi_task_dependencies(p, 2, 6, None, 0, ctypes.byref(n), None) == 1       # task out of range
        assert raw.jacobi_task_dependencies(p, 0, 0, None, 0, ctypes.byref(n), None) == 1
        assert raw.jacobi_task_dependencies(p, 2, 0, None, 3, ctypes.byref(n), None) == 1       # capacity without a buffer
        assert raw.jacobi_task_dependencies(None, 2, 0, None, 0, ctypes.byref(n), None) == 1
    finally:
        J.jacobi_destroy(p)


def test_launch_configuration_of_the_workloads_is_what_was_measured(J):
    """The settings the 0 = "choose" options resolve to (host-only figures): the configured workloads must keep
    the launch configuration their measurements and profiles were taken with, whatever is tuned for other sizes."""
    import jacobi_inputs as gen
    keys = ("rows_per_strip", "rows_per_wave", "unroll", "xcd_chunk", "strips", "one_workgroup_per_cu", "streaming_stores")

    def chosen(dims, tiles, prefix="update_", dtype=0, **opts):
        p = J.jacobi_create(dims, tiles, dtype)
        try:
            for k, v in opts.items():
                J.jacobi_set_option(p, k, v)
            return [J.jacobi_get_option(p, prefix + k) for k in keys]
        finally:
            J.jacobi_destroy(p)

    W = gen.WORKLOADS
    # 2-D: strips of 8 rows with all loads in flight, XCD chunks of 8, streaming stores beyond the Infinity Cache
    assert chosen(W["C3"].dims, W["C3"].tiles) == [8, 1, 8, 8, 64 * 16 * 256, 0, 1]
    assert chosen(W["C5"].dims, W["C5"].tiles) == [8, 1, 8, 8, 4096 * 16, 0, 1]
    assert chosen(W["C2"].dims, W["C2"].tiles) == [4, 1, 4, 8, 16 * 8 * 256, 0, 1]          # 2 x 128.8 MiB: left streaming
    # 3-D grids of 1 GiB and more: 16 planes x 4 rows, one plane per trip, one workgroup per CU, chunks of 16
    assert chosen(W["C4"].dims, W["C4"].tiles) == [16, 4, 1, 16, 64 * 32 * 8, 1, 1]
    assert chosen(W["P1"].dims, W["P1"].tiles) == [16, 4, 1, 16, 384 * 32 * 8, 1, 1]
    # their stand-alone residual passes
    assert chosen(W["C4"].dims, W["C4"].tiles, "residual_") == [16, 4, 2, 8, 64 * 32 * 8, 0, 1]
    # explicit options win
    assert chosen(W["C3"].dims, W["C3"].tiles, rows_per_strip=16, unroll=4, xcd_chunk=3, nontemporal=0)[:4] + [0] == [16, 1, 4, 3, 0]
    # cache-resident grids: plain stores; 2-D from 24 MiB on in XCD chunks of 32; small 3-D grids get about a
    # thousand wavefronts of 2 rows (1 on tiny ones), one plane per trip, the hardware's order
    assert chosen((3072, 3072), (4, 4)) == [4, 1, 4, 32, 18432, 0, 0]
    assert chosen((1024, 1024), (2, 2))[3:] == [8, 4096, 0, 0]
    assert chosen((64, 64, 64), (1, 1, 1)) == [2, 2, 1, 1, 1024, 0, 0]
    assert chosen((32, 32, 32), (1, 1, 1)) == [2, 1, 1, 1, 512, 0, 0]
    assert chosen((192, 192, 192), (2, 2, 2)) == [16, 2, 1, 16, 2304, 0, 0]
    assert chosen((256, 256, 256), (2, 2, 2)) == [16, 4, 1, 16, 2048, 0, 1]                  # 136 MiB: beyond the cache
    assert chosen((128, 128, 128), (1, 1, 1), dtype=1)[1] == 4                                # fp32 rows of 128 cells: 8-byte lanes
    with pytest.raises(J.JacobiError):
        chosen((64, 64), (1, 1), "update_nonsense_")


def test_task_execution_argument_errors_without_device(J):
    """Arguments of jacobi_sweep_tasks are checked before any device call."""
    p = J.jacobi_create((48, 48), (48, 48))
    nb = J.jacobi_grid_bytes(p)
    for bad in (lambda: J.jacobi_sweep_tasks(p, 256, 256 + nb, 1, 1, 17), lambda: J.jacobi_sweep_tasks(p, 256, 256 + nb, 1, 0, 4),
                lambda: J.jacobi_sweep_tasks(p, 256, 256 + nb, 1, 1, 0), lambda: J.jacobi_sweep_tasks(p, 256, 256, 1, 1, 4),
                lambda: J.jacobi_sweep_tasks(p, 0, 256, 1, 1, 4), lambda: J.jacobi_sweep_tasks(p, 256, 256 + nb, -1, 1, 4)):
        with pytest.raises(J.JacobiError) as e:
            bad()
        assert e.value.code == 1
    assert J.jacobi_sweep_tasks(p, 256, 256 + nb, 0, 1, 4) == 256       # zero iterations: nothing touched
    J.jacobi_destroy(p)
