"""GPU parity: the HIP library (called through its C ABI) against the CPU oracle,
element by element on the same seeded inputs.  fp64 grids must be bit-identical
(both sides evaluate 0.25*((W+E)+(S+N)) / C6*(((x-+x+)+(y-+y+))+(z-+z+)) with FP
contraction off); fp32 grids within 1e-5*max|u|; residual norms within 1e-12
relative (fp64 grids) / 1e-5 (fp32 grids) because the summation order differs."""
import numpy as np
import pytest

import jacobi_inputs as gen
from parity_util import interior, random_padded, read_tile_cell

pytestmark = pytest.mark.gpu

RES_RTOL = {np.dtype(np.float64): 1e-12, np.dtype(np.float32): 1e-5}


def run_case(H, oracle, a, tiles, iters, res_every=0, **opts):
    r = H.JacobiRun([n - 2 for n in a.shape], tiles, a.dtype, **opts)
    try:
        r.load(a)
        res = r.run(iters, res_every)
        out = r.fetch()
    finally:
        r.close()
    ref, ref_res = oracle.run(a, iters, res_every)
    return out, res, ref, ref_res


def check(out, res, ref, ref_res):
    dt = out.dtype
    if dt == np.float64:
        assert np.array_equal(out, ref), f"max diff {np.max(np.abs(out - ref))}"
    else:
        assert np.max(np.abs(out.astype(np.float64) - ref)) <= 1e-5 * np.max(np.abs(ref))
    assert len(res) == len(ref_res)
    for g, o in zip(res, ref_res):
        assert abs(g - o) <= RES_RTOL[np.dtype(dt)] * max(o, 1e-300), (g, o)


CASES_2D = [
    # (interior dims, tiles, iters, residual_every)
    ((256, 256), (1, 1), 20, 5),        # one tile, two column segments
    ((96, 200), (3, 2), 13, 4),         # tw = 100: ragged row (pitch 112), several tiles
    ((64, 1030), (2, 2), 9, 3),         # tw = 515: 5 column segments, ragged last one
    ((48, 48), (48, 48), 7, 7),         # 1x1 tiles: every cell is a tile edge
    ((40, 36), (1, 36), 6, 2),          # tiles one column wide
    ((36, 40), (36, 1), 6, 2),          # tiles one row high
    ((300, 70), (1, 1), 11, 11),        # tall single tile, odd sizes
    ((512, 512), (4, 4), 50, 10),       # 4x4 tiles of 128^2
    ((1024, 1024), (8, 8), 25, 5),      # 64 tiles of 128^2 (fine-grained tasking shape)
    ((2, 2), (1, 1), 5, 1),
    ((1, 1), (1, 1), 3, 1),
]


@pytest.mark.parametrize("fused", [0, 1])
@pytest.mark.parametrize("dims,tiles,iters,every", CASES_2D)
def test_2d_fp64_bit_exact(H, oracle_mod, dims, tiles, iters, every, fused):
    a = random_padded(dims, seed=sum(dims) + iters)
    check(*run_case(H, oracle_mod, a, tiles, iters, every, fused=fused))


CASES_3D = [
    ((24, 20, 36), (2, 2, 3), 9, 3),
    ((16, 16, 16), (1, 1, 1), 8, 4),
    ((6, 10, 130), (3, 5, 1), 5, 5),    # tw = 130: two column segments, ragged
    ((8, 8, 8), (8, 8, 8), 4, 2),       # 1x1x1 tiles
    ((128, 128, 128), (4, 4, 4), 12, 4),  # 64 tiles of 32^3
    ((70, 33, 20), (1, 1, 1), 6, 3),
    ((1, 1, 1), (1, 1, 1), 2, 1),
]


@pytest.mark.parametrize("fused", [0, 1])
@pytest.mark.parametrize("dims,tiles,iters,every", CASES_3D)
def test_3d_fp64_bit_exact(H, oracle_mod, dims, tiles, iters, every, fused):
    a = random_padded(dims, seed=sum(dims) + iters)
    check(*run_case(H, oracle_mod, a, tiles, iters, every, fused=fused))


@pytest.mark.parametrize("dims,tiles,iters,every", [
    ((96, 200), (3, 2), 13, 4), ((512, 512), (4, 4), 50, 10), ((24, 20, 36), (2, 2, 3), 9, 3),
    ((64, 64, 64), (2, 2, 2), 10, 5), ((40, 1000), (2, 1), 8, 4),
])
@pytest.mark.parametrize("fused", [0, 1])
def test_fp32_within_tolerance(H, oracle_mod, dims, tiles, iters, every, fused):
    a = random_padded(dims, dtype=np.float32, seed=7)
    check(*run_case(H, oracle_mod, a, tiles, iters, every, fused=fused))


@pytest.mark.parametrize("opts", [
    dict(rows_per_strip=1), dict(rows_per_strip=3, unroll=2), dict(rows_per_strip=7, fused=0, unroll=4),
    dict(rows_per_strip=4096, unroll=8), dict(nontemporal=0), dict(nontemporal=2), dict(nontemporal=0, fused=0, rows_per_strip=5), dict(unroll=16, rows_per_strip=16),
    dict(xcd_chunk=1), dict(xcd_chunk=3, unroll=1), dict(xcd_chunk=1000),
    dict(rows_per_wave=1), dict(rows_per_wave=2, unroll=4), dict(rows_per_wave=4, unroll=1, rows_per_strip=3),
    dict(stack=1), dict(stack=4), dict(stack=8, xcd_chunk=5),
])
def test_options_do_not_change_results(H, oracle_mod, opts):
    a = random_padded((150, 260), seed=3)
    check(*run_case(H, oracle_mod, a, (3, 2), 10, 5, **opts))
    b = random_padded((20, 18, 40), seed=4)
    check(*run_case(H, oracle_mod, b, (2, 3, 2), 6, 3, **opts))


@pytest.mark.parametrize("dims,tiles", [
    ((150, 260), (3, 2)),      # tiles 50 x 130: second band ragged (18 rows), two column segments, ragged width
    ((66, 128), (2, 1)),       # tiles 33 rows: one row in the second band
    ((64, 64), (1, 1)),        # exactly one band of 4 wavefronts (two of 8), half-empty lanes
    ((256, 100), (2, 2)),      # 128-row tiles: 4 bands of 32 / 2 of 64, tile seam in x and y
    ((520, 384), (1, 3)),      # 520 rows: 16 full bands of 32 + 8 rows
])
@pytest.mark.parametrize("stack", [4, 8])
def test_stacked_residual_pass(H, oracle_mod, dims, tiles, stack):
    """The 2-D residual pass with the wavefronts of a workgroup stacked (border rows through LDS), forced on small
    shapes: against the oracle and bit for bit against the unstacked pass on the same grid."""
    for dtype in (np.float64, np.float32):
        a = random_padded(dims, dtype=dtype, seed=sum(dims) + stack)
        ref, _ = oracle_mod.run(a, 3)
        want = oracle_mod.residual(ref)
        r = H.JacobiRun(dims, tiles, dtype, stack=stack)
        try:
            r.load(a)
            r.sweep(3)                       # leaves the inter-tile halo cells of the result to the pushes
            got = r.residual()
            r.set_option("stack", 1)
            plain = r.residual()
        finally:
            r.close()
        assert abs(got - want) <= RES_RTOL[np.dtype(dtype)] * want, (dims, tiles, stack, got, want)
        assert abs(got - plain) <= 1e-14 * plain           # other summation tree, same terms


def poison_inter_tile_halos(H, r):
    """NaN into every halo cell that has a neighbouring tile behind it (faces with their edges; Dirichlet
    halos untouched), and into the x send arrays: what a caller may leave there."""
    import torch
    lay = H.B.jacobi_get_layout(r.plan)
    Tz, Ty, Tx = lay.tiles
    td, th, tw = lay.tile
    tdt = torch.float64 if r.np_dtype == np.float64 else torch.float32
    raw = r.cur.view(tdt)
    host = raw.cpu().numpy().copy()
    rows, npl = th + 2, lay.nplanes
    for t in range(lay.ntiles):
        tz, ty, tx = t // (Ty * Tx), (t // Tx) % Ty, t % Tx
        base = t * lay.tile_stride
        main = host[base: base + npl * rows * lay.pitch].reshape(npl, rows, lay.pitch)
        xm = host[base + lay.xhalo_offset: base + lay.xhalo_offset + npl * rows].reshape(npl, rows)
        xp = host[base + lay.xhalo_offset + lay.xhalo_pitch: base + lay.xhalo_offset + lay.xhalo_pitch + npl * rows].reshape(npl, rows)
        ks = slice(1, td + 1) if lay.ndim == 3 else slice(0, 1)
        if ty > 0: main[ks, 0, :tw] = np.nan
        if ty < Ty - 1: main[ks, th + 1, :tw] = np.nan
        if tx > 0: xm[ks, 1:th + 1] = np.nan
        if tx < Tx - 1: xp[ks, 1:th + 1] = np.nan
        if lay.ndim == 3:
            if tz > 0: main[0, 1:th + 1, :tw] = np.nan
            if tz < Tz - 1: main[td + 1, 1:th + 1, :tw] = np.nan
        host[base + lay.xsend_offset: base + lay.xsend_offset + 2 * lay.xhalo_pitch] = np.nan
    raw.copy_(torch.from_numpy(host))


@pytest.mark.parametrize("dims,tiles", [
    ((96, 200), (3, 2)), ((150, 260), (3, 2)), ((48, 48), (48, 48)), ((64, 1030), (2, 2)),
    ((24, 20, 36), (2, 2, 3)), ((12, 26, 260), (2, 2, 2)),      # 13-row tiles: ragged last row group of 4
    ((9, 15, 40), (3, 5, 2)), ((8, 8, 8), (8, 8, 8)),
])
@pytest.mark.parametrize("opts", [dict(), dict(fused=0), dict(tblock=4)])
def test_stale_halo_cells_are_never_read_as_data(H, oracle_mod, dims, tiles, opts):
    """jacobi_sweep, jacobi_sweep_residual and residual_norm must not depend on what the inter-tile halo cells
    (or the x send arrays) hold when they are called: the first update of a call and the residual pass read
    the neighbouring tiles' edge cells themselves (with fused = 0 an exchange kernel runs first)."""
    import torch
    for dtype in (np.float64, np.float32):
        a = random_padded(dims, dtype=dtype, seed=sum(dims))
        r = H.JacobiRun(dims, tiles, dtype, **opts)
        try:
            r.load(a)
            poison_inter_tile_halos(H, r)
            res0 = r.residual()                                   # residual pass on poisoned halos
            poison_inter_tile_halos(H, r)
            dev = torch.zeros(1, dtype=torch.float64, device="cuda")
            r.sweep_residual(5, dev)                              # first update (with the fused residual) on poisoned halos
            poison_inter_tile_halos(H, r)
            r.sweep(4)
            poison_inter_tile_halos(H, r)
            res9 = r.residual()
            out = r.fetch()
        finally:
            r.close()
        ref, ref_res = oracle_mod.run(a, 9, 9)
        check(out, [res9], ref, ref_res)
        want0 = oracle_mod.residual(a)
        tol = RES_RTOL[np.dtype(dtype)]
        assert abs(res0 - want0) <= tol * want0 and abs(dev.item() - want0) <= tol * want0


def test_c1_workload_and_stored_values(H, oracle_mod):
    from test_oracle_pins import read_golden_c1
    w = gen.WORKLOADS["C1"]
    a = gen.generate(w)
    out, res, ref, ref_res = run_case(H, oracle_mod, a, w.tiles, w.iters, w.residual_every)
    check(out, res, ref, ref_res)
    gres, pts = read_golden_c1()
    assert abs(res[0] - gres) <= 1e-12 * gres
    for (i, j), v in pts.items():
        assert out[i, j] == v
    assert np.all(out[101:-1, 1:-1] == 0.0) and np.array_equal(out, out[:, ::-1])


def test_harmonic_lattice_fixed_point_on_gpu(H, oracle_mod):
    a = gen.lattice_field((130, 258), "i2-j2")
    out, res, ref, _ = run_case(H, oracle_mod, a, (4, 2), 6, 3)
    assert np.array_equal(out, a) and res == [0.0, 0.0]


def test_halo_exchange_fills_halos_and_is_idempotent(H):
    import torch
    dims, tiles = (24, 40), (3, 4)
    a = random_padded(dims, seed=11)
    r = H.JacobiRun(dims, tiles)
    try:
        r.load(a)
        lay = H.B.jacobi_get_layout(r.plan)
        th, tw, Tx = lay.tile[1], lay.tile[2], lay.tiles[2]
        # poison every inter-tile halo cell, then exchange
        raw = r.cur.view(torch.float64)
        host = raw.cpu().numpy().copy()
        for t in range(lay.ntiles):
            ty, tx = divmod(t, Tx)
            base = t * lay.tile_stride
            if ty > 0:
                host[base: base + tw] = np.nan
            if ty < tiles[0] - 1:
                host[base + (th + 1) * lay.pitch: base + (th + 1) * lay.pitch + tw] = np.nan
            if tx > 0:
                host[base + lay.xhalo_offset + 1: base + lay.xhalo_offset + 1 + th] = np.nan
            if tx < Tx - 1:
                o = base + lay.xhalo_offset + lay.xhalo_pitch
                host[o + 1: o + 1 + th] = np.nan
        raw.copy_(torch.from_numpy(host))
        r.exchange()
        once = raw.cpu().numpy().copy()
        r.exchange()
        twice = raw.cpu().numpy().copy()
        for t in range(lay.ntiles):
            ty, tx = divmod(t, Tx)
            for i in range(1, th + 1):
                for c in (-1, tw):
                    assert read_tile_cell(once, lay, t, 0, i, c) == a[ty * th + i, tx * tw + c + 1]
            for c in range(tw):
                for i in (0, th + 1):
                    assert read_tile_cell(once, lay, t, 0, i, c) == a[ty * th + i, tx * tw + c + 1]
        # idempotent on every cell that holds data (padding may hold anything, but is not rewritten)
        assert np.array_equal(once, twice, equal_nan=True)
        assert np.array_equal(r.fetch(), a)
    finally:
        r.close()


def test_scatter_gather_roundtrip_3d_f32(H):
    dims, tiles = (6, 10, 36), (3, 2, 2)
    a = random_padded(dims, dtype=np.float32, seed=5)
    r = H.JacobiRun(dims, tiles, np.float32)
    try:
        r.load(a)
        assert np.array_equal(r.fetch(), a)
    finally:
        r.close()


def test_residual_is_run_to_run_reproducible_and_device_variant_agrees(H, oracle_mod):
    import torch
    a = random_padded((512, 384), seed=21)
    r = H.JacobiRun((512, 384), (4, 3))
    try:
        r.load(a)
        r.sweep(3)
        v1 = r.residual()
        v2 = r.residual()
        out = torch.zeros(1, dtype=torch.float64, device="cuda")
        r.residual_async(out)
        torch.cuda.synchronize()
        assert v1 == v2 == float(out.item())
        u, _ = oracle_mod.run(a, 3)
        assert abs(v1 - oracle_mod.residual(u)) <= 1e-12 * v1
    finally:
        r.close()


def test_split_calls_equal_one_call(H, oracle_mod):
    """Every jacobi_sweep call must refresh stale halos itself."""
    a = random_padded((96, 96), seed=8)
    ref, _ = oracle_mod.run(a, 7)
    for fused in (0, 1):
        r = H.JacobiRun((96, 96), (3, 3), fused=fused)
        try:
            r.load(a)
            for n in (1, 2, 1, 3):
                r.sweep(n)
            assert np.array_equal(r.fetch(), ref)
        finally:
            r.close()


@pytest.mark.parametrize("dims,tiles,dtype", [
    ((150, 260), (3, 2), np.float64), ((512, 512), (4, 4), np.float64), ((20, 18, 40), (2, 3, 2), np.float64),
    ((64, 64, 64), (2, 2, 2), np.float64), ((96, 200), (3, 2), np.float32),
])
def test_sweep_residual_delivers_norm_of_input_grid(H, oracle_mod, dims, tiles, dtype):
    """The residual computed inside the first update equals residual_norm of the input grid,
    and the update itself is unchanged."""
    import torch
    a = random_padded(dims, dtype=dtype, seed=17)
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    r = H.JacobiRun(dims, tiles, dtype)
    try:
        r.load(a)
        r.sweep_residual(3, out[0:1])          # residual of u^0, then 3 iterations
        r.sweep_residual(2, out[1:2])          # residual of u^3, then 2 more
        got = r.fetch()
        res = out.cpu().tolist()
    finally:
        r.close()
    u3, _ = oracle_mod.run(a, 3)
    u5, _ = oracle_mod.run(a, 5)
    tol = RES_RTOL[np.dtype(dtype)]
    assert abs(res[0] - oracle_mod.residual(a)) <= tol * res[0]
    assert abs(res[1] - oracle_mod.residual(u3)) <= tol * res[1]
    if dtype == np.float64:
        assert np.array_equal(got, u5)
    else:
        assert np.max(np.abs(got.astype(np.float64) - u5)) <= 1e-5 * np.max(np.abs(u5))


T2_CASES = [
    # dims, tiles, iters, residual_every
    ((256, 256), (1, 1), 20, 5), ((96, 200), (3, 2), 13, 4), ((64, 1030), (2, 2), 9, 3),
    ((48, 48), (24, 24), 7, 7),           # 2x2 tiles: every value crosses tiles, diagonals included
    ((40, 36), (1, 18), 6, 2), ((36, 40), (18, 1), 6, 3), ((300, 70), (1, 1), 11, 11),
    ((512, 512), (4, 4), 50, 10), ((1024, 1024), (8, 8), 25, 5), ((2, 2), (1, 1), 5, 1),
    ((26, 300), (2, 1), 8, 8), ((130, 258), (5, 2), 10, 2),
]


@pytest.mark.parametrize("dims,tiles,iters,every", T2_CASES)
def test_temporal_blocking_is_bit_identical(H, oracle_mod, dims, tiles, iters, every):
    a = random_padded(dims, seed=sum(dims) + iters)
    check(*run_case(H, oracle_mod, a, tiles, iters, every, tblock=2))


def test_temporal_blocking_fp32_and_fused_residual(H, oracle_mod):
    import torch
    a = random_padded((96, 200), dtype=np.float32, seed=7)
    check(*run_case(H, oracle_mod, a, (3, 2), 13, 4, tblock=2))
    b = random_padded((192, 260), seed=9)
    out = torch.zeros(2, dtype=torch.float64, device="cuda")
    r = H.JacobiRun((192, 260), (3, 2), tblock=2)
    try:
        r.load(b)
        r.sweep_residual(4, out[0:1])
        r.sweep_residual(3, out[1:2])
        got = r.fetch()
        res = out.cpu().tolist()
    finally:
        r.close()
    u4, _ = oracle_mod.run(b, 4)
    u7, _ = oracle_mod.run(b, 7)
    assert abs(res[0] - oracle_mod.residual(b)) <= 1e-12 * res[0]
    assert abs(res[1] - oracle_mod.residual(u4)) <= 1e-12 * res[1]
    assert np.array_equal(got, u7)


def test_temporal_blocking_falls_back_on_thin_tiles_and_3d(H, oracle_mod):
    a = random_padded((40, 36), seed=5)
    check(*run_case(H, oracle_mod, a, (1, 36), 6, 2, tblock=2))      # tiles one column wide
    b = random_padded((12, 10, 41), seed=6)
    check(*run_case(H, oracle_mod, b, (2, 1, 1), 5, 5, tblock=2))    # 3-D, odd tile width: single steps
    c = random_padded((12, 5, 40), seed=8)
    check(*run_case(H, oracle_mod, c, (2, 5, 2), 5, 5, tblock=2, cooperative=0))    # 3-D, tiles one row high: single steps


CASES_3D_TB = [
    ((24, 20, 36), (2, 2, 3), 9, 3),        # tw = 12: a wavefront's columns span the whole tile row
    ((16, 16, 16), (1, 1, 1), 8, 4),
    ((6, 10, 130), (3, 5, 1), 6, 6),        # td = th = 2: every plane and row borders another tile
    ((8, 8, 8), (4, 4, 1), 7, 2),
    ((128, 128, 128), (4, 4, 4), 12, 4),    # 64 tiles of 32^3
    ((70, 33, 20), (1, 1, 1), 6, 3),        # th = 33: ragged last row group
    ((40, 18, 256), (2, 3, 1), 10, 5),      # tw = 256: three column segments, last one ragged
    ((20, 14, 448), (1, 1, 4), 8, 8),       # 4 tiles of 112 columns = one wavefront of owned columns each
    ((33, 9, 64), (1, 1, 32), 5, 5),        # tw = 2 (one fp64 vector)
    ((12, 60, 40), (3, 30, 1), 9, 4),       # th = 2: a workgroup's rows span a dozen tiles
    ((10, 57, 24), (2, 57, 2), 6, 3),       # th = 1
    ((9, 100, 16), (1, 4, 1), 8, 8),        # th = 25: row groups straddle tile boundaries at odd places
]


@pytest.mark.parametrize("opts", [dict(tblock=2), dict(tblock=3), dict(tblock=4), dict(tblock=8, rows_per_strip=3),
                                  dict(tblock=2, rows_per_strip=1), dict(tblock=3, rows_per_strip=5, xcd_chunk=1),
                                  dict(tblock=4, rows_per_strip=4096, nontemporal=0),
                                  # one wavefront per row group instead of a workgroup sharing its rows
                                  dict(tblock=2, cooperative=0), dict(tblock=8, rows_per_wave=2, cooperative=0),
                                  dict(tblock=2, rows_per_wave=4, cooperative=0),
                                  dict(tblock=2, rows_per_strip=1, cooperative=0),
                                  dict(tblock=3, rows_per_strip=5, xcd_chunk=1, cooperative=0),
                                  dict(tblock=2, rows_per_strip=4096, rows_per_wave=2, cooperative=0)])
@pytest.mark.parametrize("dims,tiles,iters,every", CASES_3D_TB)
def test_3d_temporal_blocking_is_bit_identical(H, oracle_mod, dims, tiles, iters, every, opts):
    a = random_padded(dims, seed=sum(dims) + iters)
    check(*run_case(H, oracle_mod, a, tiles, iters, every, **opts))


@pytest.mark.parametrize("tblock,rows_per_wave,cooperative", [(2, 2, 0), (2, 4, 0), (3, 0, 0), (2, 0, 1), (3, 0, 1), (4, 0, 1)])
def test_3d_temporal_blocking_fp32_and_fused_residual(H, oracle_mod, tblock, rows_per_wave, cooperative):
    a = random_padded((24, 20, 72), dtype=np.float32, seed=17)
    check(*run_case(H, oracle_mod, a, (2, 2, 3), 11, 4, tblock=tblock, rows_per_wave=rows_per_wave, cooperative=cooperative))
    b = random_padded((36, 22, 140), seed=19)
    ref, ref_res = oracle_mod.run(b, 13, 3)
    r = H.JacobiRun((36, 22, 140), (3, 2, 5), tblock=tblock, rows_per_wave=rows_per_wave, cooperative=cooperative)
    try:
        r.load(b)
        res = r.run(13, 3, fuse_residual=True)
        out = r.fetch()
    finally:
        r.close()
    check(out, res, ref, ref_res)


@pytest.mark.parametrize("tblock", [1, 2])
def test_fused_residual_schedule_equals_separate(H, oracle_mod, tblock):
    a = random_padded((260, 390), seed=31)
    ref, ref_res = oracle_mod.run(a, 23, 5)
    r = H.JacobiRun((260, 390), (2, 3), tblock=tblock)
    try:
        r.load(a)
        res = r.run(23, 5, fuse_residual=True)
        out = r.fetch()
    finally:
        r.close()
    check(out, res, ref, ref_res)


@pytest.mark.parametrize("opts", [dict(tblock=d) for d in (3, 4, 5, 6, 7, 8, 9, 10, 11, 12)] +
                         [dict(tblock=8, xcd_chunk=1), dict(tblock=4, nontemporal=0), dict(tblock=8, rows_per_strip=16),
                          dict(tblock=5, rows_per_strip=7), dict(tblock=8, rows_per_strip=4096)])
@pytest.mark.parametrize("dims,tiles,iters,every", T2_CASES + [
    ((64, 64), (8, 8), 19, 19),            # 8x8 tiles: ghost columns span exactly one neighbour tile
    ((48, 224), (3, 2), 17, 4),            # tw = 112: exactly one wavefront of owned columns
    ((40, 480), (2, 2), 16, 8),            # tw = 240: 3 column segments, last one ragged
    ((100, 128), (2, 1), 33, 11),          # th = 50: ragged last 16-row strip
    ((34, 64), (1, 4), 9, 9),              # tw = 16: a wavefront's lanes span all four tiles of a row
    ((24, 48), (3, 24), 10, 5),            # tw = 2 (one vector wide): 24 tiles under one wavefront
    ((64, 640), (2, 5), 12, 6),            # 5 tiles of 128: segments of 112 columns straddle tile boundaries
])
def test_deep_temporal_blocking_is_bit_identical(H, oracle_mod, dims, tiles, iters, every, opts):
    a = random_padded(dims, seed=sum(dims) + iters)
    check(*run_case(H, oracle_mod, a, tiles, iters, every, **opts))


@pytest.mark.parametrize("tblock", [3, 4, 5, 6, 7, 8, 9, 10, 11, 12])
def test_deep_temporal_blocking_fp32_and_fused_residual(H, oracle_mod, tblock):
    a = random_padded((96, 256), dtype=np.float32, seed=7)
    check(*run_case(H, oracle_mod, a, (3, 2), 21, 5, tblock=tblock))
    b = random_padded((192, 256), seed=9)
    ref, ref_res = oracle_mod.run(b, 23, 5)
    r = H.JacobiRun((192, 256), (3, 2), tblock=tblock)
    try:
        r.load(b)
        res = r.run(23, 5, fuse_residual=True)
        out = r.fetch()
    finally:
        r.close()
    check(out, res, ref, ref_res)


def test_sweep_can_be_captured_in_a_hip_graph(H, oracle_mod):
    """jacobi_sweep only enqueues kernels (no allocation, no memset, no synchronisation), so a
    caller may record it into a HIP graph and replay it; every replay must equal the eager result."""
    import torch
    w = gen.WORKLOADS["C1"]
    a2 = gen.generate(w)
    a3 = random_padded((24, 20, 36), seed=77)
    # n iterations per call; an even number of passes, so the result is back in the source buffer
    cases = [(a2, w.tiles, dict(), 10), (a2, w.tiles, dict(tblock=8), 10),
             (a3, (2, 2, 3), dict(), 8), (a3, (2, 2, 3), dict(tblock=4), 8),
             (a3, (2, 2, 3), dict(tblock=2, cooperative=0), 8)]
    for a, tiles, opts, n in cases:
        dims = [x - 2 for x in a.shape]
        r = H.JacobiRun(dims, tiles, **opts)
        try:
            r.load(a)
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                r.sweep(n)                        # eager, on the side stream (also warms up)
            torch.cuda.current_stream().wait_stream(s)
            torch.cuda.synchronize()
            assert np.array_equal(r.fetch(), oracle_mod.run(a, n)[0])
            # record n more iterations starting from the current buffer
            src, dst = r.cur, r.other()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                fin = H.B.jacobi_sweep(r.plan, src.data_ptr(), dst.data_ptr(), n,
                                       int(torch.cuda.current_stream().cuda_stream))
            assert fin == src.data_ptr()          # even count: result back in the source buffer
            for k in range(2):                    # two replays with eager work in between
                g.replay()
                torch.cuda.synchronize()
                got = r.fetch()
                torch.cuda.synchronize()
                exp, _ = oracle_mod.run(a, 2 * n + n * k)
                assert np.array_equal(got, exp), (opts, k)
        finally:
            r.close()


def test_residual_calls_can_be_captured_after_prepare(H, oracle_mod):
    """After jacobi_prepare nothing in jacobi_sweep_residual / residual_norm allocates or synchronises,
    whatever options change in between: both are recorded into a HIP graph on a FRESH plan (no eager
    call has run), replayed between eager calls that toggle `tblock` (other kernels, other numbers
    of partial sums in the same scratch), and every replay must give the eager bits."""
    import torch
    a = random_padded((192, 256), seed=99)
    n = 6
    for dims, tiles, a in (((192, 256), (3, 2), a), ((24, 20, 36), (2, 2, 3), random_padded((24, 20, 36), seed=98))):
        r = H.JacobiRun(dims, tiles)
        ref = H.JacobiRun(dims, tiles)
        try:
            H.B.jacobi_prepare(r.plan)
            assert H.B.jacobi_scratch_bytes(r.plan) >= 16
            g_dev = torch.from_numpy(a).cuda()
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            out = torch.zeros(2, dtype=torch.float64, device="cuda")
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=s):
                st = int(torch.cuda.current_stream().cuda_stream)
                H.B.jacobi_scatter(r.plan, g_dev.data_ptr(), r.a.data_ptr(), st)
                fin = H.B.jacobi_sweep_residual(r.plan, r.a.data_ptr(), r.b.data_ptr(), n, out[0:1].data_ptr(), st)
                H.B.residual_norm(r.plan, fin, out[1:2].data_ptr(), st)
            assert fin == r.a.data_ptr()
            # eager reference on a second plan
            ref.load(a)
            e0 = ref.residual()
            ref.sweep(n)
            e1 = ref.residual()
            want = ref.fetch()
            exp, exp_res = oracle_mod.run(a, n, n)
            assert np.array_equal(want, exp) and abs(e1 - exp_res[0]) <= 1e-12 * exp_res[0]
            for k, tb in enumerate((8, 1, 4)):
                out.zero_()
                graph.replay()
                torch.cuda.synchronize()
                r.cur = r.a
                got = r.fetch()
                vals = out.cpu().tolist()
                assert np.array_equal(got, want), (dims, k)
                assert abs(vals[0] - e0) <= 1e-12 * e0 and abs(vals[1] - e1) <= 1e-12 * e1, (dims, k, vals, e0, e1)
                # eager work on the same plan with another blocking depth between the replays: the fused
                # residual then comes from a blocked pass with a different number of workgroups
                r.set_option("tblock", tb)
                tmp = torch.zeros(1, dtype=torch.float64, device="cuda")
                r.sweep_residual(5, tmp)
                torch.cuda.synchronize()
                assert abs(tmp.item() - e1) <= 1e-12 * e1
                r.set_option("tblock", 1)
        finally:
            r.close()
            ref.close()


TASK_CASES = [
    # (interior dims, tiles, tiles per task, streams, iterations)
    ((96, 200), (3, 2), 1, 4, 7),            # one tile per task
    ((96, 200), (3, 2), 2, 3, 8),
    ((96, 200), (3, 2), 100, 1, 5),          # one task, one stream: the monolithic launch
    ((48, 48), (48, 48), 37, 16, 6),         # 2304 one-cell tiles in ragged groups of 37
    ((512, 512), (4, 4), 3, 5, 12),
    ((24, 20, 36), (2, 2, 3), 1, 16, 9),     # 3-D, every tile a task
    ((24, 20, 36), (2, 2, 3), 5, 2, 9),
    ((8, 8, 8), (8, 8, 8), 64, 7, 5),
    ((256, 256), (1, 1), 1, 4, 10),          # single tile
]


@pytest.mark.parametrize("dims,tiles,group,streams,iters", TASK_CASES)
def test_task_execution_is_bit_identical(H, oracle_mod, dims, tiles, group, streams, iters):
    """jacobi_sweep_tasks: per-tile-group tasks ordered only by events across several streams."""
    for dtype in (np.float64, np.float32):
        a = random_padded(dims, dtype=dtype, seed=sum(dims) + iters)
        r = H.JacobiRun(dims, tiles, dtype)
        try:
            r.load(a)
            r.sweep_tasks(iters, group, streams)
            r.sweep_tasks(3, group, streams)              # a second call continues from the result
            out = r.fetch()
            res = [r.residual()]
        finally:
            r.close()
        ref, ref_res = oracle_mod.run(a, iters + 3, iters + 3)
        check(out, res, ref, ref_res)


def test_whole_schedule_can_be_captured_in_a_hip_graph(H, oracle_mod):
    """jacobi_run - scatter, every block of iterations and every residual norm of a schedule - recorded into ONE
    HIP graph on a prepared plan and replayed with eager work on the same plan in between: every replay must
    give the grid and the norms of the eager run.  Launch-per-pass kernels (2-D and 3-D, single steps and
    blocked passes) and the path that runs a block of iterations in one launch."""
    import torch
    cases = [((192, 256), (3, 2), dict(resident=0), 12, 4), ((192, 256), (3, 2), dict(resident=0, tblock=4), 14, 7),
             ((24, 20, 36), (2, 2, 3), dict(), 9, 3), ((24, 20, 36), (2, 2, 3), dict(tblock=2), 8, 4),
             ((256, 256), (1, 1), dict(resident=1), 60, 20), ((40, 64), (2, 2), dict(resident=1), 30, 10)]
    for n, (dims, tiles, opts, iters, every) in enumerate(cases):
        a = random_padded(dims, seed=300 + n)
        exp, exp_res = oracle_mod.run(a, iters, every)
        r = H.JacobiRun(dims, tiles, **opts)
        try:
            H.B.jacobi_prepare(r.plan)
            g_dev = torch.from_numpy(a).cuda()
            res = torch.zeros(iters // every, dtype=torch.float64, device="cuda")
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=s):
                st = int(torch.cuda.current_stream().cuda_stream)
                H.B.jacobi_scatter(r.plan, g_dev.data_ptr(), r.a.data_ptr(), st)
                fin = H.B.jacobi_run(r.plan, r.a.data_ptr(), r.b.data_ptr(), iters, every, res.data_ptr(), st)
            for k in range(3):
                res.zero_()
                graph.replay()
                torch.cuda.synchronize()
                r.cur = r.a if fin == r.a.data_ptr() else r.b
                check(r.fetch(), res.cpu().tolist(), exp, exp_res)
                # eager work on the same plan between the replays: other kernels, the same scratch
                r.load(a)
                r.sweep(k + 1)
                r.residual()
        finally:
            r.close()


@pytest.mark.skip(reason="ending the capture of the multi-stream fork/join crashed inside the HIP runtime "
                         "(host segmentation fault in hipStreamEndCapture, cause not found); "
                         "jacobi_sweep_tasks now refuses a capturing stream")
def test_task_execution_can_be_captured_in_a_hip_graph(H, oracle_mod):
    """The fork / join over the plan's streams recorded into a graph: the graph would hold the task DAG."""
    import torch
    a = random_padded((128, 192), seed=41)
    r = H.JacobiRun((128, 192), (4, 3))
    try:
        r.load(a)
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            r.sweep_tasks(6, 2, 4)                        # eager: creates the streams and events
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        assert np.array_equal(r.fetch(), oracle_mod.run(a, 6)[0])
        src, dst = r.cur, r.other()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            fin = H.B.jacobi_sweep_tasks(r.plan, src.data_ptr(), dst.data_ptr(), 6, 2, 4,
                                         int(torch.cuda.current_stream().cuda_stream))
        assert fin == src.data_ptr()
        for k in range(3):
            g.replay()
            torch.cuda.synchronize()
            got = r.fetch()
            torch.cuda.synchronize()
            assert np.array_equal(got, oracle_mod.run(a, 12 + 6 * k)[0]), k
    finally:
        r.close()


def test_task_execution_rejects_bad_arguments(H):
    r = H.JacobiRun((32, 32), (2, 2))
    try:
        p, x, y = r.plan, r.cur.data_ptr(), r.other().data_ptr()
        for bad in (lambda: H.B.jacobi_sweep_tasks(p, x, y, 1, 0, 2), lambda: H.B.jacobi_sweep_tasks(p, x, y, 1, 1, 0),
                    lambda: H.B.jacobi_sweep_tasks(p, x, y, 1, 1, 17), lambda: H.B.jacobi_sweep_tasks(p, x, x, 1, 1, 2),
                    lambda: H.B.jacobi_sweep_tasks(p, x, y, -1, 1, 2)):
            with pytest.raises(H.B.JacobiError):
                bad()
        r.set_option("fused", 0)
        with pytest.raises(H.B.JacobiError):
            H.B.jacobi_sweep_tasks(p, x, y, 1, 1, 2)
    finally:
        r.close()


def _tasks_per_iteration(tiles, group):
    n = int(np.prod(tiles))
    return -(-n // min(group, n))


TASK_GRAPH_REMOVED = ("jacobi_sweep_task_graph (the task DAG built node by node as a HIP graph) was taken out: the HIP runtime "
                         "aborted on the host - on a 63-task-wide graph when its launch was waited for, and once in "
                         "hipGraph / plan destruction after a 3-task-wide one - cause not found (reading the removed code found no "
                         "misuse of the API); the entry point and the harness method sweep_task_graph these bodies call no "
                         "longer exist, the tests are kept as written for them")


@pytest.mark.skip(reason=TASK_GRAPH_REMOVED)
@pytest.mark.parametrize("dims,tiles,group,streams,iters",
                         [c for c in TASK_CASES if _tasks_per_iteration(c[1], c[2]) <= 16])
def test_task_graph_execution_is_bit_identical(H, oracle_mod, dims, tiles, group, streams, iters):
    """jacobi_sweep_task_graph: the same task DAG as an explicitly built HIP graph.  Three launches:
    the first builds the graph; the second either reuses it (even iteration count: same buffers) or
    rebuilds it (odd: buffers swapped); the third with another iteration count rebuilds."""
    a = random_padded(dims, seed=sum(dims) + iters)
    r = H.JacobiRun(dims, tiles)
    try:
        r.load(a)
        r.sweep_task_graph(iters, group)
        r.sweep_task_graph(iters, group)
        r.sweep_task_graph(3, group)
        out = r.fetch()
        res = [r.residual()]
    finally:
        r.close()
    ref, ref_res = oracle_mod.run(a, 2 * iters + 3, 2 * iters + 3)
    check(out, res, ref, ref_res)


@pytest.mark.skip(reason=TASK_GRAPH_REMOVED)
def test_task_graph_fp32_3d_and_option_change(H, oracle_mod):
    a = random_padded((24, 20, 72), dtype=np.float32, seed=23)
    r = H.JacobiRun((24, 20, 72), (2, 2, 3), np.float32)
    try:
        r.load(a)
        r.sweep_task_graph(4, 2)
        r.set_option("rows_per_strip", 3)             # same call, other strip geometry: the graph is rebuilt
        r.sweep_task_graph(4, 2)
        out = r.fetch()
        res = [r.residual()]
    finally:
        r.close()
    ref, ref_res = oracle_mod.run(a, 8, 8)
    check(out, res, ref, ref_res)
