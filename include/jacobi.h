/*
 * libjacobi - Jacobi relaxation on a block-decomposed Cartesian grid, on one
 * AMD MI355X (gfx950).  C ABI; no C++ or framework types cross this boundary.
 *
 * The computation is the data-parallel part of the Jacobi proxy application of
 * the paper (Sec. VI-C): the domain is cut into cuboid blocks ("tiles" here;
 * the paper wraps each in a mobile object and treats it as a task, Sec. II on
 * over-decomposition).  One iteration is
 *     1. halo exchange  - every tile's edge cells are packed, moved to the face
 *                         neighbours and unpacked into their halo cells;
 *     2. Jacobi update  - once a tile has all its halos, every interior point
 *                         becomes the mean of its 2d face neighbours;
 * repeated a fixed number of times.  A residual norm (not in the paper; added
 * so convergence can be observed) is available as a third operation.
 *
 * Arithmetic (the paper gives none; these choices are part of the contract):
 *     2-D:  new = 0.25 * ((W + E) + (S + N))
 *     3-D:  new = C6 * (((x- + x+) + (y- + y+)) + (z- + z+)),  C6 = fl(1/6)
 *     residual(u) = sqrt( sum_interior ( sum_nbrs u - 2d*u )^2 ), sum in fp64.
 * Device code is built with FP contraction off, so an fp64 grid is bit-identical
 * to a straightforward CPU loop using the same expression.
 *
 * Conventions
 *   - Row-major, last index (x) fastest.  dims/tiles arrays are ordered slowest
 *     to fastest: {Ny, Nx} or {Nz, Ny, Nx}.
 *   - "padded global array": (N+2) per dim; padded index 0 and N+1 hold the
 *     Dirichlet boundary ring, 1..N the interior.
 *   - "grid": the library's tile-major device buffer of jacobi_grid_bytes()
 *     bytes, at least 16-byte (better 256-byte) aligned, allocated and owned by the
 *     CALLER (device memory); a misaligned grid pointer is rejected with EINVAL.
 *     Its layout is described by jacobi_get_layout(); move data in and out with
 *     jacobi_scatter()/jacobi_gather().
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Unless stated, calls only enqueue work on `stream` and return at once.
 *   - Every function returns a jacobi_status (0 = OK) and never throws or exits.
 *     Arguments are validated before any device call, so argument errors are
 *     reported identically on a machine without a GPU.
 *   - A plan may be used by one host thread at a time; plans are independent.
 */
#ifndef JACOBI_H
#define JACOBI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct jacobi_plan jacobi_plan; /* opaque */

enum jacobi_dtype { JACOBI_F64 = 0, JACOBI_F32 = 1 };

enum jacobi_status {
    JACOBI_OK = 0,
    JACOBI_EINVAL = 1,  /* null or misaligned pointer, ndim not 2/3, dim <= 0, tiles <= 0, bad
                           dtype, in == out or overlapping, iters < 0, unknown option or value,
                           tile too large (2^31 elements or more, or a plane of a 3-D tile of
                           2 GiB or more) */
    JACOBI_ENOTDIV = 2, /* dims[d] % tiles[d] != 0 */
    JACOBI_ENOMEM = 3,  /* host or device allocation failed */
    JACOBI_EHIP = 4     /* a HIP call failed; text in jacobi_last_error() */
};

/*
 * Tile-major grid layout (all counts in ELEMENTS of the plan's dtype).
 * Tile t = (tz*Ty + ty)*Tx + tx starts at t*tile_stride.  Inside a tile:
 *   - cell (k, i, c), with k in [0, nplanes), i in [0, th+2), c in [0, tw), lives at
 *     (k*(th+2) + i)*pitch + c.  i = 0 and th+1 are the y halo rows; in 3-D k = 0 and
 *     td+1 are the z halo planes (2-D: nplanes = 1, k = 0).  Rows are padded to
 *     `pitch` (a multiple of 128 bytes) so every row starts on a cache-line boundary;
 *     columns [tw, pitch) are padding with unspecified contents.
 *   - the x halos are NOT stored beside the rows but in two dense arrays:
 *     x- halo of row (k, i) at xhalo_offset + k*(th+2) + i,
 *     x+ halo of row (k, i) at xhalo_offset + xhalo_pitch + k*(th+2) + i;
 *     each array is followed by at least 3 unused elements (xhalo_pitch is rounded up
 *     to a multiple of 128 bytes after adding them).
 *   - behind them two more dense arrays of the same shape, the x SEND arrays, at xsend_offset
 *     and xsend_offset + xhalo_pitch: scratch in which an update with option "fused" = 0
 *     packs the tile's own first and last column for the exchange kernel that follows it.
 *     Their contents are unspecified between calls; scatter and gather ignore them.
 * A halo cell holds either a copy of the neighbouring tile's edge cell (refreshed
 * by halo_exchange) or, on the domain boundary, the Dirichlet value.
 */
typedef struct jacobi_layout {
    int32_t ndim;          /* 2 or 3 */
    int32_t dtype;         /* jacobi_dtype */
    int64_t dims[3];       /* interior extents, slowest->fastest; dims[0] = 1 in 2-D */
    int64_t tiles[3];      /* tile counts Tz, Ty, Tx; Tz = 1 in 2-D */
    int64_t tile[3];       /* tile interior extents td, th, tw; td = 1 in 2-D */
    int64_t ntiles;
    int64_t nplanes;       /* td + 2 in 3-D, 1 in 2-D */
    int64_t pitch;         /* elements between consecutive rows */
    int64_t plane;         /* elements between consecutive planes = (th+2)*pitch */
    int64_t xhalo_offset;  /* start of the x- halo array inside a tile */
    int64_t xhalo_pitch;   /* distance from the x- to the x+ halo array */
    int64_t tile_stride;   /* elements between consecutive tiles */
    int64_t grid_bytes;    /* ntiles * tile_stride * sizeof(element) */
    int64_t xsend_offset;  /* start of the x send arrays inside a tile (xhalo_pitch apart) */
} jacobi_layout;

/*
 * jacobi_create: describe a block-decomposed domain (paper Sec. VI-C: the proxy's 3-D
 * domain is cut into cuboids; 2-D is the same with one dimension fewer).
 *   plan   out, host pointer; receives a new plan the caller frees with jacobi_destroy.
 *   ndim   2 or 3.
 *   dims   host array[ndim], interior points per dim, slowest->fastest, each > 0.
 *   tiles  host array[ndim], tile counts per dim, each > 0 and dividing dims[d].
 *   dtype  JACOBI_F64 or JACOBI_F32.
 * Touches no device (see jacobi_prepare).
 * Errors: EINVAL, ENOTDIV, ENOMEM.
 */
int jacobi_create(jacobi_plan **plan, int ndim, const int64_t *dims, const int64_t *tiles,
                  int dtype);

/*
 * jacobi_prepare: the plan's one-time device set-up, on the current device: reads the device's
 * CU count and LDS size and allocates the plan-owned scratch of the residual reduction (one
 * double per workgroup of the largest launch ANY option setting can ask for, so it never has
 * to grow: 8 bytes per 4 one-row strips of about 100 cells at most, 5 MiB for 16384^2; behind
 * it the 16 bytes of the one-launch kernel's barrier words, set to zero here once).
 * This is the only device allocation the library ever makes for a plan (the paper's runtime
 * keeps such buffers in a pre-allocated device memory pool for the same reason, Sec. VI-A).
 * jacobi_scatter, jacobi_sweep, jacobi_sweep_residual, jacobi_sweep_tasks, residual_norm and
 * residual_norm_host call it themselves if the caller has not; after it has run once, none of
 * jacobi_sweep, jacobi_sweep_residual, jacobi_run, halo_exchange and residual_norm allocates,
 * frees or synchronises anything, whatever options are changed in between, so they can be recorded
 * into a HIP graph (the call that runs the set-up cannot: do it before the capture starts).
 * Idempotent.  Errors: EINVAL (NULL), ENOMEM, EHIP.
 */
int jacobi_prepare(jacobi_plan *plan);

/* Bytes of device scratch jacobi_prepare allocates for this plan (host-only: no device call;
 * independent of the current option values); 0 if plan is NULL. */
size_t jacobi_scratch_bytes(const jacobi_plan *plan);

/* Frees the plan and the device scratch it owns (synchronises the device first if it owns any).
 * NULL is accepted. */
int jacobi_destroy(jacobi_plan *plan);

/* Bytes the caller must allocate (device memory) for one grid; 0 if plan is NULL. */
size_t jacobi_grid_bytes(const jacobi_plan *plan);

/* Copies the layout description into *layout (host memory).  EINVAL on NULL. */
int jacobi_get_layout(const jacobi_plan *plan, jacobi_layout *layout);

/*
 * jacobi_scatter / jacobi_gather: move a padded global array (DEVICE memory,
 * prod(dims[d]+2) elements, row-major) into / out of a tile-major grid.
 * scatter fills every cell of every tile, halos included (inter-tile halos get the
 * neighbour's value, boundary halos the Dirichlet ring).  gather writes the interior
 * of every tile and the boundary halos back to the global array (the whole padded
 * array is rewritten; inter-tile halo copies are ignored).  Asynchronous on `stream`.
 * Errors: EINVAL (null), EHIP.
 */
int jacobi_scatter(jacobi_plan *plan, const void *global_padded_dev, void *grid, void *stream);
int jacobi_gather(jacobi_plan *plan, const void *grid, void *global_padded_dev, void *stream);

/*
 * jacobi_sweep: `iters` Jacobi iterations (paper Sec. VI-C: per iteration, exchange
 * halos, unpack, and update a block only after all of its halos have arrived).
 *   in, out  two distinct device grids.  `in` holds the current field: tile interiors
 *            and Dirichlet boundary halos must be valid; inter-tile halos need not be
 *            (they are exchanged before the first update).  `out` may hold anything.
 *   iters    >= 0.  0 is a no-op (*final = in).
 *   final    nullable host pointer; receives the grid holding the result.  The two
 *            buffers ping-pong once per pass over memory: with the default of one
 *            iteration per pass the result is in `out` if iters is odd and in `in` if
 *            even; with option "tblock" > 1 it depends on the number of passes (see
 *            jacobi_pass_schedule), so read *final.
 * First copies the Dirichlet boundary halos in -> out so both buffers carry them, then
 * for each iteration: halo exchange on the source buffer, update into the other buffer.
 * (How the exchange is carried out depends on option "fused", below; the first update of a
 * call reads the neighbouring tiles' edge cells directly, which is why `in`'s inter-tile
 * halos need not be valid and are not refreshed.)
 * (Option "tblock" > 1 replaces this per-iteration sequence by multi-iteration passes, and small
 * 2-D grids run all iterations of the call inside one launch: option "resident".)
 * With option "fused" = 1 the update kernel itself writes each tile's fresh edge
 * cells into the neighbours' halos of the destination buffer (pack, transfer and
 * unpack fused into the update's epilogue), and only the first iteration needs a
 * separate exchange; results are identical.  With "fused" = 0 every iteration runs the
 * exchange kernel; the update then packs each tile's first and last column into dense
 * send arrays (the strided x faces: one cell per cache line otherwise), from which the
 * exchange of the next iteration copies.
 * After return, the inter-tile halos of the result are unspecified (stale or fresh
 * depending on the option); call halo_exchange if they are needed.
 * Asynchronous on `stream`; allocates no memory once the plan is prepared (jacobi_prepare; with
 * option "profile" = 1 the first call also creates its HIP events); does not synchronise.
 * Large-grid launches request LDS they never touch, to limit the workgroups per CU.
 * Errors: EINVAL (null, in == out or overlapping, misaligned, iters < 0), EHIP.
 */
int jacobi_sweep(jacobi_plan *plan, void *in, void *out, int iters, void *stream, void **final);

/*
 * jacobi_sweep_residual: jacobi_sweep that also delivers residual_norm(in) - the norm of the
 * field BEFORE the first of the `iters` iterations - to *residual_in_dev (a DEVICE double).
 * The terms sum_nbrs u - 2d*u of the source grid are exactly what the first update already
 * holds in registers, so the norm costs no extra pass over memory (a stand-alone
 * residual_norm reads the whole grid once more).  A caller that wants the residual after
 * every k-th iteration gets it from the NEXT call's first update.  Same value as
 * residual_norm(in) up to summation order; same fixed-order reduction; uses the plan's
 * device scratch (jacobi_prepare).
 * iters >= 1.  Errors: EINVAL, ENOMEM, EHIP.
 */
int jacobi_sweep_residual(jacobi_plan *plan, void *in, void *out, int iters, void *stream,
                          void **final, double *residual_in_dev);

/*
 * jacobi_run: a whole workload schedule in one call: `iters` iterations, and after every
 * `residual_every`-th of them the residual norm of the grid THAT iteration produced, written to
 * residuals_dev[k] for the (k+1)*residual_every-th iteration (a DEVICE array of
 * iters / residual_every doubles; may be NULL if that is 0; residual_every = 0: no norms).
 * Equivalent to blocks of jacobi_sweep(residual_every) each followed by residual_norm, but each norm
 * except the last is taken from inside the first update of the NEXT block (jacobi_sweep_residual), so
 * it costs no pass over memory of its own (on small 2-D grids, where a block is one launch - option
 * "resident" -, that launch delivers the norm of its own result); values agree up to summation order.
 * The blocks after the
 * first also start from what the block before left in the two grids (the Dirichlet ring in both, the
 * halo cells its last update pushed), where separate calls would copy the ring and fetch the
 * neighbours' edge cells again.  in / out / final as for jacobi_sweep (the buffers swap roles once per
 * pass of every block: read *final).
 * Asynchronous on `stream`; allocates and synchronises nothing once the plan is prepared.
 * Errors: EINVAL, ENOMEM, EHIP.
 */
int jacobi_run(jacobi_plan *plan, void *in, void *out, int iters, int residual_every,
               double *residuals_dev, void *stream, void **final);

/*
 * jacobi_pass_schedule: what jacobi_sweep(plan, ., ., iters) will launch with the current
 * options - the number of passes over memory and how many iterations each one advances
 * (1 = halo exchange + single-step update; > 1 = a blocked pass, option "tblock").
 * Host-only: no device call.  *npasses receives the number of passes; the first
 * min(*npasses, capacity) entries of depths[] are filled (depths may be NULL if capacity
 * is 0).  Errors: EINVAL.
 */
int jacobi_pass_schedule(const jacobi_plan *plan, int iters, int *depths, int capacity, int *npasses);

/*
 * jacobi_sweep_tasks: the same `iters` iterations as jacobi_sweep, executed as the paper
 * structures them (Sec. IV-A "Heterogeneous Tasks", Sec. IV-B "Execution Model", Sec. VI-A
 * "Enabling Concurrent GPU Operations"): every group of `tiles_per_task` consecutive tiles
 * is one task per iteration (update of its tiles, which also pushes their edge cells into
 * the neighbouring tiles' halo cells); a task's dependencies follow from what it reads and
 * writes - it waits for the tasks of the previous iteration that own its tiles and their
 * face neighbours - and the tasks are issued round-robin to `nstreams` streams owned by
 * the plan (default priority), ordered among each other by events only.  The work is
 * forked from and joined back into `stream`, so the call is asynchronous and in order
 * with other work on `stream`.  It must not be recorded into a HIP graph (EINVAL while
 * `stream` is capturing).  Results are bit-identical to jacobi_sweep.  Ignores "tblock".
 * Needs option "fused" = 1; tiles_per_task >= 1 (values above the tile count mean one
 * task); 1 <= nstreams <= 16.  Streams and events are created on first use (this call
 * allocates) and live until jacobi_destroy.  Errors: EINVAL, EHIP.
 */
int jacobi_sweep_tasks(jacobi_plan *plan, void *in, void *out, int iters, int tiles_per_task,
                       int nstreams, void *stream, void **final);

/*
 * jacobi_task_dependencies: the dependency graph jacobi_sweep_tasks executes (paper Sec. IV-A: a task's
 * dependencies follow from the data it reads and writes), for inspection or for a caller that wants to
 * schedule the tasks itself.  Task t of an iteration is the update of tiles [t*tiles_per_task,
 * (t+1)*tiles_per_task) (the last task may be shorter).  It reads its tiles' interiors and halo cells of the
 * grid the previous iteration wrote, so it depends on the tasks OF THE PREVIOUS ITERATION that own one of
 * its tiles or a face neighbour of one - itself included; the same edges order the reuse of the two
 * ping-pong grids.  The first min(*ndeps, capacity) entries of deps[] receive those task indices (no
 * particular order, no duplicates), *ndeps their number, *ntasks (nullable) the number of tasks per
 * iteration.  Host-only: no device call.  Errors: EINVAL (NULL, tiles_per_task < 1, task out of range).
 */
int jacobi_task_dependencies(jacobi_plan *plan, int tiles_per_task, int task, int *deps, int capacity,
                             int *ndeps, int *ntasks);

/*
 * halo_exchange: for every pair of face-adjacent tiles, copy each tile's edge cells
 * into the other's halo cells, in place in `grid` (paper Sec. VI-C: pack, transfer,
 * unpack - on one device the three collapse into one gather-scatter copy).
 * Idempotent; Dirichlet boundary halos are not touched; a single-tile plan launches
 * nothing.  Asynchronous on `stream`.  Errors: EINVAL, EHIP.
 */
int halo_exchange(jacobi_plan *plan, void *grid, void *stream);

/*
 * residual_norm: writes
 *     sqrt( sum over all interior points of (sum of face neighbours - 2d*u)^2 )
 * to *result_dev (a DEVICE double).  The inter-tile halo cells of `grid` need not be
 * current and are left alone: the pass reads the neighbouring tiles' edge cells itself
 * (the exchange is part of its loads); only the Dirichlet boundary halos are read as halos.  The sum is accumulated in fp64 in a fixed
 * two-stage order (per-wavefront shuffle tree -> LDS -> per-workgroup partial -> one
 * final workgroup), so it is bit-reproducible from run to run.  Uses the plan-owned
 * device scratch (jacobi_prepare); two calls on one plan that overlap in time (different
 * streams) would share it and race.  Asynchronous on `stream`.  Errors: EINVAL, ENOMEM, EHIP.
 */
int residual_norm(jacobi_plan *plan, void *grid, double *result_dev, void *stream);

/* Same, but delivers the value to HOST memory and synchronises `stream` first. */
int residual_norm_host(jacobi_plan *plan, void *grid, double *result_host, void *stream);

/*
 * residual_norm_noalloc: residual_norm for callers that cannot allocate device memory at all -
 * code under HIP graph capture that never ran jacobi_prepare, tight serving loops, harnesses
 * that forbid hipMalloc.  Same kernels, same summation order and therefore the same bits as
 * residual_norm, but the per-workgroup partial sums go to a fixed array inside the library's
 * own device image (JACOBI_NOALLOC_MAX_PARTIALS doubles = 1 MiB, resident on every GPU the
 * library runs on until the process ends) instead of the plan's scratch.  The call allocates
 * and frees nothing, on the device or through any allocating library routine, needs no
 * jacobi_prepare, and does not synchronise.  `grid` and `result_dev` are the caller's device
 * memory as for residual_norm.
 * Limits and hazards: the residual launch of the plan must have at most
 * JACOBI_NOALLOC_MAX_PARTIALS workgroups under the current options (16384^2 in 8 x 8 tiles:
 * 32768; 1024 x 1024 x 768 in 128^3 tiles: 24576), otherwise EINVAL with a message that names
 * both numbers and nothing is enqueued.  Every call on a GPU - of any plan - uses that GPU's
 * one array: calls that overlap in time on one GPU (different streams or host threads) race;
 * calls on one stream are safe.  Nothing in the array has to start at zero (every partial a
 * call reads it has written itself), so it is never cleared and keeps the last call's values.
 * Errors: EINVAL (NULL, misaligned, plan too large), EHIP.
 */
#define JACOBI_NOALLOC_MAX_PARTIALS 131072
int residual_norm_noalloc(jacobi_plan *plan, void *grid, double *result_dev, void *stream);

/*
 * Options (all int64).  Unknown key or out-of-range value -> EINVAL.
 *   "fused"          0 | 1   update kernel pushes edge cells to neighbour halos (default 1)
 *   "rows_per_strip" 0 | 1..4096  rows (2-D) or planes (3-D) one wavefront marches
 *                    through; 0 = choose from the shape: 8 rows / 16 planes for single steps
 *                    (fewer on small grids, so that there are about a thousand wavefronts),
 *                    up to 128 rows / the tile depth for blocked passes (default 0)
 *   "nontemporal"    0 | 1 | 2   how single-step updates store their results: 2 = streaming
 *                    (non-temporal) stores, 0 = plain stores, 1 = choose (default): plain when both
 *                    grids fit the Infinity Cache (grids of at most 124 MiB: the next iteration then
 *                    loads them from the cache), streaming beyond.  Streaming loads were measured
 *                    slower (border rows are re-read from cache) and are not offered.  Blocked passes
 *                    always stream.
 *   "unroll"         0 | 1 | 2 | 4 | 8  rows (planes) whose loads a wavefront issues back to
 *                    back before computing (3-D: planes per trip of the load pipeline); 0 = choose:
 *                    2-D the whole strip, up to 8; 3-D 1 on grids below 320 MiB and on fp64 grids of
 *                    1 GiB and more, else 2 (3-D accepts at most 4) (default 0)
 *   "rows_per_wave"  0 | 1 | 2 | 4  3-D: rows of a plane one wavefront keeps in registers
 *                    (0 = choose: 4 where the tile allows; 2 for updates of grids of at most 64 MiB -
 *                    1 on tiny ones - and for the residual pass below 1 GiB, which want more and
 *                    smaller wavefronts; default 0)
 *   "xcd_chunk"      0..2^20  G: within every 8*G consecutive workgroups, each of the 8 XCDs
 *                    takes G consecutive ones (1 = hardware order; 0 = choose: 8; 3-D updates 16,
 *                    or 1 on grids below 24 MiB; 32 for the 2-D update of cache-resident grids of
 *                    24 MiB and more; default 0)
 *   "tblock"         1..12   temporal blocking depth: jacobi_sweep advances up to this many
 *                    iterations per pass over memory (3-D: at most 4 in fp64, 3 in fp32).  The
 *                    iterations of a call are cut into equally deep passes: in 2-D as many as fit
 *                    at 8 or more iterations each (10 iterations at depth 12 run as one pass, at
 *                    depth 8 as 5 + 5; 50 as 9 + 9 + 8 + 8 + 8 + 8) - at 10 or more each on grids of
 *                    1 GiB and more (50 as 5 x 10) -, in 3-D the fewest the depth allows (10 as
 *                    4 + 3 + 3); see jacobi_pass_schedule.
 *                    2-D passes of depth 3..12 need a tile width that is a multiple of 16 bytes
 *                    and a tile height >= depth, depth 2 needs tiles >= 2 x 2; 3-D passes need
 *                    a tile width that is a multiple of 16 bytes and a tile depth >= the pass
 *                    depth; and in every case a row of tiles (tiles along x times the tile size,
 *                    jacobi_layout.tiles[2] * tile_stride elements) smaller than 2 GiB, because the
 *                    lanes of these passes address it with 32-bit byte offsets; otherwise passes of
 *                    depth 2 (2-D, 64-bit addressing) or single steps are used (jacobi_pass_schedule
 *                    shows which).  Blocked passes read the cells they
 *                    need beyond a tile straight from the neighbouring tiles, so the exchange is
 *                    part of their loads and they leave the halo cells alone.  Results are
 *                    bit-identical for every depth
 *                    (default 1: one halo exchange and one update per iteration)
 *   "cooperative"    0 | 1   3-D blocked passes: 1 = the wavefronts of a workgroup share one range
 *                    of rows and hand each other their border rows through LDS (depths 3 and 4,
 *                    and depth 2 where the other kernel cannot run); 0 = every wavefront carries
 *                    its own ghost rows (depths 2 and 3, needs a tile height >= depth) (default 1)
 *   "resident"       0 | 1   small 2-D grids: run ALL iterations of a jacobi_sweep call inside ONE kernel
 *                    launch (default 1).  Taken when the grid is 2-D, a row of the domain is at most
 *                    2 KiB (256 fp64 / 512 fp32 columns), the tile width is a multiple of 16 bytes, and
 *                    the rows fit one workgroup per CU (a workgroup owns what its 48 or 64 rows leave
 *                    after the ghost rows - 8 of 48 with 20 per side; taller grids get shallower phases,
 *                    up to ~12000 rows).
 *                    Such grids are updated in about a microsecond, so the launch-per-iteration sequence
 *                    is bound by launch latency (3.5 us per iteration); here the grid stays in registers,
 *                    the wavefronts of a workgroup pass each other their border rows through LDS, and
 *                    the workgroups meet at a barrier in device memory only every "resident_depth"
 *                    iterations (each holds that many ghost rows per side, which it recomputes), storing
 *                    their own rows to the other grid and re-reading only the ghost rows.  These phases
 *                    swap the two grids like passes do (jacobi_pass_schedule lists them; read *final).
 *                    The barrier's wait is bounded: if the workgroups cannot all be resident (the device
 *                    is busy with other work for seconds) the launch still ends and writes NaN.
 *                    The launch is the whole call: it carries the Dirichlet ring over itself, and in
 *                    jacobi_run it also delivers the residual norm of the grid it produced (NaN if the
 *                    barrier gave up).  Two launches of one plan must not overlap in time: they share
 *                    the barrier words in the plan's scratch.
 *                    Ignores "tblock"; inter-tile halo cells of the result are left alone.
 *   "resident_depth" 0 | 1..31  iterations between two barriers of that kernel (0 = choose: 20, evened
 *                    out over the call)
 *   "resident_rows"  0 | 1..4   rows each of its wavefronts keeps (0 = choose: as many as fit the
 *                    registers - 4, or 3 where a lane holds two vectors of a row -, or just enough for a
 *                    grid that fits one workgroup)
 *   "resident_spin_limit"  0 | n  polls a workgroup waits at that barrier before giving up: n - 1
 *                    beyond the first (0 = default, about 4 million: seconds)
 *   "stack"          0 | 1 | 4 | 8  2-D stand-alone residual pass: wavefronts of a workgroup stacked over
 *                    the same columns, 8 rows each, passing each other their border rows through LDS
 *                    instead of loading them again (0 = choose: 8 on tiles of 1024 rows and more, else
 *                    4; 1 = off: every wavefront loads its own border rows; default 0).  Only with
 *                    "rows_per_strip" = 0 and "unroll" = 0, and tiles at least one band high.
 *   "cu_lds"         0..2^20  LDS bytes of a CU that the workgroup limits of large-grid launches are
 *                    computed from (0 = the device's figure, read by jacobi_prepare; default 0; below
 *                    65536: no limits are requested).  Those
 *                    launches request (cu_lds / n - 4096) bytes of LDS they never touch so that at most
 *                    n workgroups share a CU (n = 1: 3-D update of fp64 grids of 1 GiB and more; n = 2:
 *                    2-D blocked passes on such grids).  Before a kernel variant uses the request for the
 *                    first time the library asks the runtime's occupancy calculator whether it has that
 *                    effect; if not, the launch runs without a limit (results are the same, it is only
 *                    a few per cent slower) and the read-only figure "lds_limit_failed" becomes 1.
 *   "profile"        0 | 1   record a HIP event pair around every update-kernel launch
 *                    made by jacobi_sweep (read with jacobi_profile_read)
 * None of the options changes any result bit.
 * jacobi_get_option also reads these figures (not settable): "lds_limit_failed" (see "cu_lds"),
 * "lds_request_1" / "lds_request_2" (the LDS bytes requested to keep 1 / 2 workgroups per CU; 0 while
 * the LDS size is unknown), "num_cu" (compute units; 256 until jacobi_prepare has asked the device),
 * and what a single-step launch will run with under the current options (host-only, the choices the
 * 0 = "choose" settings resolve to): "update_rows_per_strip", "update_rows_per_wave", "update_unroll",
 * "update_xcd_chunk", "update_strips" (wavefronts of work), "update_one_workgroup_per_cu",
 * "update_streaming_stores", and the same with "residual_" for the stand-alone residual pass.
 */
int jacobi_set_option(jacobi_plan *plan, const char *key, int64_t value);
int jacobi_get_option(const jacobi_plan *plan, const char *key, int64_t *value);

/*
 * With option "profile" = 1: waits for the recorded events, returns the summed
 * duration (milliseconds) and number of update-kernel launches since the last read
 * (with "tblock" > 1 a launch may cover several iterations),
 * and resets the record.  At most 8192 launches are recorded between reads; later
 * ones are not timed (and not counted).  Errors: EINVAL, EHIP.
 */
int jacobi_profile_read(jacobi_plan *plan, double *update_ms_total, int64_t *update_launches);

/*
 * Measurement aid, not part of the method: a plain streaming device-to-device copy kernel
 * (16 bytes per lane).  Its throughput is the practical ceiling the update kernel is
 * compared with, and its known size calibrates hardware HBM byte counters.
 * dst/src: device pointers, 16-byte aligned, not overlapping; bytes: multiple of 16.
 * Asynchronous on `stream`.  Errors: EINVAL, EHIP.
 */
int jacobi_stream_copy(void *dst, const void *src, size_t bytes, void *stream);

/* Text of the calling thread's most recent error ("" if none).  Valid until the next
 * failing call on this thread. */
const char *jacobi_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* JACOBI_H */
