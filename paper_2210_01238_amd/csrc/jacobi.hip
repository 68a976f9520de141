// C-ABI host side of libjacobi: plan/layout bookkeeping, argument validation and kernel
// launches for the block-decomposed Jacobi iteration (paper Sec. VI-C).  Declarations and
// the contract of every entry point are in include/jacobi.h.
#include "jacobi.h"
#include "aux_kernels.h"
#include "launchers.h"

#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <algorithm>
#include <vector>

using jk::Geo;
using jk::StripParams;

namespace {

thread_local std::string g_err;

int fail(int code, const char *msg)
{
    g_err = msg;
    return code;
}
int fail_hip(hipError_t e, const char *what)
{
    g_err = std::string(what) + ": " + hipGetErrorString(e);
    return JACOBI_EHIP;
}
#define HIP_TRY(expr)                                        \
    do {                                                     \
        hipError_t e_ = (expr);                              \
        if (e_ != hipSuccess) return fail_hip(e_, #expr);    \
    } while (0)

constexpr int MAX_TASK_STREAMS = 16;
constexpr int MAX_PROFILE_EVENTS = 8192;
constexpr int MAX_COPY_BLOCKS = 1 << 20;
constexpr int64_t LARGE_GRID_BYTES = 1LL << 30;   // grids from this size on get the workgroup-per-CU limits
// Two grids of at most this size each fit the 256 MiB Infinity Cache with room to spare (a plain copy of 135 MB
// to another 135 MB still runs at 7.7 TB/s, of 160 MB at 6.1).  Measured on the update: plain stores win clearly up
// to 240^3 (120 MiB: 54.0 -> 47.0 us) and 3584^2 (99 MiB: 37.2 -> 33.6); at 4096^2 (2 x 128.8 MiB, just over the
// cache) the outcome depends on where the two buffers happen to lie (42 - 48 us against 47.4 with streaming
// stores), at 4224^2 (137 MiB) they are level, and from 256^3 (136 MiB: 53.7 -> 58.5) and 4352^2 on they lose.
constexpr int64_t CACHED_GRID_BYTES = 124LL << 20;
constexpr int64_t CACHED_CHUNK_BYTES = 24LL << 20;  // cache-resident 2-D grids from this size on: XCD chunks of 32

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace

struct jacobi_plan {
    jacobi_layout lay;
    Geo geo;
    size_t esize;
    // options
    int64_t fused = 1, rows_per_strip = 0, nontemporal = 1, profile = 0, unroll = 0, xcd_chunk = 0, rows_per_wave = 0, tblock = 1, cooperative = 1;
    int64_t resident = 1, resident_depth = 0, resident_rows = 0, resident_spin_limit = 0;
    int64_t stack = 0;                // 2-D residual pass: wavefronts per workgroup stacked over one column segment (0: choose, 1: off, 4, 8)
    int64_t cu_lds_option = 0;        // option "cu_lds": LDS bytes per CU to compute the workgroup limits from (0: the device's)
    int64_t lds_limit_failed = 0;     // read-only: a launch dropped its workgroup limit (the occupancy query did not confirm it)
    // device state, set up once by prepare_plan() (jacobi_prepare, or the first call that touches the device)
    bool prepared = false;
    int64_t cu_lds = 0;       // LDS bytes of a CU of the device (0: unknown, no workgroup limits)
    int num_cu = jk::NUM_CU;  // compute units of the device
    // residual scratch (device): one partial sum per workgroup of the largest launch any option setting can
    // ask for, plus one slot for the value residual_norm_host copies back.  Never reallocated.
    double *partial = nullptr;
    int64_t partial_cap = 0;
    unsigned *sync_words = nullptr;   // behind the partial sums: arrival counter and failure flag of the resident kernel
    // profiling events around update launches
    std::vector<hipEvent_t> ev;   // pairs: 2*i start, 2*i+1 stop
    int64_t ev_used = 0;
    // task-based execution (jacobi_sweep_tasks): stream pool, events, and the dependency lists
    std::vector<hipStream_t> task_streams;
    std::vector<hipEvent_t> task_events;            // 2 per task (iteration parity), then fork, then 1 per stream
    int task_group = 0;                             // tiles per task the lists below were built for
    std::vector<std::vector<int>> task_deps;        // tasks whose previous-iteration output a task reads
};

namespace {

// How the update / residual kernels cut the tiles into strips (see jacobi_kernels.h), and
// which compiled variant runs them.
struct SweepConfig {
    StripParams sp;
    int rows_per_wave;   // 3-D only: rows one wavefront keeps in registers (1, 2 or 4)
    int unroll;          // rows (2-D) / planes (3-D) whose loads are issued back to back
    int lane_elems;      // elements per lane: 16 bytes' worth, or 2 for narrow fp32 rows in 3-D
    bool whole_cu;       // 3-D update of a large grid: one workgroup per CU
};

// Store flavour of the single-step updates (bit 2 of the kernels' NT argument: streaming stores): the option, or,
// left to the library (1), streaming unless both grids fit the Infinity Cache - there a plain store keeps the
// result on-chip for the next iteration's loads (2048^2: 15.5 -> 11.3 us per iteration, 3072^2: 28.5 -> 24.9,
// 224^3: 45.6 -> 39.4), while on grids beyond it plain stores lose (6144^2: 102 -> 110 us) because the written
// lines push out what is still to be read.
int store_flavour(const jacobi_plan *p)
{
    if (p->nontemporal != 1) return (int)p->nontemporal;
    return p->lay.grid_bytes <= CACHED_GRID_BYTES ? 0 : 2;
}

// Consecutive workgroups one XCD takes (jk::xcd_logical_wg): the option, or 8 - 16 for launches that run one
// workgroup per CU (measured: 512^3 0.401 -> 0.396 ms, 1024 x 1024 x 768 2.40 -> 2.36; 24 and more: as 8).
int xcd_chunk_of(const jacobi_plan *p, bool one_workgroup_per_cu = false)
{
    return p->xcd_chunk > 0 ? (int)p->xcd_chunk : one_workgroup_per_cu ? 16 : 8;
}

// Dynamic LDS to request with a launch so that at most `per_cu` workgroups share a CU.  Nobody touches
// those bytes: the hardware offers no other way to cap the workgroups per CU at launch time (the compiler's
// waves-per-SIMD hints only steer its register allocation).  0 if the device's LDS size is unknown.
unsigned lds_to_limit_workgroups(const jacobi_plan *p, int per_cu)
{
    const int64_t cu_lds = p->cu_lds_option > 0 ? p->cu_lds_option : p->cu_lds;
    if (cu_lds < 65536) return 0;
    // Measured with 256-thread workgroups that only wait: requests up to 20000 bytes let 8 share a CU, 26000: 6,
    // 30000-32000: 5, 36000-40000: 4, 44000-53589: 3, 54000-81000: 2, 100000 and more: 1 - slightly less than
    // 160 KiB is there to hand out.  4 KiB below an n-th of the nominal size lies well inside the range for n.
    // The launch checks the effect with the runtime's occupancy query before it uses the figure (lds_for_launch).
    return (unsigned)(cu_lds / per_cu - 4096);
}

SweepConfig make_config(const jacobi_plan *p, int mode)
{
    const Geo &g = p->geo;
    const int nv = 16 / (int)p->esize;
    const bool d3 = g.ndim == 3;
    SweepConfig c;
    StripParams &sp = c.sp;
    c.rows_per_wave = 1;
    // 3-D updates of grids that are not large (below 1 GiB the march is not limited to one workgroup per CU): what
    // the sizes from 32^3 to 384^3 measured best with - see the notes at the choices below
    const bool d3_small_update = d3 && mode != jk::MODE_RESIDUAL && p->lay.grid_bytes < LARGE_GRID_BYTES;
    const bool d3_small_residual = d3 && mode == jk::MODE_RESIDUAL && p->lay.grid_bytes < LARGE_GRID_BYTES;
    const bool narrow_f32 = d3 && p->esize == 4 && g.pitch <= 2 * jk::WAVE;
    if (d3) {
        int rw = (int)p->rows_per_wave;
        if (rw <= 0) {
            rw = g.th >= 4 ? 4 : g.th >= 2 ? 2 : 1;
            // grids that live in the caches want more, smaller wavefronts: 2 rows each (128^3 11.8 -> 8.5 us per
            // iteration, 160^3 18.3 -> 15.8, 192^3 28.0 -> 24.0; from 256^3 on 4 rows are better again).  fp32 rows of
            // 128 cells keep 4: only that variant has the 8-byte lanes they need.
            if (rw == 4 && d3_small_update && !narrow_f32 && p->lay.grid_bytes <= (64LL << 20)) rw = 2;
            // the read-only pass likes them up to 1 GiB (192^3 24.2 -> 18.6 us, 256^3 30.3 -> 26.3)
            if (rw == 4 && d3_small_residual && !narrow_f32) rw = 2;
        }
        c.rows_per_wave = rw;
    }
    // fp32 rows of at most 128 elements would leave half of a wavefront's 16-byte lanes idle: 8-byte lanes
    c.lane_elems = (narrow_f32 && c.rows_per_wave == 4) ? 2 : nv;
    sp.nseg = (int)ceil_div(g.pitch, (int64_t)jk::WAVE * c.lane_elems);
    const int extent = d3 ? g.td : g.th;       // marching direction
    int64_t lanes_of_work =
        (int64_t)g.ntiles * sp.nseg * (d3 ? ceil_div(g.th, c.rows_per_wave) : 1);
    int R = (int)p->rows_per_strip;
    if (R <= 0 && d3_small_update) {
        // 16 planes per strip, fewer until there are about a thousand wavefronts (64^3: 7.4 -> 4.5 us per iteration
        // with 1024 strips of 2 planes x 2 rows; 128^3 in 64^3 tiles 18.9 -> 10.1); tiny grids go down to one row
        // per wavefront as well (32^3: 6.3 -> 4.0)
        R = 16;
        while (R > 2 && (int64_t)ceil_div(extent, R) * lanes_of_work < 1024) R /= 2;
        if (p->rows_per_wave <= 0 && c.rows_per_wave > 1 && !narrow_f32 &&
            (int64_t)ceil_div(extent, R) * lanes_of_work < 512) {
            c.rows_per_wave = 1;
            lanes_of_work = (int64_t)g.ntiles * sp.nseg * g.th;
        }
    } else if (R <= 0) {
        // Short strips whose loads are all issued at once stream best (the chip then walks
        // through memory as one narrow front); 8 rows keeps the border re-read at 2 rows in 10.
        // Small problems get shorter strips so that there are enough wavefronts to fill the chip.
        // The read-only residual pass has no writes to keep apart from its reads and prefers
        // taller strips (fewer border re-reads): 16 rows, all in flight.
        R = d3 ? 16 : mode == jk::MODE_RESIDUAL ? 16 : 8;
        // mid-sized 2-D grids: at 8 rows a 4096^2 grid gives each CU only ~3 rounds of workgroups
        // and the last round runs half empty; 4-row strips measure 8 % faster there
        if (!d3 && mode != jk::MODE_RESIDUAL && (int64_t)ceil_div(extent, R) * lanes_of_work < 24576) R = 4;
        // (3-D: 16-plane strips until fewer than 512 strips would be left)
        while (R > 1 && (int64_t)ceil_div(extent, R) * lanes_of_work < (d3 ? 512 : 4096)) R /= 2;
    }
    if (R > extent) R = extent;
    sp.R = R;
    sp.nblk = (int)ceil_div(extent, R);
    sp.nstrips = lanes_of_work * sp.nblk;
    // option fused = 0: the exchange is a kernel of its own, and the updates pack their x edge cells for it
    sp.fused = p->fused ? jk::FUSED_PUSH : jk::FUSED_PACK;
    int u = (int)p->unroll;
    // one workgroup per CU for the 3-D update of a large grid (see launch_sweep)
    // (fp64 rows that fill a wavefront's 64 x 16 bytes only: fp32, and tiles narrower than 128 cells, lose with it)
    c.whole_cu = d3 && mode != jk::MODE_RESIDUAL && p->esize == 8 && g.pitch >= jk::WAVE * nv &&
                 p->lay.grid_bytes >= LARGE_GRID_BYTES;
    sp.xcd_chunk = xcd_chunk_of(p, c.whole_cu);
    // 3-D updates below 1 GiB: the hardware's own order on small grids (64^3 5.1 -> 4.5 us), runs of 16 from 24 MiB on
    if (d3_small_update && p->xcd_chunk <= 0) sp.xcd_chunk = p->lay.grid_bytes < CACHED_CHUNK_BYTES ? 1 : 16;
    // 2-D updates of cache-resident grids: longer runs per XCD (2048^2: 11.8 -> 11.3 us, 3072^2: 24.6 -> 23.2;
    // below 2048^2 the hardware's own order is as good or better)
    if (!d3 && mode != jk::MODE_RESIDUAL && p->xcd_chunk <= 0 && store_flavour(p) == 0 &&
        p->lay.grid_bytes >= CACHED_CHUNK_BYTES)
        sp.xcd_chunk = 32;
    if (d3) {
        // planes per trip of the pipeline: 1 with one workgroup per CU, and on grids up to ~300 MiB (160^3 15.7 ->
        // 14.5 us, 320^3 109.6 -> 105.9; 384^3, 460 MiB: 179.3 with 1, 174.6 with 2)
        if (u <= 0) u = c.whole_cu || d3_small_residual || (d3_small_update && p->lay.grid_bytes < (320LL << 20)) ? 1 : 2;
        if (u > 4) u = 4;                       // 3-D variants are compiled for 1, 2, 4
    } else if (u <= 0) {
        u = R >= 16 ? 16 : R >= 8 ? 8 : R >= 4 ? 4 : R >= 2 ? 2 : 1;   // all of a short strip at once
    }
    c.unroll = u;
    return c;
}

// The 2-D stand-alone residual pass with stacked wavefronts (residual2d_stack_kernel): wavefronts per workgroup
// and rows per wavefront, or waves = 0 if the plan and options take the one-strip-per-wavefront kernel:
// explicit strip options, tiles lower than one band, or a problem so small that it gets shorter strips.
struct StackChoice { int waves = 0, rows = 0; };
StackChoice stack_choice(const jacobi_plan *p, int mode)
{
    const Geo &g = p->geo;
    StackChoice c;
    if (mode != jk::MODE_RESIDUAL || g.ndim != 2 || p->stack == 1 || p->rows_per_strip != 0 || p->unroll != 0) return c;
    // 8 rows per wavefront; 8 wavefronts on tall tiles, 4 otherwise (16384^2 in 2048^2 tiles: 343 us with 8, 356 with 4,
    // 370 unstacked; 8192^2 in 128^2 tiles: 97 / 94 / 106; 4096^2: 26.9 / 26.6 / 30.2)
    const int rows = 8;
    const int waves = p->stack ? (int)p->stack : g.th >= 1024 ? 8 : 4;
    if (g.th < waves * rows) return c;
    if (p->stack == 0 && make_config(p, mode).sp.R != 16) return c;     // small problem: shorter strips, more workgroups
    c.waves = waves; c.rows = rows;
    return c;
}

StripParams stack_strips(const jacobi_plan *p, StackChoice c)
{
    const Geo &g = p->geo;
    StripParams sp;
    sp.R = c.rows;
    sp.nseg = (int)ceil_div(g.pitch, (int64_t)jk::WAVE * (16 / (int)p->esize));
    sp.nblk = (int)ceil_div(g.th, c.waves * c.rows);                          // bands per tile
    sp.nstrips = (int64_t)g.ntiles * sp.nseg * sp.nblk * jk::WAVES_PER_WG;   // partial sums: one per unit
    sp.fused = jk::FUSED_NONE;
    sp.xcd_chunk = p->xcd_chunk > 0 ? (int)p->xcd_chunk : 32;
    sp.pull = 1;
    return sp;
}

// Workgroups (= partial sums in the residual modes) of the single-step launch launch_sweep makes for `mode`.
int64_t single_step_workgroups(const jacobi_plan *p, int mode)
{
    if (const StackChoice sc = stack_choice(p, mode); sc.waves) return stack_strips(p, sc).nstrips / jk::WAVES_PER_WG;
    return ceil_div(make_config(p, mode).sp.nstrips, jk::WAVES_PER_WG);
}

int launch_checked(hipError_t e, const char *what)
{
    if (e == hipErrorInvalidValue) return fail(JACOBI_EINVAL, "kernel variant not compiled for these options");
    if (e != hipSuccess) return fail_hip(e, what);
    return JACOBI_OK;
}

// Single-step pass over `src` in the given mode (jk::Mode); with tile_count > 0 only over the tiles
// [tile0, tile0 + tile_count).
int launch_sweep(jacobi_plan *p, int mode, const void *src, void *dst, double *partial, hipStream_t st,
                 int tile0 = 0, int tile_count = 0, bool pull = false)
{
    if (tile_count == 0) {
        if (const StackChoice sc = stack_choice(p, mode); sc.waves) {
            const StripParams sp = stack_strips(p, sc);
            const int64_t nwg = sp.nstrips / jk::WAVES_PER_WG;
            if (nwg <= 0 || nwg > 0x7fffffffLL) return fail(JACOBI_EINVAL, "too many workgroups for one launch");
            const jk::LaunchArgs a{(unsigned)nwg, st, p->geo, sp, src, dst, partial};
            return launch_checked(p->lay.dtype == JACOBI_F64 ? jk::launch_stack_f64(sc.rows, sc.waves, a)
                                                             : jk::launch_stack_f32(sc.rows, sc.waves, a),
                                  "stacked residual kernel launch");
        }
    }
    SweepConfig c = make_config(p, mode);
    c.sp.pull = pull ? 1 : 0;
    if (tile_count > 0) {
        c.sp.nstrips = c.sp.nstrips / p->geo.ntiles * tile_count;   // strips are laid out tile by tile
        c.sp.tile0 = tile0;
    }
    const int64_t nwg = ceil_div(c.sp.nstrips, jk::WAVES_PER_WG);
    if (nwg <= 0 || nwg > 0x7fffffffLL) return fail(JACOBI_EINVAL, "too many workgroups for one launch");
    jk::LaunchArgs a{(unsigned)nwg, st, p->geo, c.sp, src, dst, partial};
    a.aux = c.lane_elems != 16 / (int)p->esize;       // 3-D fp32: the 8-byte-lane variant
    // The 3-D march over a grid much larger than the caches runs fastest with ONE workgroup on a CU (0.418 ->
    // 0.402 ms on 512^3: fewer wavefronts marching through memory at once suit the memory system better, and
    // the pipeline keeps each one's loads in flight), so the update asks for all of the CU's LDS, which it never
    // touches.  Small grids, and the read-only residual pass, measured faster without the limit.
    a.lds = c.whole_cu ? lds_to_limit_workgroups(p, 1) : 0;
    a.per_cu = 1;
    a.limit_failed = &p->lds_limit_failed;
    const bool f64 = p->lay.dtype == JACOBI_F64;
    const int nt = store_flavour(p);
    hipError_t e;
    if (p->geo.ndim == 2)
        e = f64 ? jk::launch_sweep2d_f64(mode, c.unroll, nt, a) : jk::launch_sweep2d_f32(mode, c.unroll, nt, a);
    else
        e = f64 ? jk::launch_sweep3d_f64(mode, c.rows_per_wave, c.unroll, nt, a)
                : jk::launch_sweep3d_f32(mode, c.rows_per_wave, c.unroll, nt, a);
    return launch_checked(e, "update kernel launch");
}

// pull: src's inter-tile halo cells are not current; read the neighbouring tiles' edge cells instead
int launch_update(jacobi_plan *p, const void *src, void *dst, hipStream_t st, bool pull)
{
    return launch_sweep(p, jk::MODE_UPDATE, src, dst, nullptr, st, 0, 0, pull);
}

// Update src -> dst and, in the same pass, per-workgroup partial sums of the squared residual
// terms of src.
int launch_update_with_residual(jacobi_plan *p, const void *src, void *dst, hipStream_t st, bool pull)
{
    return launch_sweep(p, jk::MODE_BOTH, src, dst, p->partial, st, 0, 0, pull);
}

// Two time steps per pass (2-D only; needs tiles of at least 2 x 2 cells).
bool t2_usable(const jacobi_plan *p)
{
    return p->geo.ndim == 2 && p->geo.th >= 2 && p->geo.tw >= 2;
}

StripParams t2_strips(const jacobi_plan *p)
{
    const Geo &g = p->geo;
    StripParams sp;
    sp.R = jk::T2_ROWS;
    sp.nseg = (int)ceil_div(g.pitch, (int64_t)jk::WAVE * (16 / (int)p->esize));
    sp.nblk = (int)ceil_div(g.th, sp.R);
    sp.nstrips = (int64_t)g.ntiles * sp.nseg * sp.nblk;
    sp.fused = 0;
    sp.xcd_chunk = xcd_chunk_of(p);
    return sp;
}

int launch_t2(jacobi_plan *p, const void *src, void *dst, bool with_residual, hipStream_t st)
{
    const StripParams sp = t2_strips(p);
    const int64_t nwg = ceil_div(sp.nstrips, jk::WAVES_PER_WG);
    if (nwg <= 0 || nwg > 0x7fffffffLL) return fail(JACOBI_EINVAL, "too many workgroups for one launch");
    const jk::LaunchArgs a{(unsigned)nwg, st, p->geo, sp, src, dst, with_residual ? p->partial : nullptr};
    return launch_checked(jk::launch_t2(p->lay.dtype == JACOBI_F64, with_residual ? jk::MODE_BOTH : jk::MODE_UPDATE, a),
                          "two-step kernel launch");
}

// ---- pipelined temporal blocking (tall strips) ----------------------------------------------
bool tp_usable(const jacobi_plan *p, int depth)
{
    const Geo &g = p->geo;
    const int nv = 16 / (int)p->esize;
    return depth >= jk::TP_MIN && depth <= jk::TP_MAX && g.ndim == 2 && g.tw % nv == 0 && g.th >= depth &&
           (int64_t)g.Tx * g.tile_stride * (int64_t)p->esize < 0x7fffffffLL;   // per-lane byte offsets are 32-bit
}

// columns a wavefront owns in a blocked pass of this depth (jk::TpGeometry<T, depth, ndim>::SEGW)
int tp_segment_width(const jacobi_plan *p, int depth)
{
    const int nv = 16 / (int)p->esize;
    return (jk::WAVE - 2 * jk::tp_ghost_lanes((int)p->esize, p->geo.ndim, depth)) * nv;
}

StripParams tp_strips(const jacobi_plan *p, int depth)
{
    const Geo &g = p->geo;
    StripParams sp;
    // column segments run along a whole row of tiles; strips = rows of tiles x row blocks x segments
    sp.nseg = (int)ceil_div((int64_t)g.Tx * g.tw, tp_segment_width(p, depth));
    int R = (int)p->rows_per_strip;
    if (R <= 0) {
        // every strip pays a run-in of 2*depth rows, so strips should be tall - but not so tall
        // that there are fewer than ~4 workgroups per CU to run
        R = 128;
        while (R > 8 && (int64_t)g.Ty * sp.nseg * ceil_div(g.th, R) < 4096) R /= 2;
    }
    if (R > g.th) R = g.th;
    sp.R = R;
    sp.nblk = (int)ceil_div(g.th, sp.R);
    sp.nstrips = (int64_t)g.Ty * sp.nseg * sp.nblk;
    sp.fused = 0;
    sp.xcd_chunk = xcd_chunk_of(p);
    return sp;
}

int launch_tp(jacobi_plan *p, int depth, const void *src, void *dst, bool with_residual, hipStream_t st)
{
    const StripParams sp = tp_strips(p, depth);
    const int64_t nwg = ceil_div(sp.nstrips, jk::WAVES_PER_WG);
    if (nwg <= 0 || nwg > 0x7fffffffLL) return fail(JACOBI_EINVAL, "too many workgroups for one launch");
    jk::LaunchArgs a{(unsigned)nwg, st, p->geo, sp, src, dst, with_residual ? p->partial : nullptr};
    // On a grid much larger than the caches a blocked pass streams best with at most 2 workgroups on a CU
    // (more wavefronts marching through memory at once slow the memory system down: 16384^2 at depth 4 takes
    // 0.86 ms per pass with the 5 that fit, 0.83 with 3, 0.80 with 2, 0.85 with 1), so half of the CU's LDS,
    // which the kernel never touches, is requested with each workgroup.  Grids of 0.5 GB and less measured
    // faster without the limit.  (Depth 9, at 167 registers, would otherwise run 3 per CU: 0.99 ms per pass
    // against 0.94 for depth 10.)
    a.lds = p->lay.grid_bytes >= LARGE_GRID_BYTES ? lds_to_limit_workgroups(p, 2) : 0;
    a.per_cu = 2;
    a.limit_failed = &p->lds_limit_failed;
    const int mode = with_residual ? jk::MODE_BOTH : jk::MODE_UPDATE;
    return launch_checked(p->lay.dtype == JACOBI_F64 ? jk::launch_tp_f64(depth, mode, a) : jk::launch_tp_f32(depth, mode, a),
                          "pipelined blocked-pass kernel launch");
}

// ---- 3-D pipelined temporal blocking ------------------------------------------------------------
bool tp3d_usable(const jacobi_plan *p, int depth)
{
    const Geo &g = p->geo;
    const int nv = 16 / (int)p->esize;
    return g.ndim == 3 && depth >= jk::TP3D_MIN && depth <= jk::TP3D_MAX && g.tw % nv == 0 && g.th >= depth &&
           g.td >= depth &&
           (int64_t)g.Tx * g.tile_stride * (int64_t)p->esize < 0x7fffffffLL;   // per-lane byte offsets are 32-bit
}

int tp3d_rows_per_wave(const jacobi_plan *p, int depth)
{
    if (depth == 3) return 2;
    const int rw = (int)p->rows_per_wave;
    return rw == 2 ? 2 : rw == 4 ? 4 : (p->geo.th >= 4 ? 4 : 2);
}

StripParams tp3d_strips(const jacobi_plan *p, int depth, int *nrg_out)
{
    const Geo &g = p->geo;
    StripParams sp;
    const int rw = tp3d_rows_per_wave(p, depth);
    const int nrg = (int)ceil_div(g.th, rw);
    sp.nseg = (int)ceil_div((int64_t)g.Tx * g.tw, tp_segment_width(p, depth));
    int R = (int)p->rows_per_strip;
    if (R <= 0) {
        // a strip pays a run-in of 2*depth planes: keep it deep, but leave enough strips to fill the chip
        R = g.td;
        while (R > 8 && (int64_t)g.Tz * g.Ty * nrg * sp.nseg * ceil_div(g.td, R) < 8192) R = (R + 1) / 2;
    }
    if (R > g.td) R = g.td;
    sp.R = R;
    sp.nblk = (int)ceil_div(g.td, R);
    sp.nstrips = (int64_t)g.Tz * g.Ty * sp.nblk * nrg * sp.nseg;
    sp.fused = 0;
    sp.xcd_chunk = xcd_chunk_of(p);
    // depth 3 (2 owned rows of 8 loaded) runs faster when a workgroup's wavefronts are neighbours in y;
    // depth 2 (4 of 8) when they are neighbours in x
    sp.rows_fastest = depth >= 3;
    if (nrg_out) *nrg_out = nrg;
    return sp;
}

int launch_tp3d(jacobi_plan *p, int depth, const void *src, void *dst, bool with_residual, hipStream_t st)
{
    int nrg = 0;
    const StripParams sp = tp3d_strips(p, depth, &nrg);
    const int64_t nwg = ceil_div(sp.nstrips, jk::WAVES_PER_WG);
    if (nwg <= 0 || nwg > 0x7fffffffLL) return fail(JACOBI_EINVAL, "too many workgroups for one launch");
    jk::LaunchArgs a{(unsigned)nwg, st, p->geo, sp, src, dst, with_residual ? p->partial : nullptr};
    a.aux = nrg;
    const int mode = with_residual ? jk::MODE_BOTH : jk::MODE_UPDATE;
    const int rw = tp3d_rows_per_wave(p, depth);
    return launch_checked(p->lay.dtype == JACOBI_F64 ? jk::launch_tp3d_f64(depth, rw, mode, a)
                                                     : jk::launch_tp3d_f32(depth, rw, mode, a),
                          "3-D blocked-pass kernel launch");
}

// ---- 3-D workgroup-cooperative temporal blocking --------------------------------------------------
bool tc3d_usable(const jacobi_plan *p, int depth)
{
    const Geo &g = p->geo;
    const int nv = 16 / (int)p->esize;
    return p->cooperative && g.ndim == 3 && depth >= jk::TC3D_MIN && depth <= jk::TC3D_MAX && g.tw % nv == 0 &&
           g.td >= depth && (int64_t)g.Ty * g.th < 0x7fffffffLL - 64 &&
           (int64_t)g.Tx * g.tile_stride * (int64_t)p->esize < 0x7fffffffLL;   // per-lane byte offsets are 32-bit
}

// sp.nstrips = 4 per work unit (one partial sum per unit); *nyg_out = row groups along the whole column of tiles
StripParams tc3d_strips(const jacobi_plan *p, int depth, int *nyg_out)
{
    const Geo &g = p->geo;
    StripParams sp;
    const int own = jk::TC3D_WAVES * jk::tc3d_rows_per_wave(depth) - 2 * depth;
    const int nyg = (int)ceil_div((int64_t)g.Ty * g.th, own);
    sp.nseg = (int)ceil_div((int64_t)g.Tx * g.tw, tp_segment_width(p, depth));
    int R = (int)p->rows_per_strip;
    if (R <= 0) {
        // One workgroup runs per CU and all units of a launch take the same time (R + 2*depth plane
        // steps), so the launch takes about ceil(units / CUs) rounds of that: pick the split of the tile
        // depth that minimises rounds x steps (deep units amortise the run-in, more units fill the last round).
        int64_t best = -1;
        R = g.td;
        for (int nblk = 1; nblk <= 16 && nblk <= g.td; ++nblk) {
            const int r = (int)ceil_div(g.td, nblk);
            if ((int)ceil_div(g.td, r) != nblk) continue;
            const int64_t units = (int64_t)g.Tz * nyg * sp.nseg * nblk;
            const int64_t cost = ceil_div(units, p->num_cu) * (r + 2 * depth);
            if (best < 0 || cost < best) { best = cost; R = r; }
        }
    }
    if (R > g.td) R = g.td;
    sp.R = R;
    sp.nblk = (int)ceil_div(g.td, R);
    sp.nstrips = (int64_t)g.Tz * sp.nblk * sp.nseg * nyg * jk::WAVES_PER_WG;   // partial sums: one per unit
    sp.fused = 0;
    sp.xcd_chunk = xcd_chunk_of(p);
    if (nyg_out) *nyg_out = nyg;
    return sp;
}

int launch_tc3d(jacobi_plan *p, int depth, const void *src, void *dst, bool with_residual, hipStream_t st)
{
    int nyg = 0;
    const StripParams sp = tc3d_strips(p, depth, &nyg);
    const int64_t nwg = sp.nstrips / jk::WAVES_PER_WG;      // exactly one workgroup per unit: all of them have work
    if (nwg <= 0 || nwg > 0x7fffffffLL) return fail(JACOBI_EINVAL, "too many workgroups for one launch");
    jk::LaunchArgs a{(unsigned)nwg, st, p->geo, sp, src, dst, with_residual ? p->partial : nullptr};
    a.aux = nyg;
    const int mode = with_residual ? jk::MODE_BOTH : jk::MODE_UPDATE;
    return launch_checked(p->lay.dtype == JACOBI_F64 ? jk::launch_tc3d_f64(depth, mode, a)
                                                     : jk::launch_tc3d_f32(depth, mode, a),
                          "3-D cooperative blocked-pass kernel launch");
}

// ---- all iterations of a call in one launch (resident_kernel.h) -----------------------------------------
// Which small 2-D plans run that way, and how: column segments and rows per wavefront, rows a workgroup owns
// (B) and ghost rows per side (d), workgroups, and the phases the iterations are cut into.
struct ResidentChoice {
    bool ok = false;
    int nseg = 0, rw = 0, B = 0, d = 0, nwg = 0, nphase = 0, depth = 0, n_deep = 0;
};

constexpr int RESIDENT_DEFAULT_DEPTH = 20;
constexpr int RESIDENT_MAX_WORKGROUPS = 1024;           // the plan's scratch holds a partial sum for each
constexpr unsigned RESIDENT_DEFAULT_SPIN = 1u << 22;    // polls of about a microsecond each: seconds

// with_residual: the kernel is also to deliver the residual norm of its result, for which the rows next to a
// workgroup's own must still be exact after the deepest phase: one more ghost row per side.
ResidentChoice resident_choice(const jacobi_plan *p, int iters, bool with_residual = false)
{
    ResidentChoice c;
    const Geo &g = p->geo;
    const int nv = 16 / (int)p->esize;
    if (!p->resident || g.ndim != 2 || iters < 1 || g.tw % nv) return c;
    const int64_t Nx = (int64_t)g.Tx * g.tw, Ny = (int64_t)g.Ty * g.th;
    const int nseg = (int)ceil_div(Nx, (int64_t)jk::WAVE * nv);
    if (nseg > jk::RES_MAX_SEG) return c;
    // rows a wavefront can keep: two register sets of rows x vectors have to fit 128 registers
    const int max_rw = nseg == 2 ? jk::RES_MAX_RW - 1 : jk::RES_MAX_RW;
    int rw = (int)p->resident_rows;
    if (rw > max_rw) rw = max_rw;
    // one workgroup holds the whole grid and its two ring rows if they fit: no barrier, one phase
    const int rw_single = (int)ceil_div(Ny + 2, jk::RES_WAVES);
    if (rw_single <= max_rw && (rw == 0 || rw >= rw_single)) {
        c.ok = true;
        c.nseg = nseg; c.rw = rw ? rw : rw_single; c.B = (int)Ny; c.d = 1; c.nwg = 1;
        c.nphase = 1; c.depth = iters; c.n_deep = 0;
        return c;
    }
    if (rw == 0) rw = max_rw;
    const int held = jk::RES_WAVES * rw;
    const int spare = with_residual ? 1 : 0;
    int d0 = p->resident_depth > 0 ? (int)p->resident_depth : RESIDENT_DEFAULT_DEPTH;
    if (d0 > (held - 1) / 2 - spare) d0 = (held - 1) / 2 - spare;     // at least one owned row
    if (d0 > iters) d0 = iters;                           // no more ghost rows than a phase can use
    // deep phases leave few owned rows per workgroup; the grid barrier needs every workgroup resident, so
    // tall grids get shallower phases
    for (; d0 >= 1; --d0) {
        c.nphase = (int)ceil_div(iters, d0);
        c.depth = iters / c.nphase;
        c.n_deep = iters % c.nphase;
        c.d = c.depth + (c.n_deep ? 1 : 0) + spare;      // the phases are equally deep: ghost rows for the deepest
        c.B = held - 2 * c.d;
        const int64_t nwg = ceil_div(Ny, c.B);
        if (nwg > p->num_cu || nwg > RESIDENT_MAX_WORKGROUPS) continue;
        c.ok = true;
        c.nseg = nseg; c.rw = rw; c.nwg = (int)nwg;
        return c;
    }
    return c;
}

// copy_ring: `out` does not carry the Dirichlet ring yet; residual_out_dev: if not null, the residual norm of
// the grid the launch produces (the choice must have been made with_residual).
int launch_resident(jacobi_plan *p, const ResidentChoice &c, void *in, void *out, hipStream_t st, bool copy_ring,
                    double *residual_out_dev)
{
    jk::ResidentLaunch a;
    a.nwg = (unsigned)c.nwg;
    a.st = st;
    a.g = p->geo;
    a.rp.B = c.B; a.rp.d = c.d; a.rp.nphase = c.nphase; a.rp.depth = c.depth; a.rp.n_deep = c.n_deep;
    a.rp.spin_limit = p->resident_spin_limit > 0 ? (unsigned)(p->resident_spin_limit - 1) : RESIDENT_DEFAULT_SPIN;
    a.rp.sync = p->sync_words;
    a.rp.copy_ring = copy_ring ? 1 : 0;
    a.rp.partial = p->partial;
    a.rp.residual = residual_out_dev;
    a.in = in; a.out = out;
    return launch_checked(jk::launch_resident(p->lay.dtype == JACOBI_F64, c.nseg, c.rw, a), "resident kernel launch");
}

// What the next pass does with `left` iterations to go.  The iterations are spread evenly over
// few passes of equal depth (10 iterations at depth 8 run as 5 + 5, not 8 + 2: up to depth 8 a
// pass costs no more for being deeper).  kernel: 0 single step (needs current
// halos), 1 two-step kernel (2-D), 2 pipelined kernel (2-D, depths 3..12), 3 / 4 pipelined 3-D
// kernels (depths 2..4).
struct PassChoice { int depth; int kernel; };

// 3-D blocked pass of this depth: 4 = workgroup-cooperative kernel, 3 = one wavefront per row group
// (the faster one at depth 2, and the only one with option cooperative = 0), 0 = neither can run it.
int pick_3d_kernel(const jacobi_plan *p, int depth)
{
    const bool per_wave = tp3d_usable(p, depth) && (p->lay.dtype == JACOBI_F64 || depth == jk::TP3D_MIN);
    if (depth == 2 && per_wave) return 3;
    if (tc3d_usable(p, depth)) return 4;
    return per_wave ? 3 : 0;
}

PassChoice choose_pass(const jacobi_plan *p, int left)
{
    int maxd = (int)(p->tblock < left ? p->tblock : left);
    if (maxd > jk::TP_MAX) maxd = jk::TP_MAX;
    if (maxd >= 2 && p->geo.ndim == 3) {
        // fp32 passes deeper than 3 are bound by arithmetic and measured slower per iteration
        int deepest = 0;
        for (int d = p->lay.dtype == JACOBI_F64 ? jk::TC3D_MAX : 3; d >= 2 && !deepest; --d)
            if (pick_3d_kernel(p, d)) deepest = d;
        if (deepest) {
            if (maxd > deepest) maxd = deepest;
            const int passes = (left + maxd - 1) / maxd;
            for (int d = (left + passes - 1) / passes; d >= 2; --d)
                if (const int k = pick_3d_kernel(p, d)) return {d, k};
        }
    } else if (maxd >= 2) {
        int deepest = 0;                 // low tiles limit the depth (a pass reaches at most one tile up and down)
        for (int d = maxd; d >= jk::TP_MIN && !deepest; --d)
            if (tp_usable(p, d)) deepest = d;
        if (deepest) {
            // A pass is bound by memory up to about depth 8 (it costs nearly the same whatever its depth) and by
            // arithmetic beyond (cost proportional to the depth).  Cheapest plan: as many passes as fit at 8 or
            // more iterations each, equally deep, none deeper than `deepest` (10 iterations: one pass of 10, not
            // 5 + 5; 50: 9 + 9 + 8 + 8 + 8 + 8).  On grids much larger than the caches passes of 10 run the most
            // iterations per second (16384^2: 0.094 ms per iteration in passes of 10, 0.106 in passes of 8, 0.110
            // in passes of 9), so there the passes are made 10 or more deep (50: 5 x 10); smaller grids lose
            // with that (4096^2: 0.0104 against 0.0092-0.0097).
            const int target = p->lay.grid_bytes >= LARGE_GRID_BYTES ? 10 : 8;
            const int cap = deepest < target ? deepest : target;
            int passes = left / cap > 0 ? left / cap : 1;
            if ((left + passes - 1) / passes > deepest) passes = (left + deepest - 1) / deepest;
            const int best_d = (left + passes - 1) / passes;
            if (best_d >= jk::TP_MIN) return {best_d, 2};
        }
        if (t2_usable(p)) return {2, 1};
    }
    return {1, 0};
}

template <typename T>
int launch_boundary_t(jacobi_plan *p, const T *src, T *dst, hipStream_t st)
{
    const Geo &g = p->geo;
    // largest face, in cells, including its edge cells
    const int64_t pd = g.nplanes, ph = g.rows;
    int64_t max_face = pd * ph;                                    // x faces
    if (pd * g.tw > max_face) max_face = pd * g.tw;                // y faces
    if (g.ndim == 3 && ph * g.tw > max_face) max_face = ph * g.tw; // z faces
    const int chunks = (int)ceil_div(max_face, jk::FACE_CHUNK);
    const int64_t nitems = (int64_t)g.ntiles * 2 * g.ndim * chunks;
    const int64_t nblk = nitems < MAX_COPY_BLOCKS ? nitems : MAX_COPY_BLOCKS;
    hipLaunchKernelGGL((jk::boundary_copy_kernel<T>), dim3((unsigned)nblk), dim3(jk::WG), 0, st, g, src, dst,
                       chunks, (long long)nitems);
    HIP_TRY(hipGetLastError());
    return JACOBI_OK;
}

template <typename T, int XSRC>
int launch_exchange_t(jacobi_plan *p, T *grid, hipStream_t st)
{
    const Geo &g = p->geo;
    const int nv = 16 / (int)sizeof(T);
    const int64_t vrow = ceil_div(g.tw, nv);
    // largest face in its copy units: cells of an x face, 16-byte vectors of a y or z face
    int64_t units = (int64_t)g.td * g.th;
    if ((int64_t)g.td * vrow > units) units = (int64_t)g.td * vrow;
    if (g.ndim == 3 && (int64_t)g.th * vrow > units) units = (int64_t)g.th * vrow;
    const int chunks = (int)ceil_div(units, jk::HALO_CHUNK);
    const int64_t nitems = (int64_t)g.ntiles * 2 * g.ndim * chunks;            // one per wavefront
    const int64_t nwg = ceil_div(nitems, jk::WAVES_PER_WG);
    const int64_t nblk = nwg < MAX_COPY_BLOCKS ? nwg : MAX_COPY_BLOCKS;
    hipLaunchKernelGGL((jk::halo_exchange_kernel<T, XSRC>), dim3((unsigned)nblk), dim3(jk::WG), 0, st, g, grid, chunks,
                       (long long)nitems);
    HIP_TRY(hipGetLastError());
    return JACOBI_OK;
}

// Halo exchange of `grid`.  from_send_arrays: the x faces are copied from the tiles' dense x send arrays (only
// valid if the grid was just produced by an update in FUSED_PACK mode) instead of gathered from their columns.
int launch_exchange(jacobi_plan *p, void *grid, hipStream_t st, bool from_send_arrays = false)
{
    if (p->geo.ntiles == 1) return JACOBI_OK;   // no neighbours, nothing to copy
    if (p->lay.dtype == JACOBI_F64)
        return from_send_arrays ? launch_exchange_t<double, 1>(p, (double *)grid, st) : launch_exchange_t<double, 0>(p, (double *)grid, st);
    return from_send_arrays ? launch_exchange_t<float, 1>(p, (float *)grid, st) : launch_exchange_t<float, 0>(p, (float *)grid, st);
}

int launch_boundary_sync(jacobi_plan *p, const void *in, void *out, hipStream_t st)
{
    return p->lay.dtype == JACOBI_F64 ? launch_boundary_t<double>(p, (const double *)in, (double *)out, st)
                                      : launch_boundary_t<float>(p, (const float *)in, (float *)out, st);
}

template <typename T, bool GATHER>
int launch_sg_t(jacobi_plan *p, const T *from, T *to, hipStream_t st)
{
    const Geo &g = p->geo;
    const long long GP = p->lay.dims[2] + 2, GQ = (p->lay.dims[1] + 2) * GP;
    const int64_t nrows = (int64_t)g.ntiles * g.nplanes * g.rows;
    if (nrows > 0x7fffffffLL) return fail(JACOBI_EINVAL, "too many tile rows for one scatter / gather launch");
    const int cols = g.tw + 2;
    // a wavefront per row and chunk of up to 256 cells, four per lane in flight (fewer for narrower tiles)
    const int q = (int)std::min<int64_t>(4, ceil_div(cols, jk::WAVE));
    const int64_t nchunks = ceil_div(cols, q * jk::WAVE), nitems = nrows * nchunks;
    const int64_t nwg = ceil_div(nitems, jk::WAVES_PER_WG);
    if (nitems > 0xfffffff0LL) return fail(JACOBI_EINVAL, "too many row chunks for one scatter / gather launch");
#define JK_SG(Q_) \
    hipLaunchKernelGGL((jk::scatter_gather_kernel<T, GATHER, Q_>), dim3((unsigned)nwg), dim3(jk::WG), 0, st, g, from, to, \
                       GP, GQ, (unsigned)nchunks, (unsigned)nitems)
    switch (q) {
    case 1: JK_SG(1); break;
    case 2: JK_SG(2); break;
    case 3: JK_SG(3); break;
    default: JK_SG(4); break;
    }
#undef JK_SG
    HIP_TRY(hipGetLastError());
    return JACOBI_OK;
}

// Partial sums (one per workgroup) the largest residual-producing launch can write, over every pass kind and
// every value the options can take: the finest strips (one row or plane each, the fewest rows per wavefront)
// give the most workgroups.  The plan's scratch is sized for this once, so no option change ever makes it grow.
int64_t max_partials(jacobi_plan *p)
{
    const int64_t saved_rps = p->rows_per_strip, saved_rpw = p->rows_per_wave;
    p->rows_per_strip = 1;
    int64_t most = 0;
    auto take = [&](int64_t strips) { most = std::max(most, ceil_div(strips, jk::WAVES_PER_WG)); };
    for (int64_t rpw : {1, 2, 4}) {
        p->rows_per_wave = rpw;
        take(make_config(p, jk::MODE_RESIDUAL).sp.nstrips);
        take(make_config(p, jk::MODE_BOTH).sp.nstrips);
        if (p->geo.ndim == 2) take(stack_strips(p, StackChoice{4, 8}).nstrips);      // the stacked kernel: never more than the others
        if (p->geo.ndim == 3)
            for (int d = jk::TP3D_MIN; d <= jk::TP3D_MAX; ++d) take(tp3d_strips(p, d, nullptr).nstrips);
    }
    if (p->geo.ndim == 2) {
        take(t2_strips(p).nstrips);
        for (int d = jk::TP_MIN; d <= jk::TP_MAX; ++d) take(tp_strips(p, d).nstrips);
    } else {
        for (int d = jk::TC3D_MIN; d <= jk::TC3D_MAX; ++d) take(tc3d_strips(p, d, nullptr).nstrips);
    }
    p->rows_per_strip = saved_rps;
    p->rows_per_wave = saved_rpw;
    if (p->geo.ndim == 2) most = std::max<int64_t>(most, RESIDENT_MAX_WORKGROUPS);      // the one-launch kernel's
    return most;
}

// One-time device set-up of a plan: reads the device's CU count and LDS size and allocates the residual
// scratch.  The only place the library allocates device memory; called by jacobi_prepare and, if the caller
// has not done so, by the first entry point that enqueues work (which therefore cannot be recorded into a
// HIP graph; every later call can).
int prepare_plan(jacobi_plan *p)
{
    if (p->prepared) return JACOBI_OK;
    int dev = 0, v = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) p->num_cu = v;
    else (void)hipGetLastError();
    // 160 KiB on gfx950: a workgroup may use all of a CU's LDS
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) == hipSuccess && v >= 65536) p->cu_lds = v;
    else (void)hipGetLastError();
    const int64_t need = max_partials(p) + 1;      // + the slot residual_norm_host reads back
    // behind them: two doubles' worth of words for the resident kernel's grid barrier
    hipError_t e = hipMalloc((void **)&p->partial, (size_t)(need + 2) * sizeof(double));
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        return fail(JACOBI_ENOMEM, "device allocation of residual scratch failed");
    }
    if (e != hipSuccess) return fail_hip(e, "hipMalloc(residual scratch)");
    p->partial_cap = need;
    p->sync_words = (unsigned *)(p->partial + need);
    // the resident kernel's barrier words are zero between launches: it clears them itself when it finishes
    e = hipMemset(p->sync_words, 0, 2 * sizeof(double));
    if (e != hipSuccess) {
        (void)hipFree(p->partial);
        p->partial = nullptr;
        return fail_hip(e, "hipMemset(barrier words)");
    }
    p->prepared = true;
    return JACOBI_OK;
}

int check_partials(const jacobi_plan *p, int64_t nwg)
{
    // cannot happen (max_partials covers every launch); kept so that a planning mistake is an error, not a fault
    if (nwg + 1 > p->partial_cap) return fail(JACOBI_EINVAL, "internal: residual scratch smaller than the launch");
    return JACOBI_OK;
}

// Residual pass of `grid` (it reads the neighbouring tiles' edge cells itself: the grid's halo cells need not be
// current and are left alone), partial sums into `partial` (at least nwg entries), result to *out.
int residual_launches(jacobi_plan *p, void *grid, double *partial, double *out, hipStream_t st)
{
    const int64_t nwg = single_step_workgroups(p, jk::MODE_RESIDUAL);
    int rc = launch_sweep(p, jk::MODE_RESIDUAL, grid, grid, partial, st, 0, 0, /*pull=*/true);
    if (rc) return rc;
    hipLaunchKernelGGL(jk::residual_final_kernel, dim3(1), dim3(1024), 0, st, partial, (long long)nwg, out);
    HIP_TRY(hipGetLastError());
    return JACOBI_OK;
}

int residual_common(jacobi_plan *p, void *grid, double *result_dev, hipStream_t st)
{
    int rc = prepare_plan(p);
    if (rc) return rc;
    const int64_t nwg = single_step_workgroups(p, jk::MODE_RESIDUAL);
    rc = check_partials(p, nwg);
    if (rc) return rc;
    // the last slot of the scratch holds the result for the host variant
    return residual_launches(p, grid, p->partial, result_dev ? result_dev : p->partial + p->partial_cap - 1, st);
}

// Grid buffers must be 16-byte aligned (every lane moves 16 bytes at a time).
bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

// Two grids of this plan overlap if their start addresses are closer than one grid.
bool grids_overlap(const jacobi_plan *p, const void *a, const void *b)
{
    const uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
    const uintptr_t d = x > y ? x - y : y - x;
    return d < (uintptr_t)p->lay.grid_bytes;
}

// The settable options: where the value lives, its range, and - where only a few values inside the range are
// meaningful - those values (zero-terminated list after the always-allowed 0).
struct OptionSpec {
    const char *key;
    int64_t jacobi_plan::*field;
    int64_t lo, hi;
    int64_t only[6];        // if only[0] != 0: the value must be 0 or one of these
};
const OptionSpec OPTIONS[] = {
    {"fused", &jacobi_plan::fused, 0, 1, {}},
    {"rows_per_strip", &jacobi_plan::rows_per_strip, 0, 4096, {}},
    {"nontemporal", &jacobi_plan::nontemporal, 0, 2, {}},
    {"profile", &jacobi_plan::profile, 0, 1, {}},
    {"unroll", &jacobi_plan::unroll, 0, 16, {1, 2, 4, 8, 16}},
    {"xcd_chunk", &jacobi_plan::xcd_chunk, 0, 1 << 20, {}},
    {"rows_per_wave", &jacobi_plan::rows_per_wave, 0, 4, {1, 2, 4}},
    {"tblock", &jacobi_plan::tblock, 1, jk::TP_MAX, {}},
    {"cooperative", &jacobi_plan::cooperative, 0, 1, {}},
    {"resident", &jacobi_plan::resident, 0, 1, {}},
    {"resident_depth", &jacobi_plan::resident_depth, 0, 31, {}},
    {"resident_rows", &jacobi_plan::resident_rows, 0, jk::RES_MAX_RW, {}},
    {"resident_spin_limit", &jacobi_plan::resident_spin_limit, 0, 1LL << 31, {}},
    {"cu_lds", &jacobi_plan::cu_lds_option, 0, 1LL << 20, {}},
    {"stack", &jacobi_plan::stack, 0, 8, {1, 4, 8}},
};

const OptionSpec *find_option(const char *key)
{
    for (const OptionSpec &o : OPTIONS)
        if (!strcmp(key, o.key)) return &o;
    return nullptr;
}

}  // namespace

extern "C" {

const char *jacobi_last_error(void) { return g_err.c_str(); }

int jacobi_create(jacobi_plan **plan, int ndim, const int64_t *dims, const int64_t *tiles, int dtype)
{
    if (!plan) return fail(JACOBI_EINVAL, "plan is NULL");
    *plan = nullptr;
    if (!dims || !tiles) return fail(JACOBI_EINVAL, "dims or tiles is NULL");
    if (ndim != 2 && ndim != 3) return fail(JACOBI_EINVAL, "ndim must be 2 or 3");
    if (dtype != JACOBI_F64 && dtype != JACOBI_F32) return fail(JACOBI_EINVAL, "unknown dtype");
    for (int d = 0; d < ndim; ++d) {
        if (dims[d] <= 0) return fail(JACOBI_EINVAL, "dims must be positive");
        if (tiles[d] <= 0) return fail(JACOBI_EINVAL, "tiles must be positive");
    }
    for (int d = 0; d < ndim; ++d)
        if (dims[d] % tiles[d]) return fail(JACOBI_ENOTDIV, "dims[d] is not a multiple of tiles[d]");

    jacobi_plan *p = new (std::nothrow) jacobi_plan();
    if (!p) return fail(JACOBI_ENOMEM, "host allocation failed");
    jacobi_layout &L = p->lay;
    memset(&L, 0, sizeof(L));
    L.ndim = ndim;
    L.dtype = dtype;
    p->esize = dtype == JACOBI_F64 ? 8 : 4;
    L.dims[0] = L.tiles[0] = L.tile[0] = 1;
    for (int d = 0; d < ndim; ++d) {
        const int s = 3 - ndim + d;
        L.dims[s] = dims[d];
        L.tiles[s] = tiles[d];
        L.tile[s] = dims[d] / tiles[d];
    }
    const int64_t line = 128 / (int64_t)p->esize;   // elements per 128-byte cache line
    L.ntiles = L.tiles[0] * L.tiles[1] * L.tiles[2];
    L.nplanes = ndim == 3 ? L.tile[0] + 2 : 1;
    L.pitch = round_up(L.tile[2], line);
    L.plane = (L.tile[1] + 2) * L.pitch;
    L.xhalo_offset = L.nplanes * L.plane;
    // at least 3 spare elements after each array: a vector read that starts at the last entry stays inside the tile
    L.xhalo_pitch = round_up(L.nplanes * (L.tile[1] + 2) + 3, line);
    L.xsend_offset = L.xhalo_offset + 2 * L.xhalo_pitch;
    L.tile_stride = L.xsend_offset + 2 * L.xhalo_pitch;
    L.grid_bytes = L.ntiles * L.tile_stride * (int64_t)p->esize;

    const int64_t lim = 0x7fffffffLL;
    if (L.tile_stride > lim || L.ntiles > lim || L.dims[0] + 2 > lim || L.dims[1] + 2 > lim || L.dims[2] + 2 > lim) {
        delete p;
        return fail(JACOBI_EINVAL, "tile or tile count too large (32-bit index limit inside a tile)");
    }
    if (ndim == 3 && L.plane * (int64_t)p->esize >= 0x80000000LL) {
        delete p;
        return fail(JACOBI_EINVAL, "tile too large (a plane of a 3-D tile must be smaller than 2 GiB)");
    }
    Geo &g = p->geo;
    g.ndim = ndim;
    g.Tz = (int)L.tiles[0]; g.Ty = (int)L.tiles[1]; g.Tx = (int)L.tiles[2];
    g.td = (int)L.tile[0];  g.th = (int)L.tile[1];  g.tw = (int)L.tile[2];
    g.rows = g.th + 2;
    g.nplanes = (int)L.nplanes;
    g.z0 = ndim == 3 ? 1 : 0;
    g.pitch = (int)L.pitch;
    g.ntiles = (int)L.ntiles;
    g.plane = L.plane;
    g.xoff = L.xhalo_offset;
    g.hpitch = L.xhalo_pitch;
    g.xsend = L.xsend_offset;
    g.tile_stride = L.tile_stride;
    *plan = p;
    return JACOBI_OK;
}

int jacobi_destroy(jacobi_plan *plan)
{
    if (!plan) return JACOBI_OK;
    int rc = JACOBI_OK;
    if (plan->partial || !plan->ev.empty() || !plan->task_streams.empty() || !plan->task_events.empty()) {
        hipError_t e = hipDeviceSynchronize();
        if (e != hipSuccess) rc = fail_hip(e, "hipDeviceSynchronize");
        if (plan->partial) (void)hipFree(plan->partial);
        for (hipEvent_t ev : plan->ev) (void)hipEventDestroy(ev);
        for (hipEvent_t ev : plan->task_events) (void)hipEventDestroy(ev);
        for (hipStream_t s : plan->task_streams) (void)hipStreamDestroy(s);
    }
    delete plan;
    return rc;
}

int jacobi_prepare(jacobi_plan *plan)
{
    if (!plan) return fail(JACOBI_EINVAL, "plan is NULL");
    return prepare_plan(plan);
}

size_t jacobi_scratch_bytes(const jacobi_plan *plan)
{
    return plan ? (size_t)(max_partials(const_cast<jacobi_plan *>(plan)) + 1 + 2) * sizeof(double) : 0;
}

size_t jacobi_grid_bytes(const jacobi_plan *plan) { return plan ? (size_t)plan->lay.grid_bytes : 0; }

int jacobi_get_layout(const jacobi_plan *plan, jacobi_layout *layout)
{
    if (!plan || !layout) return fail(JACOBI_EINVAL, "plan or layout is NULL");
    *layout = plan->lay;
    return JACOBI_OK;
}

int jacobi_scatter(jacobi_plan *plan, const void *global_padded_dev, void *grid, void *stream)
{
    if (!plan || !global_padded_dev || !grid) return fail(JACOBI_EINVAL, "NULL argument");
    if (misaligned(grid)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    if (int rc = prepare_plan(plan)) return rc;
    return plan->lay.dtype == JACOBI_F64
               ? launch_sg_t<double, false>(plan, (const double *)global_padded_dev, (double *)grid, st)
               : launch_sg_t<float, false>(plan, (const float *)global_padded_dev, (float *)grid, st);
}

int jacobi_gather(jacobi_plan *plan, const void *grid, void *global_padded_dev, void *stream)
{
    if (!plan || !global_padded_dev || !grid) return fail(JACOBI_EINVAL, "NULL argument");
    if (misaligned(grid)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    return plan->lay.dtype == JACOBI_F64
               ? launch_sg_t<double, true>(plan, (const double *)grid, (double *)global_padded_dev, st)
               : launch_sg_t<float, true>(plan, (const float *)grid, (float *)global_padded_dev, st);
}

int halo_exchange(jacobi_plan *plan, void *grid, void *stream)
{
    if (!plan || !grid) return fail(JACOBI_EINVAL, "NULL argument");
    if (misaligned(grid)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    return launch_exchange(plan, grid, (hipStream_t)stream);
}

// What a block of iterations leaves behind for the block that jacobi_run enqueues next on the same two grids.
struct RunCarry {
    bool ring_done = false;         // both grids carry the Dirichlet ring
    bool halos_current = false;     // the inter-tile halo cells of the block's result hold its own edge cells
    bool x_packed = false;          // its x send arrays hold its first / last columns
};

// residual_in_dev: if not null, also the residual norm of `in`; residual_out_dev: if not null, also that of the
// grid the iterations produce.
static int sweep_common(jacobi_plan *plan, void *in, void *out, int iters, hipStream_t st, void **final,
                        double *residual_in_dev, RunCarry *carry = nullptr, double *residual_out_dev = nullptr)
{
    int rc = prepare_plan(plan);
    if (rc) return rc;
    if (plan->profile && plan->ev.empty()) {
        plan->ev.reserve(2 * MAX_PROFILE_EVENTS);
        for (int i = 0; i < 2 * MAX_PROFILE_EVENTS; ++i) {
            hipEvent_t e;
            HIP_TRY(hipEventCreate(&e));
            plan->ev.push_back(e);
        }
    }
    ResidentChoice rc_res = resident_choice(plan, iters, residual_out_dev != nullptr);
    const bool norm_in_launch = rc_res.ok && residual_out_dev;
    if (!rc_res.ok && residual_out_dev) rc_res = resident_choice(plan, iters);
    if (rc_res.ok) {
        // small 2-D grid: every iteration inside one launch, which also carries the ring over and delivers the
        // residual of its result; the residual of `in`, if asked for, from the stand-alone reduction first
        if (residual_in_dev) {
            const int64_t nwg = single_step_workgroups(plan, jk::MODE_RESIDUAL);
            rc = check_partials(plan, nwg);
            if (rc) return rc;
            rc = residual_launches(plan, in, plan->partial, residual_in_dev, st);
            if (rc) return rc;
        }
        rc = check_partials(plan, rc_res.nwg);
        if (rc) return rc;
        const bool copy_ring = !(carry && carry->ring_done);
        if (carry) *carry = RunCarry{true, false, false};      // the kernel stores rows only
        const bool timed = plan->profile && plan->ev_used < MAX_PROFILE_EVENTS;
        if (timed) HIP_TRY(hipEventRecord(plan->ev[2 * plan->ev_used], st));
        rc = launch_resident(plan, rc_res, in, out, st, copy_ring, norm_in_launch ? residual_out_dev : nullptr);
        if (rc) return rc;
        if (timed) {
            HIP_TRY(hipEventRecord(plan->ev[2 * plan->ev_used + 1], st));
            ++plan->ev_used;
        }
        void *result = (rc_res.nphase & 1) ? out : in;
        if (final) *final = result;
        if (residual_out_dev && !norm_in_launch) return residual_common(plan, result, residual_out_dev, st);
        return JACOBI_OK;
    }
    const PassChoice first = choose_pass(plan, iters);
    int64_t nwg_res = 0;
    if (residual_in_dev) {
        const int64_t strips = first.kernel == 0   ? single_step_workgroups(plan, jk::MODE_BOTH) * jk::WAVES_PER_WG
                               : first.kernel == 1 ? t2_strips(plan).nstrips
                               : first.kernel == 2 ? tp_strips(plan, first.depth).nstrips
                               : first.kernel == 4 ? tc3d_strips(plan, first.depth, nullptr).nstrips
                                                   : tp3d_strips(plan, first.depth, nullptr).nstrips;
        nwg_res = ceil_div(strips, jk::WAVES_PER_WG);
        rc = check_partials(plan, nwg_res);
        if (rc) return rc;
    }

    if (!(carry && carry->ring_done)) {
        rc = launch_boundary_sync(plan, in, out, st);
        if (rc) return rc;
    }
    void *src = in, *dst = out;
    int k = 0;
    bool halos_current = carry && carry->halos_current;     // inter-tile halos of src hold src's own edge cells
    bool x_packed = carry && carry->x_packed;   // src's x send arrays hold its first / last columns (the last pass packed them)
    while (k < iters) {
        const PassChoice pc = choose_pass(plan, iters - k);
        const bool with_res = k == 0 && residual_in_dev;
        // A single-step update needs the cells beyond each tile (blocked passes fetch theirs themselves).  With the
        // fused push they are in src's halo cells from the second update of a run on; the first one PULLS them
        // from the neighbouring tiles' edges instead of waiting for an exchange kernel.  With fused = 0 the exchange
        // is a kernel of its own before every update (paper Sec. VI-C: pack, transfer, unpack, then update).
        const bool pull = pc.depth == 1 && !halos_current && plan->fused;
        if (pc.depth == 1 && !halos_current && !plan->fused) {
            rc = launch_exchange(plan, src, st, x_packed);
            if (rc) return rc;
        }
        const bool timed = plan->profile && plan->ev_used < MAX_PROFILE_EVENTS;
        if (timed) HIP_TRY(hipEventRecord(plan->ev[2 * plan->ev_used], st));
        if (pc.kernel == 0)      rc = with_res ? launch_update_with_residual(plan, src, dst, st, pull) : launch_update(plan, src, dst, st, pull);
        else if (pc.kernel == 1) rc = launch_t2(plan, src, dst, with_res, st);
        else if (pc.kernel == 2) rc = launch_tp(plan, pc.depth, src, dst, with_res, st);
        else if (pc.kernel == 3) rc = launch_tp3d(plan, pc.depth, src, dst, with_res, st);
        else                     rc = launch_tc3d(plan, pc.depth, src, dst, with_res, st);
        if (rc) return rc;
        if (timed) {
            HIP_TRY(hipEventRecord(plan->ev[2 * plan->ev_used + 1], st));
            ++plan->ev_used;
        }
        if (with_res) {
            hipLaunchKernelGGL(jk::residual_final_kernel, dim3(1), dim3(1024), 0, st, plan->partial,
                               (long long)nwg_res, residual_in_dev);
            HIP_TRY(hipGetLastError());
        }
        // a single-step update with the fused push leaves dst's halos current; without it, dst's x send arrays
        halos_current = pc.depth == 1 && plan->fused;
        x_packed = pc.depth == 1 && !plan->fused;
        void *t = src; src = dst; dst = t;
        k += pc.depth;
    }
    if (carry) *carry = RunCarry{true, halos_current, x_packed};
    if (final) *final = src;
    if (residual_out_dev) return residual_common(plan, src, residual_out_dev, st);
    return JACOBI_OK;
}

int jacobi_sweep(jacobi_plan *plan, void *in, void *out, int iters, void *stream, void **final)
{
    if (!plan || !in || !out) return fail(JACOBI_EINVAL, "NULL argument");
    if (in == out) return fail(JACOBI_EINVAL, "in and out must be different grids");
    if (misaligned(in) || misaligned(out)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    if (grids_overlap(plan, in, out)) return fail(JACOBI_EINVAL, "in and out overlap");
    if (iters < 0) return fail(JACOBI_EINVAL, "iters must be >= 0");
    if (final) *final = in;
    if (iters == 0) return JACOBI_OK;
    return sweep_common(plan, in, out, iters, (hipStream_t)stream, final, nullptr);
}

// Tasks of `group` consecutive tiles.  A task of iteration k+1 reads its tiles of the grid that
// iteration k wrote - interiors (written by the same task) and halo cells (pushed there by the tasks
// that own the face-neighbour tiles) - so it depends on exactly those tasks of iteration k.  The same
// edges cover the write-after-read hazards of the ping-pong buffers.
static void build_task_deps(jacobi_plan *p, int group)
{
    const Geo &g = p->geo;
    const int ntasks = (int)ceil_div(g.ntiles, group);
    p->task_deps.assign(ntasks, std::vector<int>());
    for (int t = 0; t < g.ntiles; ++t) {
        const int tz = t / (g.Ty * g.Tx), ty = (t / g.Tx) % g.Ty, tx = t % g.Tx;
        std::vector<int> &d = p->task_deps[t / group];
        auto add = [&](int z, int y, int x) {
            if (z < 0 || z >= g.Tz || y < 0 || y >= g.Ty || x < 0 || x >= g.Tx) return;
            const int task = ((z * g.Ty + y) * g.Tx + x) / group;
            if (std::find(d.begin(), d.end(), task) == d.end()) d.push_back(task);
        };
        add(tz, ty, tx);
        add(tz, ty, tx - 1); add(tz, ty, tx + 1);
        add(tz, ty - 1, tx); add(tz, ty + 1, tx);
        add(tz - 1, ty, tx); add(tz + 1, ty, tx);
    }
    p->task_group = group;
}

int jacobi_sweep_tasks(jacobi_plan *plan, void *in, void *out, int iters, int tiles_per_task, int nstreams,
                       void *stream, void **final)
{
    if (!plan || !in || !out) return fail(JACOBI_EINVAL, "NULL argument");
    if (in == out) return fail(JACOBI_EINVAL, "in and out must be different grids");
    if (misaligned(in) || misaligned(out)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    if (grids_overlap(plan, in, out)) return fail(JACOBI_EINVAL, "in and out overlap");
    if (iters < 0) return fail(JACOBI_EINVAL, "iters must be >= 0");
    if (tiles_per_task < 1 || nstreams < 1 || nstreams > MAX_TASK_STREAMS)
        return fail(JACOBI_EINVAL, "tiles_per_task must be >= 1 and nstreams in 1..16");
    if (!plan->fused) return fail(JACOBI_EINVAL, "task execution needs option fused = 1 (tasks push their edge cells)");
    if (final) *final = in;
    if (iters == 0) return JACOBI_OK;
    const Geo &g = plan->geo;
    hipStream_t st = (hipStream_t)stream;
    int rc = prepare_plan(plan);
    if (rc) return rc;
    {
        // Recording this fork / join pattern into a HIP graph crashed inside the runtime when the capture
        // was ended (host-side segmentation fault, cause not found), and the same DAG built node by node
        // made the runtime abort now and then: task execution stays outside HIP graphs.
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        HIP_TRY(hipStreamIsCapturing(st, &cs));
        if (cs != hipStreamCaptureStatusNone)
            return fail(JACOBI_EINVAL, "jacobi_sweep_tasks cannot be recorded into a HIP graph");
    }
    const int group = tiles_per_task > g.ntiles ? g.ntiles : tiles_per_task;
    const int ntasks = (int)ceil_div(g.ntiles, group);
    const int S = nstreams < ntasks ? nstreams : ntasks;

    if (plan->task_group != group) build_task_deps(plan, group);
    while ((int)plan->task_streams.size() < S) {
        hipStream_t s;
        HIP_TRY(hipStreamCreateWithFlags(&s, hipStreamNonBlocking));
        plan->task_streams.push_back(s);
    }
    const size_t nev = 2 * (size_t)ntasks + 1 + MAX_TASK_STREAMS;
    while (plan->task_events.size() < nev) {
        hipEvent_t e;
        HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        plan->task_events.push_back(e);
    }
    hipEvent_t *done = plan->task_events.data();                  // done[2*task + parity]
    const hipEvent_t fork = plan->task_events[2 * (size_t)ntasks];
    hipEvent_t *joined = plan->task_events.data() + 2 * (size_t)ntasks + 1;

    // on the caller's stream: the Dirichlet ring of `out`, and current halos of `in` for the first iteration
    rc = launch_boundary_sync(plan, in, out, st);
    if (rc) return rc;
    rc = launch_exchange(plan, in, st);
    if (rc) return rc;
    HIP_TRY(hipEventRecord(fork, st));
    for (int s = 0; s < S; ++s) HIP_TRY(hipStreamWaitEvent(plan->task_streams[s], fork, 0));

    void *src = in, *dst = out;
    for (int k = 0; k < iters; ++k) {
        for (int a = 0; a < ntasks; ++a) {
            hipStream_t s = plan->task_streams[a % S];
            if (k > 0)
                for (int b : plan->task_deps[a])
                    if (b % S != a % S)                              // same stream: already in order
                        HIP_TRY(hipStreamWaitEvent(s, done[2 * b + ((k - 1) & 1)], 0));
            const int t0 = a * group, cnt = t0 + group <= g.ntiles ? group : g.ntiles - t0;
            rc = launch_sweep(plan, jk::MODE_UPDATE, src, dst, nullptr, s, t0, cnt);
            if (rc) return rc;
            HIP_TRY(hipEventRecord(done[2 * a + (k & 1)], s));
        }
        void *t = src; src = dst; dst = t;
    }
    for (int s = 0; s < S; ++s) {
        HIP_TRY(hipEventRecord(joined[s], plan->task_streams[s]));
        HIP_TRY(hipStreamWaitEvent(st, joined[s], 0));
    }
    if (final) *final = src;
    return JACOBI_OK;
}

int jacobi_task_dependencies(jacobi_plan *plan, int tiles_per_task, int task, int *deps, int capacity, int *ndeps,
                             int *ntasks)
{
    if (!plan || !ndeps || (capacity > 0 && !deps)) return fail(JACOBI_EINVAL, "NULL argument");
    if (tiles_per_task < 1 || capacity < 0) return fail(JACOBI_EINVAL, "tiles_per_task must be >= 1 and capacity >= 0");
    const int group = tiles_per_task > plan->geo.ntiles ? plan->geo.ntiles : tiles_per_task;
    const int n = (int)ceil_div(plan->geo.ntiles, group);
    if (ntasks) *ntasks = n;
    if (task < 0 || task >= n) return fail(JACOBI_EINVAL, "task index out of range");
    if (plan->task_group != group) build_task_deps(plan, group);
    const std::vector<int> &d = plan->task_deps[task];
    for (int i = 0; i < (int)d.size() && i < capacity; ++i) deps[i] = d[i];
    *ndeps = (int)d.size();
    return JACOBI_OK;
}

int jacobi_pass_schedule(const jacobi_plan *plan, int iters, int *depths, int capacity, int *npasses)
{
    if (!plan || !npasses || (capacity > 0 && !depths)) return fail(JACOBI_EINVAL, "NULL argument");
    if (iters < 0 || capacity < 0) return fail(JACOBI_EINVAL, "iters and capacity must be >= 0");
    int n = 0;
    const ResidentChoice rc = resident_choice(plan, iters);
    if (rc.ok) {
        // one launch; its phases swap the grids like passes do
        for (int ph = 0; ph < rc.nphase; ++ph, ++n)
            if (n < capacity) depths[n] = rc.depth + (ph < rc.n_deep ? 1 : 0);
        *npasses = n;
        return JACOBI_OK;
    }
    for (int k = 0; k < iters;) {
        const PassChoice pc = choose_pass(plan, iters - k);
        if (n < capacity) depths[n] = pc.depth;
        ++n;
        k += pc.depth;
    }
    *npasses = n;
    return JACOBI_OK;
}

int jacobi_sweep_residual(jacobi_plan *plan, void *in, void *out, int iters, void *stream, void **final,
                          double *residual_in_dev)
{
    if (!plan || !in || !out || !residual_in_dev) return fail(JACOBI_EINVAL, "NULL argument");
    if (in == out) return fail(JACOBI_EINVAL, "in and out must be different grids");
    if (misaligned(in) || misaligned(out)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    if (grids_overlap(plan, in, out)) return fail(JACOBI_EINVAL, "in and out overlap");
    if (iters < 1) return fail(JACOBI_EINVAL, "iters must be >= 1");
    if (final) *final = in;
    return sweep_common(plan, in, out, iters, (hipStream_t)stream, final, residual_in_dev);
}

int jacobi_run(jacobi_plan *plan, void *in, void *out, int iters, int residual_every, double *residuals_dev,
               void *stream, void **final)
{
    if (!plan || !in || !out) return fail(JACOBI_EINVAL, "NULL argument");
    if (in == out) return fail(JACOBI_EINVAL, "in and out must be different grids");
    if (misaligned(in) || misaligned(out)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    if (grids_overlap(plan, in, out)) return fail(JACOBI_EINVAL, "in and out overlap");
    if (iters < 0 || residual_every < 0) return fail(JACOBI_EINVAL, "iters and residual_every must be >= 0");
    const int nres = residual_every > 0 ? iters / residual_every : 0;
    if (nres > 0 && !residuals_dev) return fail(JACOBI_EINVAL, "residuals_dev is NULL");
    hipStream_t st = (hipStream_t)stream;
    void *cur = in, *other = out;
    int done = 0, pending = -1;      // pending: index of a residual still owed for the grid in `cur`
    RunCarry carry;                  // blocks after the first start from what the one before left in the grids
    while (done < iters) {
        const int n = std::min(residual_every > 0 ? residual_every : iters, iters - done);
        const bool norm_due = residual_every > 0 && (done + n) % residual_every == 0;
        const int k = norm_due ? (done + n) / residual_every - 1 : -1;
        // The norm of the grid a block produces comes from the block's own launch if that is the one-launch
        // kernel, else from inside the first update of the next block; the last block's from the stand-alone pass.
        const bool in_launch = norm_due && resident_choice(plan, n, true).ok;
        const bool stand_alone = norm_due && !in_launch && done + n == iters;
        void *fin = cur;
        int rc = sweep_common(plan, cur, other, n, st, &fin, pending >= 0 ? residuals_dev + pending : nullptr, &carry,
                              in_launch || stand_alone ? residuals_dev + k : nullptr);
        if (rc) return rc;
        pending = norm_due && !in_launch && !stand_alone ? k : -1;
        if (fin != cur) std::swap(cur, other);
        done += n;
    }
    if (final) *final = cur;
    return JACOBI_OK;
}

int residual_norm(jacobi_plan *plan, void *grid, double *result_dev, void *stream)
{
    if (!plan || !grid || !result_dev) return fail(JACOBI_EINVAL, "NULL argument");
    if (misaligned(grid)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    return residual_common(plan, grid, result_dev, (hipStream_t)stream);
}

// ---- residual_norm_noalloc: the partial sums live in an array of the library's own device image ----
// Every GPU that loads the library holds its own copy of `scratch` at its own address.  In host code the
// name is only a handle for hipGetSymbolAddress; the device address it yields (looked up once per device,
// with that device current) is what the kernels are given.
static __device__ __align__(256) double scratch[JACOBI_NOALLOC_MAX_PARTIALS];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_lock;
double *g_scratch_ptr[MAX_DEVICES];     // device address of `scratch` on each device; nullptr: not looked up yet

int static_scratch_of_current_device(double **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(JACOBI_EINVAL, "device ordinal beyond the 64 the library keeps scratch addresses for");
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(JACOBI_EHIP, "hipGetSymbolAddress returned no address for the static scratch");
        g_scratch_ptr[dev] = (double *)ptr;
    }
    *out = g_scratch_ptr[dev];
    return JACOBI_OK;
}
}  // namespace

int residual_norm_noalloc(jacobi_plan *plan, void *grid, double *result_dev, void *stream)
{
    if (!plan || !grid || !result_dev) return fail(JACOBI_EINVAL, "NULL argument");
    if (misaligned(grid)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    const int64_t nwg = single_step_workgroups(plan, jk::MODE_RESIDUAL);
    if (nwg > JACOBI_NOALLOC_MAX_PARTIALS) {
        char msg[160];
        snprintf(msg, sizeof(msg), "residual_norm_noalloc: the plan's residual launch has %lld workgroups, the static "
                 "scratch holds %d partial sums", (long long)nwg, JACOBI_NOALLOC_MAX_PARTIALS);
        return fail(JACOBI_EINVAL, msg);
    }
    double *partials = nullptr;
    if (int rc = static_scratch_of_current_device(&partials)) return rc;
    return residual_launches(plan, grid, partials, result_dev, (hipStream_t)stream);
}

int residual_norm_host(jacobi_plan *plan, void *grid, double *result_host, void *stream)
{
    if (!plan || !grid || !result_host) return fail(JACOBI_EINVAL, "NULL argument");
    if (misaligned(grid)) return fail(JACOBI_EINVAL, "grids must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    int rc = residual_common(plan, grid, nullptr, st);
    if (rc) return rc;
    HIP_TRY(hipMemcpyAsync(result_host, plan->partial + plan->partial_cap - 1, sizeof(double), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    return JACOBI_OK;
}

int jacobi_set_option(jacobi_plan *plan, const char *key, int64_t value)
{
    if (!plan || !key) return fail(JACOBI_EINVAL, "NULL argument");
    const OptionSpec *o = find_option(key);
    if (!o) return fail(JACOBI_EINVAL, "unknown option");
    bool ok = value >= o->lo && value <= o->hi;
    if (ok && value != 0 && o->only[0] != 0) {
        ok = false;
        for (int64_t allowed : o->only) ok = ok || (allowed != 0 && value == allowed);
    }
    if (!ok) {
        std::string msg = std::string("option ") + key + ": value out of range (" + std::to_string(o->lo) + ".." +
                          std::to_string(o->hi);
        if (o->only[0] != 0) {
            msg += "; 0";
            for (int64_t allowed : o->only)
                if (allowed != 0) msg += ", " + std::to_string(allowed);
            msg += " only";
        }
        return fail(JACOBI_EINVAL, (msg + ")").c_str());
    }
    plan->*(o->field) = value;
    return JACOBI_OK;
}

int jacobi_get_option(const jacobi_plan *plan, const char *key, int64_t *value)
{
    if (!plan || !key || !value) return fail(JACOBI_EINVAL, "NULL argument");
    // read-only figures
    if (!strcmp(key, "lds_limit_failed")) { *value = plan->lds_limit_failed; return JACOBI_OK; }
    if (!strcmp(key, "lds_request_1")) { *value = lds_to_limit_workgroups(plan, 1); return JACOBI_OK; }
    if (!strcmp(key, "lds_request_2")) { *value = lds_to_limit_workgroups(plan, 2); return JACOBI_OK; }
    if (!strcmp(key, "num_cu")) { *value = plan->num_cu; return JACOBI_OK; }
    // what the single-step launches will run with under the current options: "update_..." for the update,
    // "residual_..." for the stand-alone residual pass (the strip-per-wavefront kernel)
    for (const char *prefix : {"update_", "residual_"}) {
        const size_t n = strlen(prefix);
        if (strncmp(key, prefix, n)) continue;
        const int mode = prefix[0] == 'u' ? jk::MODE_UPDATE : jk::MODE_RESIDUAL;
        const SweepConfig c = make_config(plan, mode);
        const char *what = key + n;
        if (!strcmp(what, "rows_per_strip")) { *value = c.sp.R; return JACOBI_OK; }
        if (!strcmp(what, "rows_per_wave")) { *value = c.rows_per_wave; return JACOBI_OK; }
        if (!strcmp(what, "unroll")) { *value = c.unroll; return JACOBI_OK; }
        if (!strcmp(what, "xcd_chunk")) { *value = c.sp.xcd_chunk; return JACOBI_OK; }
        if (!strcmp(what, "strips")) { *value = c.sp.nstrips; return JACOBI_OK; }
        if (!strcmp(what, "one_workgroup_per_cu")) { *value = c.whole_cu ? 1 : 0; return JACOBI_OK; }
        if (!strcmp(what, "streaming_stores")) { *value = store_flavour(plan) == 2 ? 1 : 0; return JACOBI_OK; }
        return fail(JACOBI_EINVAL, "unknown option");
    }
    const OptionSpec *o = find_option(key);
    if (!o) return fail(JACOBI_EINVAL, "unknown option");
    *value = plan->*(o->field);
    return JACOBI_OK;
}

int jacobi_stream_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src) return fail(JACOBI_EINVAL, "NULL argument");
    if (bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16) return fail(JACOBI_EINVAL, "bytes and pointers must be multiples of 16");
    if (bytes == 0) return JACOBI_OK;
    const long long n16 = (long long)(bytes / 16);
    const long long nblk = (n16 + jk::WG - 1) / jk::WG;
    if (nblk > 0x7fffffffLL) return fail(JACOBI_EINVAL, "copy too large for one launch");
    hipLaunchKernelGGL(jk::stream_copy_kernel, dim3((unsigned)nblk), dim3(jk::WG), 0, (hipStream_t)stream,
                       (const uint4 *)src, (uint4 *)dst, n16);
    HIP_TRY(hipGetLastError());
    return JACOBI_OK;
}

int jacobi_profile_read(jacobi_plan *plan, double *update_ms_total, int64_t *update_launches)
{
    if (!plan || !update_ms_total || !update_launches) return fail(JACOBI_EINVAL, "NULL argument");
    double tot = 0.0;
    for (int64_t i = 0; i < plan->ev_used; ++i) {
        HIP_TRY(hipEventSynchronize(plan->ev[2 * i + 1]));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, plan->ev[2 * i], plan->ev[2 * i + 1]));
        tot += ms;
    }
    *update_ms_total = tot;
    *update_launches = plan->ev_used;
    plan->ev_used = 0;
    return JACOBI_OK;
}

}  // extern "C"
