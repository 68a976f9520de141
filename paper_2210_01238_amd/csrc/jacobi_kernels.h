// Device code for the block-decomposed Jacobi iteration (paper Sec. VI-C) on gfx950.
//
// Work decomposition.  The paper's unit of work is a block (tile) = one task; on one
// MI355X a tile is far too coarse (and, with thousands of small tiles, too fine) to be
// a launch, so every kernel here covers ALL tiles in one launch and splits each tile
// into "strips": a strip is the part of a tile one 64-lane wavefront marches through,
//   2-D: 64*NV consecutive columns x R consecutive rows,
//   3-D: 64*NV consecutive columns of one row x R consecutive planes,
// with NV elements (16 bytes) per lane, so every wavefront load/store is one contiguous,
// 16-byte-per-lane, cache-line-aligned 1 KiB access.  The marching direction keeps the
// previous/current/next row (plane) in registers, so the two neighbours along it cost
// no memory traffic; the x neighbours come from the adjacent lanes through DPP wave
// shifts (plain VALU moves) and, at the two ends of the wavefront, from a small gather load
// (the neighbouring strip's cell or the tile's dense x-halo array).
//
// Workgroups (4 wavefronts = 4 consecutive strips) walk the strip list, which is in memory
// order, so the chip as a whole streams through the grid front to back; see
// xcd_logical_wg() for how runs of workgroups are pinned to one XCD's L2.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

namespace jk {

constexpr int WAVE = 64;
constexpr int WAVES_PER_WG = 4;
constexpr int WG = WAVE * WAVES_PER_WG;
constexpr int NUM_XCD = 8;
constexpr int NUM_CU = 256;         // compute units of the chip

// Geometry of a plan, passed to kernels by value.
struct Geo {
    int ndim;
    int Tz, Ty, Tx;   // tile counts
    int td, th, tw;   // tile interior extents (td = 1 in 2-D)
    int rows;         // th + 2
    int nplanes;      // td + 2 (3-D) or 1 (2-D)
    int z0;           // index of the first interior plane: 1 (3-D) or 0 (2-D)
    int pitch;        // elements per row, multiple of 128 bytes
    int ntiles;
    long long plane;        // rows * pitch
    long long xoff;         // x- halo array offset inside a tile
    long long hpitch;       // x- -> x+ halo array distance
    long long xsend;        // x send arrays (packed copies of the tile's own first / last column), hpitch apart
    long long tile_stride;  // elements per tile
};

__device__ __forceinline__ long long main_off(const Geo &g, int k, int i, int c)
{
    return ((long long)k * g.rows + i) * g.pitch + c;
}
__device__ __forceinline__ long long xm_off(const Geo &g, int k, int i)
{
    return g.xoff + (long long)k * g.rows + i;
}
__device__ __forceinline__ long long xp_off(const Geo &g, int k, int i)
{
    return g.xoff + g.hpitch + (long long)k * g.rows + i;
}

template <typename T> struct Vec;
template <> struct Vec<double> {
    static constexpr int N = 2;
    typedef double type __attribute__((ext_vector_type(2)));
};
template <> struct Vec<float> {
    static constexpr int N = 4;
    typedef float type __attribute__((ext_vector_type(4)));
};

template <typename T> struct Coef;
template <> struct Coef<double> {
    static constexpr double quarter = 0.25, sixth = 1.0 / 6.0, four = 4.0, six = 6.0;
};
template <> struct Coef<float> {
    static constexpr float quarter = 0.25f, sixth = 1.0f / 6.0f, four = 4.0f, six = 6.0f;
};

template <bool NT, typename V> __device__ __forceinline__ V ldv(const V *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename V> __device__ __forceinline__ void stv(V *p, V v)
{
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// ---- buffer stores ----------------------------------------------------------------
// A store through a buffer descriptor (base, size in bytes) with a per-lane byte offset: the
// hardware drops every lane whose offset lies beyond the size.  A pipelined loop can therefore
// issue exactly one store per step, whoever has something to store (lanes and steps that have
// not are given BUF_SKIP), and the compiler can count the outstanding memory operations: with
// stores inside branches it cannot, and every wait for a prefetched row then also waits for the
// stores issued after that row's load.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr unsigned BUF_SKIP = 0x80000000u;          // beyond any buffer used here (sizes stay below 2 GiB)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(void *base, unsigned bytes)
{
    // 4th descriptor word: raw 32-bit data format, no swizzle, offsets checked against the size
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)bytes, 0x00020000);
}
template <typename V>
__device__ __forceinline__ void buffer_store_stream(V v, __amdgpu_buffer_rsrc_t buf, unsigned byte_offset)
{
    static_assert(sizeof(V) == 16, "one 16-byte vector per lane");
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), buf, (int)byte_offset, 0, 2 /* streaming */);
}
// The same with a second, wave-uniform offset (on this chip it counts towards the checked offset like the
// per-lane one: measured); 16 or 8 bytes per lane.  Loads of lanes beyond the size return zero.
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
template <typename V>
__device__ __forceinline__ V buffer_load(__amdgpu_buffer_rsrc_t buf, unsigned byte_offset, unsigned row_offset)
{
    static_assert(sizeof(V) == 16 || sizeof(V) == 8, "8 or 16 bytes per lane");
    if constexpr (sizeof(V) == 16)
        return __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b128(buf, (int)byte_offset, (int)row_offset, 0));
    else
        return __builtin_bit_cast(V, __builtin_amdgcn_raw_buffer_load_b64(buf, (int)byte_offset, (int)row_offset, 0));
}
template <bool STREAM, typename V>
__device__ __forceinline__ void buffer_store(V v, __amdgpu_buffer_rsrc_t buf, unsigned byte_offset, unsigned row_offset)
{
    static_assert(sizeof(V) == 16 || sizeof(V) == 8, "8 or 16 bytes per lane");
    if constexpr (sizeof(V) == 16)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), buf, (int)byte_offset, (int)row_offset, STREAM ? 2 : 0);
    else
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), buf, (int)byte_offset, (int)row_offset, STREAM ? 2 : 0);
}

// ---- cross-lane moves -------------------------------------------------------------
// DPP wave shifts (full-rate VALU moves, no LDS traffic): lane i receives the value of
// lane i-1 (wave_shr:1) or lane i+1 (wave_shl:1); the lane at the open end keeps `fill`.
__device__ __forceinline__ int dpp_from_prev(int v, int fill)
{
    return __builtin_amdgcn_update_dpp(fill, v, 0x138 /* wave_shr:1 */, 0xf, 0xf, false);
}
__device__ __forceinline__ int dpp_from_next(int v, int fill)
{
    return __builtin_amdgcn_update_dpp(fill, v, 0x130 /* wave_shl:1 */, 0xf, 0xf, false);
}
// Same moves with the hardware's own zero fill for the lane that has no source (no fill register).
__device__ __forceinline__ int dpp_from_prev_z(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x138 /* wave_shr:1 */, 0xf, 0xf, true);
}
__device__ __forceinline__ int dpp_from_next_z(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, 0x130 /* wave_shl:1 */, 0xf, 0xf, true);
}
struct Int2 { int lo, hi; };
__device__ __forceinline__ float from_prev_lane(float v, float fill)
{
    return __builtin_bit_cast(float, dpp_from_prev(__builtin_bit_cast(int, v), __builtin_bit_cast(int, fill)));
}
__device__ __forceinline__ float from_next_lane(float v, float fill)
{
    return __builtin_bit_cast(float, dpp_from_next(__builtin_bit_cast(int, v), __builtin_bit_cast(int, fill)));
}
__device__ __forceinline__ double from_prev_lane(double v, double fill)
{
    const Int2 a = __builtin_bit_cast(Int2, v), f = __builtin_bit_cast(Int2, fill);
    const Int2 r = {dpp_from_prev(a.lo, f.lo), dpp_from_prev(a.hi, f.hi)};
    return __builtin_bit_cast(double, r);
}
__device__ __forceinline__ double from_next_lane(double v, double fill)
{
    const Int2 a = __builtin_bit_cast(Int2, v), f = __builtin_bit_cast(Int2, fill);
    const Int2 r = {dpp_from_next(a.lo, f.lo), dpp_from_next(a.hi, f.hi)};
    return __builtin_bit_cast(double, r);
}
__device__ __forceinline__ float from_prev_lane_or_zero(float v)
{
    return __builtin_bit_cast(float, dpp_from_prev_z(__builtin_bit_cast(int, v)));
}
__device__ __forceinline__ float from_next_lane_or_zero(float v)
{
    return __builtin_bit_cast(float, dpp_from_next_z(__builtin_bit_cast(int, v)));
}
__device__ __forceinline__ double from_prev_lane_or_zero(double v)
{
    const Int2 a = __builtin_bit_cast(Int2, v);
    const Int2 r = {dpp_from_prev_z(a.lo), dpp_from_prev_z(a.hi)};
    return __builtin_bit_cast(double, r);
}
__device__ __forceinline__ double from_next_lane_or_zero(double v)
{
    const Int2 a = __builtin_bit_cast(Int2, v);
    const Int2 r = {dpp_from_next_z(a.lo), dpp_from_next_z(a.hi)};
    return __builtin_bit_cast(double, r);
}
// Value held by lane `l` (a compile-time constant after unrolling), as a wave-uniform scalar.
__device__ __forceinline__ float lane_value(float v, int l)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ double lane_value(double v, int l)
{
    const Int2 a = __builtin_bit_cast(Int2, v);
    const Int2 r = {__builtin_amdgcn_readlane(a.lo, l), __builtin_amdgcn_readlane(a.hi, l)};
    return __builtin_bit_cast(double, r);
}

// Workgroup renumbering.  The hardware hands consecutive workgroup ids to the 8 XCDs
// round-robin, and each XCD has its own L2.  Strips that are neighbours in a tile re-read each
// other's border rows, which only hits in L2 if both run on the same XCD; on the other hand HBM
// is fastest when the whole chip walks through memory as one compact front.  Compromise: cut
// the strip list into groups of 8*G workgroups; inside a group XCD x takes the G consecutive
// logical ids [x*G, (x+1)*G).  G = 1 is the identity (one front, no L2 sharing); a large G gives
// every XCD a long private run (8 fronts).  The tail that does not fill a group is left as is.
__device__ __forceinline__ long long xcd_logical_wg(int G)
{
    const long long b = blockIdx.x;
    if (G <= 1) return b;
    const long long span = (long long)NUM_XCD * G;
    const long long full = ((long long)gridDim.x / span) * span;
    if (b >= full) return b;
    const long long grp = b / span, within = b - grp * span;
    return grp * span + (within % NUM_XCD) * G + within / NUM_XCD;
}

// Sum over the 64 lanes in a fixed butterfly order (same bits on every run).
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, WAVE);
    return v;
}

// Workgroup sum: wavefront shuffle tree -> one LDS slot per wavefront -> fixed-order add.
// Every thread of the workgroup must call it; the result is valid in thread 0.
__device__ __forceinline__ double wg_sum(double v, double *lds /* WAVES_PER_WG (or more) slots */)
{
    const int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
    v = wave_sum(v);
    if (lane == 0) lds[wave] = v;
    __syncthreads();
    double s = 0.0;
    if (threadIdx.x == 0) {
        const int nw = blockDim.x / WAVE;
        for (int w = 0; w < nw; ++w) s += lds[w];
    }
    return s;
}

// MODE_BOTH: update, and in the same pass the residual of the SOURCE grid (its terms need
// exactly the values the update already holds in registers).
enum Mode { MODE_UPDATE = 0, MODE_RESIDUAL = 1, MODE_BOTH = 2 };

// What an update does with a tile's fresh edge cells besides storing them in place.  PUSH: writes them into the
// face neighbours' halo cells of the destination grid (pack, transfer and unpack in the update's epilogue).
// PACK: writes the first / last column into the tile's own dense x send arrays (the paper's "pack into a
// contiguous message buffer", Sec. VI-C; rows and planes are contiguous already), from which the stand-alone
// exchange kernel then copies instead of gathering one cell per cache line.
enum Fused { FUSED_NONE = 0, FUSED_PUSH = 1, FUSED_PACK = 2 };

struct StripParams {
    int R;               // rows (2-D) / planes (3-D) per strip
    int nseg;            // column segments per row = ceil(pitch / (64*NV))
    int nblk;            // strips along the marching direction = ceil(extent / R)
    long long nstrips;   // total
    int fused;           // update mode: 1 = push edge cells into the neighbours' halo cells of dst (FUSED_PUSH),
                         // 2 = pack the x edge cells into the tile's own send arrays of dst (FUSED_PACK)
    int xcd_chunk;       // G of xcd_logical_wg(): consecutive workgroups one XCD takes
    int rows_fastest = 0; // 3-D blocked passes: consecutive strips are neighbours in y (else in x)
    int tile0 = 0;        // single-step kernels: first tile this launch covers (a task = a range of tiles)
    int pull = 0;         // single-step kernels: run the variant that reads the cells beyond a tile from the neighbouring
                          // tiles' edge cells instead of the tile's halo cells (which may then be stale: no exchange
                          // needed); the stand-alone residual pass always does
};

// ------------------------------------------------------------------------------------
// 2-D: 5-point update (or residual) of every tile.  new = 0.25*((W+E)+(S+N)).
// ------------------------------------------------------------------------------------
// PULL: cells beyond a tile are read from the neighbouring tiles' edge cells instead of the tile's halo cells (a
// compile-time switch: as a run-time one its address selects cost the steady-state update 5-7 %).
template <typename T, int MODE, int U, int NT, bool PULL>
__global__ __launch_bounds__(WG) void sweep2d_kernel(Geo g, StripParams sp,
                                                     const T *__restrict__ src, T *__restrict__ dst,
                                                     double *__restrict__ partial)
{
    using V = typename Vec<T>::type;
    constexpr int NV = Vec<T>::N;
    __shared__ double red[WAVES_PER_WG];

    const int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
    const long long lwg = xcd_logical_wg(sp.xcd_chunk);
    const long long s = lwg * WAVES_PER_WG + wave;
    double acc = 0.0;

    if (s < sp.nstrips) {
        const int per_tile = sp.nblk * sp.nseg;
        const int tl = (int)(s / per_tile);                       // tile within this launch
        const int rem = (int)(s - (long long)tl * per_tile);
        const int t = sp.tile0 + tl;
        const int rb = rem / sp.nseg, seg = rem - rb * sp.nseg;
        const int ty = t / g.Tx, tx = t - ty * g.Tx;
        const int r0 = 1 + rb * sp.R;
        const int r1 = min(g.th, r0 + sp.R - 1);
        const int col0 = (seg * WAVE + lane) * NV;
        const bool active = col0 < g.pitch;   // pitch is a multiple of NV: no straddling
        const int last = g.tw - 1;
        const bool has_last = active && col0 <= last && last < col0 + NV;
        const int jlast = last - col0;
        // x-edge cells of the wavefront: left of its first column (the x- halo for segment 0) and
        // right of its last column (the x+ halo if the tile ends inside this segment)
        const int seg_c0 = seg * WAVE * NV;
        const bool seg_has_last = seg_c0 <= last && last < seg_c0 + WAVE * NV;
        const bool w_halo = seg_c0 == 0;
        const int e_col = seg_c0 + WAVE * NV;
        const bool e_in_row = e_col < g.pitch;
        const T *tsrc = src + (long long)t * g.tile_stride;
        T *tdst = dst + (long long)t * g.tile_stride;
        // Pull mode: a cell beyond the tile is read from the neighbouring tile's edge (row th of the tile above
        // for halo row 0, row 1 of the tile below for halo row th+1, the last / first column of the tile to the
        // left / right for the x halos); on the domain boundary the halo cell holds the Dirichlet value as ever.
        const long long ystep = (long long)g.Tx * g.tile_stride;
        const bool pull_ym = PULL && ty > 0, pull_yp = PULL && ty < g.Ty - 1;
        const bool pull_xm = PULL && tx > 0, pull_xp = PULL && tx < g.Tx - 1;
        // first cell of row `row` (0 .. th+1) as this strip has to read it
        auto row_ptr = [&](int row) -> const T * {
            if (row == 0 && pull_ym) return tsrc - ystep + main_off(g, 0, g.th, 0);
            if (row == g.th + 1 && pull_yp) return tsrc + ystep + main_off(g, 0, 1, 0);
            return tsrc + main_off(g, 0, row, 0);
        };
        // where this strip's edge cells go besides their own place: the neighbour tiles' halo cells of dst
        // (push), or for the x edges the tile's own send arrays (pack); x targets are indexed by the row
        const bool push = MODE != MODE_RESIDUAL && sp.fused == FUSED_PUSH;
        const bool xcopy = MODE != MODE_RESIDUAL && sp.fused != FUSED_NONE;
        T *dst_ym = (push && ty > 0) ? tdst - (long long)g.Tx * g.tile_stride : nullptr;
        T *dst_yp = (push && ty < g.Ty - 1) ? tdst + (long long)g.Tx * g.tile_stride : nullptr;
        T *dst_xm = (xcopy && tx > 0 && col0 == 0 && active)
                        ? (push ? tdst - g.tile_stride + g.xoff + g.hpitch : tdst + g.xsend) : nullptr;
        T *dst_xp = (xcopy && tx < g.Tx - 1 && has_last)
                        ? (push ? tdst + g.tile_stride + g.xoff : tdst + g.xsend + g.hpitch) : nullptr;

        V prev = V(0), cur = V(0);
        if (active) {
            prev = ldv<(NT & 1) != 0>((const V *)(row_ptr(r0 - 1) + col0));
            cur = ldv<(NT & 1) != 0>((const V *)(row_ptr(r0) + col0));
        }
        for (int r = r0; r <= r1; r += U) {
            V nx[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int rn = min(r + u + 1, g.th + 1);   // clamped: stays inside the tile
                nx[u] = active ? ldv<(NT & 1) != 0>((const V *)(row_ptr(rn) + col0)) : V(0);
            }
            // One gather load fetches every x-edge cell of this group of rows.  It is issued LAST on
            // purpose: the first row then cannot be finished before all row loads have landed, so a
            // wavefront reads its whole strip, then writes its whole strip.  Letting rows be stored
            // as they arrive interleaves reads and writes at the memory and measures 3 % slower.
            // lane l < U -> W edge of row r+l, lane 32+l -> E edge of row r+l
            T edge = T(0);
            {
                const int el = lane & 31;
                if (el < U) {
                    const int rc = min(r + el, g.th + 1);
                    if (lane < 32)
                        edge = !w_halo ? tsrc[main_off(g, 0, rc, seg_c0 - 1)]
                               : pull_xm ? tsrc[main_off(g, 0, rc, g.tw - 1) - g.tile_stride] : tsrc[xm_off(g, 0, rc)];
                    else if (seg_has_last)
                        edge = pull_xp ? tsrc[main_off(g, 0, rc, 0) + g.tile_stride] : tsrc[xp_off(g, 0, rc)];
                    else if (e_in_row) edge = tsrc[main_off(g, 0, rc, e_col)];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int rr = r + u;
                const T ew = lane_value(edge, u), ee = lane_value(edge, 32 + u);
                const T left = from_prev_lane(cur[NV - 1], ew);    // lane 0 keeps the W edge
                const T right = from_next_lane(cur[0], ee);        // lane 63 keeps the E edge
                if (rr <= r1) {
                    V out;
#pragma unroll
                    for (int j = 0; j < NV; ++j) {
                        const T w = j == 0 ? left : cur[j - 1];
                        T e = j == NV - 1 ? right : cur[j + 1];
                        if (has_last && j == jlast) e = ee;
                        const T we = w + e;
                        const T sn = prev[j] + nx[u][j];
                        if constexpr (MODE != MODE_RESIDUAL) out[j] = Coef<T>::quarter * (we + sn);
                        if constexpr (MODE != MODE_UPDATE) {
                            const T res = (we + sn) - Coef<T>::four * cur[j];
                            const double rd = (double)res;
                            if (col0 + j <= last) acc += rd * rd;
                        }
                    }
                    if constexpr (MODE != MODE_RESIDUAL) {
                        if (active) {
                            stv<(NT & 2) != 0>((V *)(tdst + main_off(g, 0, rr, col0)), out);
                            if (xcopy) {
                                if (rr == 1 && dst_ym) *(V *)(dst_ym + main_off(g, 0, g.th + 1, col0)) = out;
                                if (rr == g.th && dst_yp) *(V *)(dst_yp + main_off(g, 0, 0, col0)) = out;
                                if (dst_xm) dst_xm[rr] = out[0];
                                if (dst_xp) dst_xp[rr] = out[jlast];
                            }
                        }
                    }
                }
                prev = cur;
                cur = nx[u];
            }
        }
    }
    if constexpr (MODE != MODE_UPDATE) {
        const double tot = wg_sum(acc, red);
        if (threadIdx.x == 0) partial[lwg] = tot;
    }
}

// ------------------------------------------------------------------------------------
// 2-D stand-alone residual pass, wavefronts of a workgroup STACKED: the NW wavefronts of a workgroup take NW
// consecutive R-row strips of the same 64*NV columns, and the row just above / below a wavefront's strip - the
// last / first row of its neighbour in the workgroup - comes through LDS instead of being loaded again.  A
// workgroup then reads R*NW + 2 rows for R*NW rows (sweep2d_kernel: R + 2 for R; the two extra rows are the
// neighbouring strips' and only come from cache if those run on the same XCD at the same time).  For the
// read-only pass this is worth 6-12 % (16384^2: 369 -> 346 us, 128^2 tiles: 107 -> 94 us); the UPDATE was built
// the same way and ran 4 % slower than with independent wavefronts (the barrier makes four wavefronts read, then
// four write), so it keeps sweep2d_kernel.  Always pulls: cells beyond a tile are read from the neighbouring
// tiles' edge cells (see sweep2d_kernel).  Work unit = (tile, band of R*NW rows, column segment), one workgroup
// each: every wavefront reaches the barrier; a wavefront whose rows lie beyond the tile (ragged last band)
// loads clamped rows and adds nothing.  Same terms as everywhere; one partial sum per workgroup.
// ------------------------------------------------------------------------------------
template <typename T, int R, int NW>
__global__ __launch_bounds__(NW * WAVE) void residual2d_stack_kernel(Geo g, StripParams sp, const T *__restrict__ src,
                                                                     double *__restrict__ partial)
{
    using V = typename Vec<T>::type;
    constexpr int NV = Vec<T>::N;
    static_assert(R >= 1 && R <= 32, "the edge gather gives each side 32 lanes");
    __shared__ V xrow[NW][2][WAVE];           // [wavefront][its first / last row][lane]
    __shared__ double red[NW];

    const int lane = threadIdx.x % WAVE;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const long long lwg = xcd_logical_wg(sp.xcd_chunk);        // the work unit: the grid has exactly one workgroup each
    double acc = 0.0;

    const int per_tile = sp.nblk * sp.nseg;                    // sp.nblk: bands per tile
    const int t = (int)(lwg / per_tile);
    const int rem = (int)(lwg - (long long)t * per_tile);
    const int band = rem / sp.nseg, seg = rem - band * sp.nseg;
    const int ty = t / g.Tx, tx = t - ty * g.Tx;
    const int r0 = 1 + (band * NW + wave) * R;                 // may lie beyond the tile (ragged last band)
    const int r1 = min(g.th, r0 + R - 1);
    const int col0 = (seg * WAVE + lane) * NV;
    const bool active = col0 < g.pitch;
    const int last = g.tw - 1;
    const bool has_last = active && col0 <= last && last < col0 + NV;
    const int jlast = last - col0;
    const int seg_c0 = seg * WAVE * NV;
    const bool seg_has_last = seg_c0 <= last && last < seg_c0 + WAVE * NV;
    const bool w_halo = seg_c0 == 0;
    const int e_col = seg_c0 + WAVE * NV;
    const bool e_in_row = e_col < g.pitch;
    const T *tsrc = src + (long long)t * g.tile_stride;
    const long long ystep = (long long)g.Tx * g.tile_stride;
    const bool pull_ym = ty > 0, pull_yp = ty < g.Ty - 1, pull_xm = tx > 0, pull_xp = tx < g.Tx - 1;
    // first cell of row `row` (clamped to 0 .. th+1) as it has to be read: halo rows from the tiles above / below
    auto row_ptr = [&](int row) -> const T * {
        row = min(row, g.th + 1);
        if (row == 0 && pull_ym) return tsrc - ystep + main_off(g, 0, g.th, 0);
        if (row == g.th + 1 && pull_yp) return tsrc + ystep + main_off(g, 0, 1, 0);
        return tsrc + main_off(g, 0, row, 0);
    };

    // rows r0-1 .. r0+R: index 0 and R+1 are the neighbours' (LDS, or memory at the ends of the band)
    V row[R + 2];
#pragma unroll
    for (int q = 1; q <= R; ++q) row[q] = active ? *(const V *)(row_ptr(r0 + q - 1) + col0) : V(0);
    row[0] = V(0);
    row[R + 1] = V(0);
    if (wave == 0 && active) row[0] = *(const V *)(row_ptr(r0 - 1) + col0);
    if (wave == NW - 1 && active) row[R + 1] = *(const V *)(row_ptr(r0 + R) + col0);
    // the x-edge cells of the strip: lane l < R -> W edge of row r0+l, lane 32+l -> E edge
    T edge = T(0);
    {
        const int el = lane & 31;
        if (el < R) {
            const int rc = min(r0 + el, g.th + 1);
            if (lane < 32)
                edge = !w_halo ? tsrc[main_off(g, 0, rc, seg_c0 - 1)]
                       : pull_xm ? tsrc[main_off(g, 0, rc, g.tw - 1) - g.tile_stride] : tsrc[xm_off(g, 0, rc)];
            else if (seg_has_last)
                edge = pull_xp ? tsrc[main_off(g, 0, rc, 0) + g.tile_stride] : tsrc[xp_off(g, 0, rc)];
            else if (e_in_row) edge = tsrc[main_off(g, 0, rc, e_col)];
        }
    }
    xrow[wave][0][lane] = row[1];
    xrow[wave][1][lane] = row[R];
    __syncthreads();
    if (wave > 0) row[0] = xrow[wave > 0 ? wave - 1 : 0][1][lane];
    if (wave < NW - 1) row[R + 1] = xrow[wave < NW - 1 ? wave + 1 : wave][0][lane];

#pragma unroll
    for (int u = 0; u < R; ++u) {
        const V prev = row[u], cur = row[u + 1], nxt = row[u + 2];
        const T ew = lane_value(edge, u), ee = lane_value(edge, 32 + u);
        const T left = from_prev_lane(cur[NV - 1], ew);    // lane 0 keeps the W edge
        const T right = from_next_lane(cur[0], ee);        // lane 63 keeps the E edge
        if (r0 + u <= r1) {
#pragma unroll
            for (int j = 0; j < NV; ++j) {
                const T w = j == 0 ? left : cur[j - 1];
                T e = j == NV - 1 ? right : cur[j + 1];
                if (has_last && j == jlast) e = ee;
                const T we = w + e;
                const T sn = prev[j] + nxt[j];
                const T res = (we + sn) - Coef<T>::four * cur[j];
                const double rd = (double)res;
                if (col0 + j <= last) acc += rd * rd;
            }
        }
    }
    const double tot = wg_sum(acc, red);
    if (threadIdx.x == 0) partial[lwg] = tot;
}

// ------------------------------------------------------------------------------------
// 2-D, two time steps per pass over memory (temporal blocking, T = 2).
//
// A strip produces RT rows x 64*NV columns of u(t+2).  It needs u(t) on RT+4 rows and 2 more
// columns on either side, and computes u(t+1) on RT+2 rows and 1 more column on either side
// (the rim is recomputed by the neighbouring strips: redundant arithmetic instead of memory
// traffic).  Cells outside the tile are read straight from the neighbouring tiles' interiors
// (including the diagonal ones), so this kernel neither needs nor refreshes inter-tile halos:
// the depth-2 "exchange" is folded into its loads.  Dirichlet ring cells are read from the
// boundary tiles' halo cells and are constant in time, so u(t+1) on the ring is the ring.
// Every u(t+1) and u(t+2) value is formed by the same expression as in the single-step
// kernel, so the result is bit-identical to two single steps.
//
// The 2*(RT+4) + 2*(RT+2) cells beside the wavefront's columns come from ONE gather load:
// lanes 0-15 column c0-1, lanes 16-31 column c0-2, lanes 32-47 the column right of the
// wavefront (or of the tile's last column), lanes 48-63 the one after it; lane offset = row.
// The u(t+1) value in the column just outside the wavefront ("ghost") is a wave-uniform
// scalar computed from those cells.
// ------------------------------------------------------------------------------------
// Offset of the cell at row rho in [-1, th+2], column c in [-2, tw+1] relative to tile
// (ty, tx), following it into the neighbouring tile or, on the domain boundary, onto the
// Dirichlet halo cell (rows/columns beyond the ring are clamped onto it; they are never used).
// Needs th >= 2 and tw >= 2.
__device__ __forceinline__ long long t2_cell_off(const Geo &g, int ty, int tx, int rho, int c)
{
    int rr = rho, cc = c;
    if (rho <= 0) {
        if (ty > 0) { --ty; rr = g.th + rho; } else rr = 0;
    } else if (rho > g.th) {
        if (ty < g.Ty - 1) { ++ty; rr = rho - g.th; } else rr = g.th + 1;
    }
    if (c < 0) {
        if (tx > 0) { --tx; cc = g.tw + c; } else cc = -1;
    } else if (c >= g.tw) {
        if (tx < g.Tx - 1) { ++tx; cc = c - g.tw; } else cc = g.tw;
    }
    const long long base = ((long long)ty * g.Tx + tx) * g.tile_stride;
    return base + (cc < 0 ? xm_off(g, 0, rr) : cc >= g.tw ? xp_off(g, 0, rr) : main_off(g, 0, rr, cc));
}

template <typename T, int NV> __device__ __forceinline__ T vec_pick(const typename Vec<T>::type &v, int j)
{
    T r = v[0];
#pragma unroll
    for (int q = 1; q < NV; ++q) r = j == q ? v[q] : r;
    return r;
}

template <typename T, int MODE, int RT, int NT>
__global__ __launch_bounds__(WG) void sweep2d_t2_kernel(Geo g, StripParams sp,
                                                        const T *__restrict__ src, T *__restrict__ dst,
                                                        double *__restrict__ partial)
{
    using V = typename Vec<T>::type;
    constexpr int NV = Vec<T>::N;
    static_assert(RT >= 1 && RT + 4 <= 16, "the edge gather gives each column 16 lanes");
    static_assert(MODE != MODE_RESIDUAL, "stand-alone residual uses the single-step kernel");
    __shared__ double red[WAVES_PER_WG];

    const int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
    const long long lwg = xcd_logical_wg(sp.xcd_chunk);
    const long long s = lwg * WAVES_PER_WG + wave;
    double acc = 0.0;

    if (s < sp.nstrips) {
        const int per_tile = sp.nblk * sp.nseg;
        const int t = (int)(s / per_tile);
        const int rem = (int)(s - (long long)t * per_tile);
        const int rb = rem / sp.nseg, seg = rem - rb * sp.nseg;
        const int ty = t / g.Tx, tx = t - ty * g.Tx;
        const int r0 = 1 + rb * RT;
        const int r1 = min(g.th, r0 + RT - 1);
        const int col0 = (seg * WAVE + lane) * NV;
        const bool active = col0 < g.pitch;
        const int last = g.tw - 1;
        const bool has_last = active && col0 <= last && last < col0 + NV;
        const int jlast = last - col0;
        const int seg_c0 = seg * WAVE * NV;
        const bool seg_has_last = seg_c0 <= last && last < seg_c0 + WAVE * NV;
        const int ecol = seg_has_last ? g.tw : seg_c0 + WAVE * NV;   // first column right of our cells
        const bool w_ring = tx == 0 && seg_c0 == 0;                  // column c0-1 is the Dirichlet ring
        const bool e_ring = tx == g.Tx - 1 && seg_has_last;
        // lane / component holding the cell left of column `ecol`
        const int ll = seg_has_last ? (last - seg_c0) / NV : WAVE - 1;
        const int jl = seg_has_last ? (last - seg_c0) % NV : NV - 1;

        // rows r0-2 .. r0+RT+1 of u(t); index q, row rho = r0-2+q (clamped to th+2 for ragged strips)
        auto rho_of = [&](int q) { return min(r0 - 2 + q, g.th + 2); };
        auto ring_row = [&](int rho) { return (rho <= 0 && ty == 0) || (rho > g.th && ty == g.Ty - 1); };

        V in[RT + 4];
#pragma unroll
        for (int q = 0; q < RT + 4; ++q) {
            in[q] = V(0);
            if (active) {
                // same columns, row followed into the tile above / below (column 0 <= col0 < tw region)
                const long long off = t2_cell_off(g, ty, tx, rho_of(q), 0) + col0;
                in[q] = ldv<(NT & 1) != 0>((const V *)(src + off));
            }
        }
        T edge = T(0);
        {
            const int q = lane & 15, grp = lane >> 4;
            const int c = grp == 0 ? seg_c0 - 1 : grp == 1 ? seg_c0 - 2 : grp == 2 ? ecol : ecol + 1;
            const bool unused = (grp == 1 && w_ring) || (grp == 3 && e_ring);
            if (q < RT + 4 && !unused) edge = src[t2_cell_off(g, ty, tx, rho_of(q), c)];
        }

        // u(t+1): rows r0-1 .. r0+RT (index m, row r0-1+m, source index q = m+1), kept in a window of 3
        V mid[RT + 2];
        T gw[RT + 2], ge[RT + 2];
#pragma unroll
        for (int m = 0; m < RT + 2; ++m) {
            const int q = m + 1;
            const int rho = r0 - 1 + m;
            const T w1 = lane_value(edge, q), e1 = lane_value(edge, 32 + q);
            if (ring_row(min(rho, g.th + 2))) {
                mid[m] = in[q];
                gw[m] = w1;
                ge[m] = e1;
            } else {
                const T left = from_prev_lane(in[q][NV - 1], w1);
                const T right = from_next_lane(in[q][0], e1);
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    const T w = j == 0 ? left : in[q][j - 1];
                    T e = j == NV - 1 ? right : in[q][j + 1];
                    if (has_last && j == jlast) e = e1;
                    const T we = w + e;
                    const T sn = in[q - 1][j] + in[q + 1][j];
                    mid[m][j] = Coef<T>::quarter * (we + sn);
                    if constexpr (MODE == MODE_BOTH) {
                        if (rho >= r0 && rho <= r1 && col0 + j <= last) {
                            const T res = (we + sn) - Coef<T>::four * in[q][j];
                            const double rd = (double)res;
                            acc += rd * rd;
                        }
                    }
                }
                // ghosts: u(t+1) in the columns just left / right of our cells
                const T first = lane_value(in[q][0], 0);
                const T lastv = lane_value(vec_pick<T, NV>(in[q], jl), ll);
                const T w1u = lane_value(edge, q - 1), w1d = lane_value(edge, q + 1);
                const T e1u = lane_value(edge, 32 + q - 1), e1d = lane_value(edge, 32 + q + 1);
                const T w2 = lane_value(edge, 16 + q), e2 = lane_value(edge, 48 + q);
                gw[m] = w_ring ? w1 : Coef<T>::quarter * ((w2 + first) + (w1u + w1d));
                ge[m] = e_ring ? e1 : Coef<T>::quarter * ((lastv + e2) + (e1u + e1d));
            }
            // u(t+2) for row r0+o, o = m-2, as soon as its three u(t+1) rows exist
            if (m >= 2) {
                const int o = m - 2, mm = m - 1;
                const int rr = r0 + o;
                const T left = from_prev_lane(mid[mm][NV - 1], gw[mm]);
                const T right = from_next_lane(mid[mm][0], ge[mm]);
                if (rr <= r1) {
                    V out;
#pragma unroll
                    for (int j = 0; j < NV; ++j) {
                        const T w = j == 0 ? left : mid[mm][j - 1];
                        T e = j == NV - 1 ? right : mid[mm][j + 1];
                        if (has_last && j == jlast) e = ge[mm];
                        out[j] = Coef<T>::quarter * ((w + e) + (mid[mm - 1][j] + mid[mm + 1][j]));
                    }
                    if (active) stv<(NT & 2) != 0>((V *)(dst + (long long)t * g.tile_stride + main_off(g, 0, rr, col0)), out);
                }
            }
        }
    }
    if constexpr (MODE == MODE_BOTH) {
        const double tot = wg_sum(acc, red);
        if (threadIdx.x == 0) partial[lwg] = tot;
    }
}

// ------------------------------------------------------------------------------------
// 2-D, TB time steps per pass over memory (temporal blocking, depths 3..12), pipelined down
// the rows.
//
// Overlapped wavefronts: a wavefront still loads 64 lanes x 16 bytes per row, but only its
// middle 56 lanes (896 bytes = 7 whole cache lines) own output columns; the 4 lanes (64 bytes)
// on either side are ghost lanes that carry the neighbouring columns through the time steps
// and are recomputed by the neighbouring wavefront (a level is valid on one column less per
// side than the level before, so TB <= ghost width).  The 896-byte segments are laid out along
// a whole ROW OF TILES, not per tile, so narrow tiles cost nothing: a wavefront's lanes simply
// address whichever tile their column falls in.  No halo cells are needed or written: rows
// beyond the tile are read from the tiles above / below; Dirichlet ring cells come from the
// boundary tiles' halo cells.
//
// A strip is tall (sp.R rows) and is processed as a software pipeline: every step loads ONE
// new row of u(t) and advances each of the TB levels by one row - level l produces its row
// (rho - l) from the three rows (rho-l-1, rho-l, rho-l+1) of level l-1, the last of which the
// level before has just produced.  Only two rows per level stay in registers (2*TB vectors),
// whatever the strip height, and the only redundant work is the 2*TB-row run-in of a strip.
// Ring cells keep their value by selecting the centre value (the same cell one level down);
// strips that cannot reach a ring cell run a copy of the loop without the selects.  Every
// value is formed by the single-step expression, so a pass is bit-identical to TB single steps.
// Memory operations in the loop are unconditional and counted: one load per row PF rows ahead
// and one buffer store per row (see buffer_store_stream), so the only wait of a trip is for
// its own loads and a trip's stores stay in flight during the next one.
// Needs tw a multiple of the vector width, th >= TB, and a row of tiles smaller than 2 GiB.
// ------------------------------------------------------------------------------------
// Column geometry of a blocked pass of depth TB: every level loses one ghost column per side,
// so at least ceil(TB / vector width) lanes per side are ghosts and the rest own their columns.
// In 2-D, fp64 passes keep 4 ghost lanes at every depth: the owned part of a wavefront's row is
// then 896 bytes = 7 whole cache lines, which measured faster than fewer ghosts and ragged lines;
// 3-D passes measured best with 2.
constexpr int tp_ghost_lanes(int elem_size, int ndim, int depth)
{
    const int nv = 16 / elem_size;
    const int need = (depth + nv - 1) / nv;
    const int least = ndim == 2 ? (elem_size == 8 ? 4 : 2) : 2;
    return need > least ? need : least;
}
template <typename T, int TB, int NDIM> struct TpGeometry {
    static constexpr int NV = Vec<T>::N;
    static constexpr int GHOST_LANES = tp_ghost_lanes((int)sizeof(T), NDIM, TB);
    static constexpr int OWN_LANES = WAVE - 2 * GHOST_LANES;
    static constexpr int SEGW = OWN_LANES * NV;            // columns a wavefront owns
};

// Where a lane of a blocked pass sits along a row of tiles.  A wavefront's 64 lanes cover the columns
// [seg*SEGW - GH, seg*SEGW - GH + 64*NV) counted along the whole row of tiles (0 .. Tx*tw-1; -1 and Tx*tw
// are the Dirichlet ring).  kind: 0 cells of some tile, 1 the W ring cell in the last component, 2 the E
// ring cell in the first component, 3 nothing there.  `bytes` is the per-lane byte offset, the same for
// every row (relative to the row's first cell in the first tile of the row of tiles): the lane's cells,
// or (ring lanes) the place in the first / last tile's x-halo array from which a vector read puts the ring
// value into the component next to the tile cells (a ring lane's other components are never used).
struct TpLane {
    int kind;
    unsigned bytes;
    bool ring_lane;       // kind 1 or 2
    bool wave_has_ring;   // some lane of the wavefront is a ring lane
    bool owner;           // the lane stores its columns (not a ghost lane, and there are cells)
};
template <typename T, int NV, int GL, int SEGW>
__device__ __forceinline__ TpLane tp_lane(const Geo &g, int seg, int lane)
{
    const int wrow = g.Tx * g.tw;
    const int gc = seg * SEGW - GL * NV + lane * NV;
    TpLane L;
    int txx = 0, cc = 0;
    L.kind = 0;
    if (gc < 0) L.kind = gc == -NV ? 1 : 3;
    else if (gc >= wrow) L.kind = gc == wrow ? 2 : 3;
    else { txx = gc / g.tw; cc = gc - txx * g.tw; }
    long long elems = 0;
    if (L.kind == 0) elems = (long long)txx * g.tile_stride + cc;
    else if (L.kind == 1) elems = g.xoff - (NV - 1);
    else if (L.kind == 2) elems = (long long)(g.Tx - 1) * g.tile_stride + g.xoff + g.hpitch;
    L.bytes = (unsigned)(elems * (long long)sizeof(T));
    L.ring_lane = L.kind == 1 || L.kind == 2;
    L.wave_has_ring = __any(L.ring_lane) != 0;
    L.owner = lane >= GL && lane < WAVE - GL && L.kind == 0;
    return L;
}

// Plane kappa of u(t), counted from a tile of z-layer tz and clamped onto the Dirichlet planes: the
// element offset of its cells (z-layer of tiles + plane), and the distance from a row's first cell to
// the row's x-halo entry that the plane contributes.  kappa in (-td, 2*td]: at most one tile away.
struct TpPlane { long long cells; int to_halo; };
__device__ __forceinline__ TpPlane tp_locate_plane(const Geo &g, int tz, bool z_lo_ring, bool z_hi_ring,
                                                   long long layer_stride, int kappa, int max_beyond)
{
    int tzz = tz, kk;
    kappa = min(kappa, g.td + max_beyond);
    if (kappa <= 0) {
        if (!z_lo_ring) { tzz = tz - 1; kk = g.td + kappa; }
        else kk = 0;
    } else if (kappa > g.td) {
        if (!z_hi_ring) { tzz = tz + 1; kk = kappa - g.td; }
        else kk = g.td + 1;
    } else kk = kappa;
    TpPlane P;
    P.cells = (long long)tzz * layer_stride + (long long)kk * g.plane;
    P.to_halo = kk * g.rows - (int)((long long)kk * g.plane);
    return P;
}

template <typename T, int MODE, int TB, int PF, int MINW>
__global__ __launch_bounds__(WG, MINW) void sweep2d_tp_kernel(Geo g, StripParams sp,
                                                              const T *__restrict__ src, T *__restrict__ dst,
                                                              double *__restrict__ partial)
{
    using V = typename Vec<T>::type;
    constexpr int NV = Vec<T>::N;
    typedef T VU __attribute__((ext_vector_type(NV), aligned(sizeof(T))));
    constexpr int GL = TpGeometry<T, TB, 2>::GHOST_LANES;
    constexpr int SEGW = TpGeometry<T, TB, 2>::SEGW;
    static_assert(PF >= 2 && PF % 2 == 0, "the two-row windows swap roles every step");
    static_assert(MODE != MODE_RESIDUAL, "stand-alone residual uses the single-step kernel");
    __shared__ double red[WAVES_PER_WG];

    const int lane = threadIdx.x % WAVE;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);   // uniform: keeps row math scalar
    const long long lwg = xcd_logical_wg(sp.xcd_chunk);
    const long long s = lwg * WAVES_PER_WG + wave;
    double acc = 0.0;

    if (s < sp.nstrips) {
        // strip = (row of tiles ty, row block rb, column segment seg); the segments run across the
        // whole row of tiles, so a wavefront's lanes may lie in two (or more) neighbouring tiles
        const int per_tyrow = sp.nblk * sp.nseg;
        const int ty = (int)(s / per_tyrow);
        const int rem = (int)(s - (long long)ty * per_tyrow);
        const int rb = rem / sp.nseg, seg = rem - rb * sp.nseg;
        const int r0 = 1 + rb * sp.R;
        const int r1 = min(g.th, r0 + sp.R - 1);

        const TpLane L = tp_lane<T, NV, GL, SEGW>(g, seg, lane);
        const int kind = L.kind;
        const unsigned lane_bytes = L.bytes;
        const bool ring_lane = L.ring_lane, wave_has_ring = L.wave_has_ring, owner = L.owner;
        const bool top_ring = ty == 0, bottom_ring = ty == g.Ty - 1;
        const long long tilerow = (long long)g.Tx * g.tile_stride;
        T *trow = dst + (long long)ty * tilerow;                 // first tile of this row of tiles
        const __amdgpu_buffer_rsrc_t out_rows = buffer_of(trow, (unsigned)(tilerow * (long long)sizeof(T)));

        // u(t) row rho (relative to this tile; clamped to [-(TB), th+1+TB] and onto the ring)
        auto load_row = [&](int rho) -> V {
            int tyy = ty, rr;
            rho = min(rho, g.th + TB);
            if (rho <= 0) {
                if (!top_ring) { tyy = ty - 1; rr = g.th + rho; }
                else rr = 0;
            } else if (rho > g.th) {
                if (!bottom_ring) { tyy = ty + 1; rr = rho - g.th; }
                else rr = g.th + 1;
            } else rr = rho;
            const T *rowp = src + ((long long)tyy * tilerow + (long long)rr * g.pitch);
            unsigned off = lane_bytes;
            if (wave_has_ring) off += ring_lane ? (unsigned)((rr - rr * g.pitch) * (int)sizeof(T)) : 0u;
            return *(const VU *)((const char *)rowp + off);      // ring lanes read element-aligned
        };

        // The strip's pipeline, compiled twice: with the selects that keep Dirichlet cells (FREEZE), and
        // without them for the strips that can never produce one - no ring lane in the wavefront and no
        // ring row within reach of the strip's rows (a level-l row matters up to TB - l rows beyond them).
        // The selects are a quarter of the loop's vector instructions.
        auto run_strip = [&](auto freeze) {
            constexpr bool FREEZE = decltype(freeze)::value;
            V w[TB][2];                      // per level l (0..TB-1): the two newest rows, roles swap each step
#pragma unroll
            for (int l = 0; l < TB; ++l) w[l][0] = w[l][1] = V(0);

            const int nsteps = (r1 - r0 + 1) + 2 * TB;          // rows rho = r0-TB .. r1+TB
            const int nblocks = (nsteps + PF - 1) / PF;
            V cur[PF], nxt[PF];
#pragma unroll
            for (int u = 0; u < PF; ++u) cur[u] = load_row(r0 - TB + u);
            // The first rows have to have arrived before the loop is entered: the compiler places the loop's
            // waits for the longer-waiting of the two ways into it, and entered with loads still in flight the
            // loop would wait at every row for the stores of the row before as well.
#pragma unroll
            for (int u = 0; u < PF; ++u) asm volatile("" : "+v"(cur[u]));

            // one block of PF rows; `storing`: whether the block can contain a row to store
            auto block = [&](int b, auto storing) {
#pragma unroll
                for (int u = 0; u < PF; ++u) nxt[u] = load_row(r0 - TB + (b + 1) * PF + u);
#pragma unroll
                for (int u = 0; u < PF; ++u) {
                    const int q = b * PF + u;
                    const int rho = r0 - TB + q;             // row of u(t) entering the pipeline
                    const int p = u & 1;                     // slot holding the OLDER row of every level
                    V down = cur[u];
#pragma unroll
                    for (int l = 1; l <= TB; ++l) {
                        const V up = w[l - 1][p], c = w[l - 1][1 - p];
                        const int row = rho - l;             // the row this level produces
                        // Dirichlet cells keep their value: whole rows (wave-uniform) and the one component of
                        // a ring lane that is the ring column.  Selects, not branches: with branches the
                        // compiler copied the whole vector around at every level (9 moves per level and row).
                        const bool frozen_all = FREEZE && ((top_ring && row == 0) || (bottom_ring && row == g.th + 1));
                        const T left = from_prev_lane_or_zero(c[NV - 1]);
                        const T right = from_next_lane_or_zero(c[0]);
                        V nw;
#pragma unroll
                        for (int j = 0; j < NV; ++j) {
                            const T we = (j == 0 ? left : c[j - 1]) + (j == NV - 1 ? right : c[j + 1]);
                            const T sn = up[j] + down[j];
                            const bool frozen = frozen_all || (j == NV - 1 && kind == 1) || (j == 0 && kind == 2);
                            nw[j] = FREEZE && frozen ? c[j] : Coef<T>::quarter * (we + sn);
                            if constexpr (MODE == MODE_BOTH) {
                                if (l == 1 && row >= r0 && row <= r1 && owner) {
                                    const T res = (we + sn) - Coef<T>::four * c[j];
                                    const double rd = (double)res;
                                    acc += rd * rd;
                                }
                            }
                        }
                        w[l - 1][p] = down;                  // the older row is dead: its slot takes the newest
                        down = nw;
                    }
                    const int orow = rho - TB;               // `down` is now u(t+TB) of this row
                    const bool stores = q >= 2 * TB && orow <= r1;
                    const unsigned row_bytes = (unsigned)orow * (unsigned)(g.pitch * (int)sizeof(T));
                    if constexpr (decltype(storing)::value)
                        buffer_store_stream(down, out_rows, stores && owner ? lane_bytes + row_bytes : BUF_SKIP);
                }
#pragma unroll
                for (int u = 0; u < PF; ++u) cur[u] = nxt[u];
            };
            // the run-in blocks (rows that only fill the pipeline) issue no stores at all; every later block
            // issues exactly PF, so that they can be counted
            const int run_in = min(2 * TB / PF, nblocks);
            for (int b = 0; b < run_in; ++b) block(b, std::false_type{});
            for (int b = run_in; b < nblocks; ++b) block(b, std::true_type{});
        };
        const bool reaches_ring = wave_has_ring || (top_ring && r0 <= TB) || (bottom_ring && r1 + TB > g.th);
        if (reaches_ring) run_strip(std::true_type{});
        else run_strip(std::false_type{});
    }
    if constexpr (MODE == MODE_BOTH) {
        const double tot = wg_sum(acc, red);
        if (threadIdx.x == 0) partial[lwg] = tot;
    }
}

// ------------------------------------------------------------------------------------
// 3-D: 7-point update (or residual).  new = C6*(((x- + x+)+(y- + y+))+(z- + z+)).
// A wavefront owns RW consecutive rows x 64*NV columns and marches through R planes,
// keeping planes k-1, k, k+1 of its rows in registers.  The y neighbours of the inner rows
// are then registers too; only row i0-1 and row i0+RW of the current plane are loaded (they
// are current rows of the neighbouring wavefronts, so they come from cache).  All x-edge
// cells a plane needs are fetched by ONE gather load (lane l < RW: W edge of row l, lane
// 32+l: E edge of row l) and handed to lanes 0 / 63 as wave-uniform scalars (v_readlane).
// Strip order: tile -> plane block -> row group -> column segment.
// ------------------------------------------------------------------------------------
// NVEC: elements per lane.  16 bytes by default; fp32 grids whose rows are at most 128 elements
// use 2 (8 bytes per lane), so that a 128-wide tile row fills the wavefront instead of half of it.
//
// The march is a software pipeline: everything a trip of U planes needs from memory (the U planes
// above, the two border rows and the edge cells of its own planes) is requested one trip ahead, and
// every memory operation of the loop is unconditional - rows are read and written through a buffer
// descriptor of their plane, lanes beyond the row and rows that must not be stored get BUF_SKIP -
// so that the compiler can count what is outstanding: a trip waits for its own data only, while
// its stores and the next trip's loads stay in flight.  (With loads and stores under branches every
// trip began by waiting for all of them.)  Needs planes smaller than 2 GiB.
template <typename T, int MODE, int RW, int U, int NT, bool PULL, int NVEC = Vec<T>::N>
__global__ __launch_bounds__(WG) void sweep3d_kernel(Geo g, StripParams sp,
                                                     const T *__restrict__ src, T *__restrict__ dst,
                                                     double *__restrict__ partial)
{
    typedef T V __attribute__((ext_vector_type(NVEC)));
    constexpr int NV = NVEC;
    constexpr bool STORES = MODE != MODE_RESIDUAL;
    static_assert(RW >= 1 && RW <= 32, "edge gather uses lanes [0,RW) and [32,32+RW)");
    __shared__ double red[WAVES_PER_WG];

    const int lane = threadIdx.x % WAVE;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);   // uniform: keeps the strip's geometry scalar
    const long long lwg = xcd_logical_wg(sp.xcd_chunk);
    const long long s = lwg * WAVES_PER_WG + wave;
    double acc = 0.0;

    if (s < sp.nstrips) {
        const int ngrp = (g.th + RW - 1) / RW;
        const long long per_tile = (long long)sp.nblk * ngrp * sp.nseg;
        // (the divisions run on the vector unit; their results are uniform and go back to scalar registers)
        const int tl = __builtin_amdgcn_readfirstlane((int)(s / per_tile));      // tile within this launch
        int rem = (int)(s - (long long)tl * per_tile);
        const int t = sp.tile0 + tl;
        const int kb = __builtin_amdgcn_readfirstlane(rem / (ngrp * sp.nseg));
        rem -= kb * ngrp * sp.nseg;
        const int rg = __builtin_amdgcn_readfirstlane(rem / sp.nseg);
        const int i0 = 1 + rg * RW, seg = rem - rg * sp.nseg;
        const int tz = __builtin_amdgcn_readfirstlane(t / (g.Ty * g.Tx));
        const int ty = __builtin_amdgcn_readfirstlane((t / g.Tx) % g.Ty), tx = __builtin_amdgcn_readfirstlane(t % g.Tx);
        const int k0 = 1 + kb * sp.R;
        const int k1 = min(g.td, k0 + sp.R - 1);
        const int col0 = (seg * WAVE + lane) * NV;
        const bool active = col0 < g.pitch;
        const int last = g.tw - 1;
        const bool has_last = active && col0 <= last && last < col0 + NV;
        const int jlast = last - col0;
        // which lane holds the tile's last column in this segment (if any), and whether the
        // wavefront's last lane has a right-hand neighbour cell inside the row
        const int seg_c0 = seg * WAVE * NV;
        const bool seg_has_last = seg_c0 <= last && last < seg_c0 + WAVE * NV;
        const bool w_halo = seg_c0 == 0;
        const int e_col = seg_c0 + WAVE * NV;           // column right of the wavefront
        const bool e_in_row = e_col < g.pitch;

        const T *tsrc = src + (long long)t * g.tile_stride;
        T *tdst = dst + (long long)t * g.tile_stride;
        // push: edge cells into the neighbour tiles' halo cells of dst; pack: x edge cells into the tile's own
        // send arrays (see Fused); x targets are indexed by (plane, row)
        const bool push = MODE != MODE_RESIDUAL && sp.fused == FUSED_PUSH;
        const bool xcopy = MODE != MODE_RESIDUAL && sp.fused != FUSED_NONE;
        const long long zs = (long long)g.Ty * g.Tx * g.tile_stride, ys = (long long)g.Tx * g.tile_stride;
        T *dst_zm = (push && tz > 0) ? tdst - zs : nullptr;
        T *dst_zp = (push && tz < g.Tz - 1) ? tdst + zs : nullptr;
        T *dst_ym = (push && ty > 0) ? tdst - ys : nullptr;
        T *dst_yp = (push && ty < g.Ty - 1) ? tdst + ys : nullptr;
        T *dst_xm = (xcopy && tx > 0 && col0 == 0 && active)
                        ? (push ? tdst - g.tile_stride + g.xoff + g.hpitch : tdst + g.xsend) : nullptr;
        T *dst_xp = (xcopy && tx < g.Tx - 1 && has_last)
                        ? (push ? tdst + g.tile_stride + g.xoff : tdst + g.xsend + g.hpitch) : nullptr;

        // rows below the tile (ragged last row group) are clamped to the y+ halo row th+1, so the
        // register row after the last real row IS that row's y+ neighbour; clamped rows never store
        auto row_of = [&](int rw) { return min(i0 + rw, g.th + 1); };

        // one plane of a tile as a buffer: the lane's column and the row's start add up to the checked offset;
        // lanes at or beyond the pitch get BUF_SKIP (they read zeros and store nothing)
        const unsigned row_bytes = (unsigned)g.pitch * (unsigned)sizeof(T);
        const unsigned plane_bytes = (unsigned)(g.plane * (long long)sizeof(T));       // below 2 GiB
        const unsigned col_bytes = active ? (unsigned)col0 * (unsigned)sizeof(T) : BUF_SKIP;
        // Pull mode (see sweep2d_kernel): cells beyond the tile come from the neighbouring tiles' edge planes,
        // rows and columns instead of the halo cells.  Everything here is wave-uniform.
        const bool pull_zm = PULL && tz > 0, pull_zp = PULL && tz < g.Tz - 1;
        const bool pull_xm = PULL && tx > 0, pull_xp = PULL && tx < g.Tx - 1;
        // where plane k (0 .. td+1) of the tile has to be read: the halo planes from the tiles below / above
        auto plane_off = [&](int k) -> long long {
            return (k == 0 && pull_zm) ? -zs + (long long)g.td * g.plane : (k == g.td + 1 && pull_zp) ? zs + g.plane : (long long)k * g.plane;
        };
        // this wavefront's row rw in such a plane.  In the ragged last row group the rows beyond the tile are
        // clamped onto halo row th+1, which is then a register row's y+ neighbour: pulled from row 1 of the tile behind
        long long row_tile[RW];
        unsigned row_begin[RW];
#pragma unroll
        for (int rw = 0; rw < RW; ++rw) {
            const int row = min(i0 + rw, g.th + 1);
            const bool from_next_tile = PULL && ty < g.Ty - 1 && row == g.th + 1;
            row_tile[rw] = from_next_tile ? ys : 0;
            row_begin[rw] = (unsigned)(from_next_tile ? 1 : row) * row_bytes;
        }
        auto load_row = [&](int k, int rw) {
            return buffer_load<V>(buffer_of(const_cast<T *>(tsrc) + (plane_off(k) + row_tile[rw]), plane_bytes), col_bytes, row_begin[rw]);
        };
        auto dst_plane = [&](int k) { return buffer_of(tdst + (long long)k * g.plane, plane_bytes); };
        auto row_start = [&](int row) { return (unsigned)row * row_bytes; };
        // the rows just above / below this wavefront's rows, in plane k (1 .. td; other k: values unused): halo rows
        // from the tiles before / behind in y
        const int ym_row_own = i0 - 1, yp_row_own = min(i0 + RW, g.th + 1);
        const bool pull_ym = PULL && ty > 0 && ym_row_own == 0, pull_yp = PULL && ty < g.Ty - 1 && yp_row_own == g.th + 1;
        const long long ym_tile = pull_ym ? -ys : 0, yp_tile = pull_yp ? ys : 0;
        const unsigned ym_start = row_start(pull_ym ? g.th : ym_row_own), yp_start = row_start(pull_yp ? 1 : yp_row_own);
        auto ym_plane = [&](int k) { return buffer_of(const_cast<T *>(tsrc) + (ym_tile + (long long)k * g.plane), plane_bytes); };
        auto yp_plane = [&](int k) { return buffer_of(const_cast<T *>(tsrc) + (yp_tile + (long long)k * g.plane), plane_bytes); };

        // x-edge gather: lane l < RW fetches the W edge of row l, lane 32+l the E edge - from the x-halo
        // arrays, or from the neighbouring segment's cells; the other lanes re-read the tile's first cell.
        // (selects, not branches: a branch on the lane would drag wave-uniform values into vector registers)
        const int el = lane & 31, ir = row_of(el);
        const bool fetches = el < RW, w_side = lane < 32;
        const bool w_dense = w_halo && !pull_xm, e_dense = seg_has_last && !pull_xp;    // read from the x-halo arrays
        const long long w_off = w_dense ? xm_off(g, 0, ir) : w_halo ? main_off(g, 0, ir, g.tw - 1) - g.tile_stride
                                                                    : main_off(g, 0, ir, seg_c0 - 1);
        const long long e_off = e_dense ? xp_off(g, 0, ir) : seg_has_last ? main_off(g, 0, ir, 0) + g.tile_stride
                                : e_in_row ? main_off(g, 0, ir, e_col) : 0;
        const long long w_step = w_dense ? (long long)g.rows : g.plane;
        const long long e_step = e_dense ? (long long)g.rows : (seg_has_last || e_in_row) ? g.plane : 0;
        const long long edge_off = fetches ? (w_side ? w_off : e_off) : 0;      // element offset in plane 0
        const long long edge_step = fetches ? (w_side ? w_step : e_step) : 0;   // and per plane

        // what the planes k .. k+U-1 need beyond the two planes already in registers
        struct PlaneIn { V up[RW]; V ym, yp; T edge; };
        auto fetch = [&](PlaneIn (&P)[U], int k) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kc = min(k + u, g.td + 1);          // clamped: stays inside the tile
                const int kn = min(k + u + 1, g.td + 1);
#pragma unroll
                for (int rw = 0; rw < RW; ++rw) P[u].up[rw] = load_row(kn, rw);
                P[u].ym = buffer_load<V>(ym_plane(kc), col_bytes, ym_start);
                P[u].yp = buffer_load<V>(yp_plane(kc), col_bytes, yp_start);
                P[u].edge = tsrc[edge_off + (long long)kc * edge_step];
            }
        };

        V below[RW], cur[RW];
        {
#pragma unroll
            for (int rw = 0; rw < RW; ++rw) {
                below[rw] = load_row(k0 - 1, rw);
                cur[rw] = load_row(k0, rw);
            }
        }

        // planes k .. k+U-1 from the registers and P; stores nothing for planes beyond the strip
        auto advance = [&](PlaneIn (&P)[U], int k) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int kk = k + u;
                const __amdgpu_buffer_rsrc_t out_plane = dst_plane(min(kk, g.td + 1));
#pragma unroll
                for (int rw = 0; rw < RW; ++rw) {
                    const int i = i0 + rw;
                    const bool wanted = kk <= k1 && i <= g.th;               // wave-uniform
                    const V c = cur[rw];
                    const T ew = lane_value(P[u].edge, rw), ee = lane_value(P[u].edge, 32 + rw);
                    const T left = from_prev_lane(c[NV - 1], ew);    // lane 0 keeps the W edge
                    const T right = from_next_lane(c[0], ee);        // lane 63 keeps the E edge
                    const V ymv = rw == 0 ? P[u].ym : cur[rw == 0 ? 0 : rw - 1];
                    const V ypv = rw == RW - 1 ? P[u].yp : cur[rw == RW - 1 ? rw : rw + 1];
                    V out;
#pragma unroll
                    for (int j = 0; j < NV; ++j) {
                        const T w = j == 0 ? left : c[j - 1];
                        T e = j == NV - 1 ? right : c[j + 1];
                        if (has_last && j == jlast) e = ee;
                        const T xx = w + e;
                        const T yy = ymv[j] + ypv[j];
                        const T zz = below[rw][j] + P[u].up[rw][j];
                        out[j] = Coef<T>::sixth * ((xx + yy) + zz);
                        if constexpr (MODE != MODE_UPDATE) {
                            const T res = ((xx + yy) + zz) - Coef<T>::six * c[j];
                            const double rd = (double)res;
                            if (wanted && col0 + j <= last) acc += rd * rd;
                        }
                    }
                    if constexpr (STORES) {
                        buffer_store<(NT & 2) != 0>(out, out_plane, wanted ? col_bytes : BUF_SKIP, row_start(min(i, g.th + 1)));
                        if (xcopy && wanted && active) {
                            if (kk == 1 && dst_zm) *(V *)(dst_zm + main_off(g, g.td + 1, i, col0)) = out;
                            if (kk == g.td && dst_zp) *(V *)(dst_zp + main_off(g, 0, i, col0)) = out;
                            if (i == 1 && dst_ym) *(V *)(dst_ym + main_off(g, kk, g.th + 1, col0)) = out;
                            if (i == g.th && dst_yp) *(V *)(dst_yp + main_off(g, kk, 0, col0)) = out;
                            if (dst_xm) dst_xm[(long long)kk * g.rows + i] = out[0];
                            if (dst_xp) dst_xp[(long long)kk * g.rows + i] = out[jlast];
                        }
                    }
                }
#pragma unroll
                for (int rw = 0; rw < RW; ++rw) {
                    below[rw] = cur[rw];
                    cur[rw] = P[u].up[rw];
                }
            }
        };

        // Two sets of inputs take turns, so that no register is copied.  The first set has to have arrived
        // before the loop: entered with loads in flight, the loop's waits would be placed for that longer wait.
        PlaneIn A[U], B[U];
        fetch(A, k0);
#pragma unroll
        for (int rw = 0; rw < RW; ++rw) {
            asm volatile("" : "+v"(below[rw]));
            asm volatile("" : "+v"(cur[rw]));
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int rw = 0; rw < RW; ++rw) asm volatile("" : "+v"(A[u].up[rw]));
            asm volatile("" : "+v"(A[u].ym));
            asm volatile("" : "+v"(A[u].yp));
            asm volatile("" : "+v"(A[u].edge));
        }
        for (int k = k0; k <= k1; k += 2 * U) {
            fetch(B, k + U);
            advance(A, k);
            fetch(A, k + 2 * U);
            advance(B, k + U);
        }
    }
    if constexpr (MODE != MODE_UPDATE) {
        const double tot = wg_sum(acc, red);
        if (threadIdx.x == 0) partial[lwg] = tot;
    }
}

// ------------------------------------------------------------------------------------
// 3-D, TB time steps per pass over memory, pipelined along z (temporal blocking for the
// 7-point update).  In x a wavefront owns the columns of its inner lanes and carries
// ceil(TB / vector width) ghost lanes per side; segments are laid along a whole row of tiles
// as in sweep2d_tp_kernel.  In y a wavefront owns RW rows and carries TB ghost rows on either
// side (NRW = RW + 2*TB rows per plane; the neighbouring wavefronts recompute them).  In z a
// strip of sp.R planes is a software pipeline: every step loads ONE new plane of u(t) (its NRW
// rows) and advances each level by one plane.  Level l makes its plane (kappa - l) from planes
// (kappa-l-1, kappa-l, kappa-l+1) of level l-1; per level two planes stay in registers.  Rows
// are processed one after the other through all levels, so no third plane buffer is needed.
// Ring cells (planes, rows, columns) keep their value by copying the centre value under
// wave-uniform branches.  All addresses are a wave-uniform base plus one per-lane byte offset
// that never changes.  Bit-identical to TB single steps.  Needs tw a multiple of the vector
// width, th >= TB, td >= TB, and a row of tiles smaller than 2 GiB.
// ------------------------------------------------------------------------------------
template <typename T, int MODE, int TB, int RW, int PF, int MINW>
__global__ __launch_bounds__(WG, MINW) void sweep3d_tp_kernel(Geo g, StripParams sp, int nrg,
                                                              const T *__restrict__ src, T *__restrict__ dst,
                                                              double *__restrict__ partial)
{
    using V = typename Vec<T>::type;
    using G3 = TpGeometry<T, TB, 3>;
    constexpr int NV = Vec<T>::N;
    typedef T VU __attribute__((ext_vector_type(NV), aligned(sizeof(T))));
    constexpr int GL = G3::GHOST_LANES;
    constexpr int SEGW = G3::SEGW;
    constexpr int NRW = RW + 2 * TB;
    static_assert(MODE != MODE_RESIDUAL, "stand-alone residual uses the single-step kernel");
    __shared__ double red[WAVES_PER_WG];

    const int lane = threadIdx.x % WAVE;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const long long lwg = xcd_logical_wg(sp.xcd_chunk);
    const long long s = lwg * WAVES_PER_WG + wave;
    double acc = 0.0;

    if (s < sp.nstrips) {
        // strip = (tz, ty) row of tiles -> plane block -> (column segment, row group), either one fastest:
        // with rows fastest the wavefronts of a workgroup are neighbours in y and share their ghost rows
        const long long per_tilerow = (long long)sp.nblk * nrg * sp.nseg;
        const int tr = (int)(s / per_tilerow);
        int rem = (int)(s - (long long)tr * per_tilerow);
        const int kb = rem / (nrg * sp.nseg);
        rem -= kb * nrg * sp.nseg;
        int seg, rg;
        if (sp.rows_fastest) { seg = rem / nrg; rg = rem - seg * nrg; }
        else { rg = rem / sp.nseg; seg = rem - rg * sp.nseg; }
        const int tz = tr / g.Ty, ty = tr - tz * g.Ty;
        const int k0 = 1 + kb * sp.R, k1 = min(g.td, k0 + sp.R - 1);
        const int i0 = 1 + rg * RW;
        const long long tilerow = (long long)g.Tx * g.tile_stride;     // elements in one row of tiles

        const TpLane L = tp_lane<T, NV, GL, SEGW>(g, seg, lane);
        const int kind = L.kind;
        const unsigned lane_bytes = L.bytes;
        const bool ring_lane = L.ring_lane, wave_has_ring = L.wave_has_ring, owner = L.owner;
        const bool z_lo_ring = tz == 0, z_hi_ring = tz == g.Tz - 1;

        // ---- rows j = 0..NRW-1 <-> tile row iota = i0 - TB + j, followed into the tiles above / below
        long long row_base[NRW];     // element offset of the row inside a z-layer of tiles
        int row_to_halo[NRW];        // (halo entry of the row) - (first cell of the row), elements, plane part aside
        bool ring_row[NRW];
#pragma unroll
        for (int j = 0; j < NRW; ++j) {
            const int iota = min(i0 - TB + j, g.th + TB);
            int tyy = ty, rr = iota;
            ring_row[j] = false;
            if (iota <= 0) {
                if (ty > 0) { tyy = ty - 1; rr = g.th + iota; }
                else { rr = 0; ring_row[j] = true; }
            } else if (iota > g.th) {
                if (ty < g.Ty - 1) { tyy = ty + 1; rr = iota - g.th; }
                else { rr = g.th + 1; ring_row[j] = true; }
            }
            row_base[j] = (long long)tyy * tilerow + (long long)rr * g.pitch;
            row_to_halo[j] = rr - rr * g.pitch;
        }
        // plane kappa of u(t), relative to this tile: where its cells and x-halo entries are
        long long pl_cells;
        int pl_to_halo;
        auto locate_plane = [&](int kappa) {
            const TpPlane P = tp_locate_plane(g, tz, z_lo_ring, z_hi_ring, g.Ty * tilerow, kappa, TB);
            pl_cells = P.cells;
            pl_to_halo = P.to_halo;
        };
        auto load_row = [&](int j) -> V {
            const T *rowp = src + (pl_cells + row_base[j]);
            unsigned off = lane_bytes;
            if (wave_has_ring) off += ring_lane ? (unsigned)((pl_to_halo + row_to_halo[j]) * (int)sizeof(T)) : 0u;
            return *(const VU *)((const char *)rowp + off);      // ring lanes read element-aligned
        };

        V st[TB][2][NRW];                // per level l-1: the two newest planes; roles swap each step
#pragma unroll
        for (int l = 0; l < TB; ++l)
#pragma unroll
            for (int j = 0; j < NRW; ++j) st[l][0][j] = st[l][1][j] = V(0);

        const int nsteps = (k1 - k0 + 1) + 2 * TB;          // planes kappa = k0-TB .. k1+TB
        // the plane in use plus PF planes in flight; the step loop is unrolled so that both the
        // buffer in use and the older state slot are compile-time indices
        constexpr int LDN = PF + 1;
        constexpr int UN = LDN % 2 == 0 ? LDN : 2 * LDN;
        V ld[LDN][NRW];
#pragma unroll
        for (int f = 0; f < PF; ++f) {
            locate_plane(k0 - TB + f);
#pragma unroll
            for (int j = 0; j < NRW; ++j) ld[f][j] = load_row(j);
        }

        const long long out_tile = ((long long)tz * g.Ty + ty) * tilerow;

        for (int q0 = 0; q0 < nsteps; q0 += UN) {
#pragma unroll
            for (int u = 0; u < UN; ++u) {
                const int q = q0 + u;
                if (q >= nsteps) break;
                const int p = u & 1;                         // slot holding the OLDER plane of every level
                const int kappa = k0 - TB + q;               // plane of u(t) entering the pipeline
                locate_plane(kappa + PF);
#pragma unroll
                for (int j = 0; j < NRW; ++j) ld[(u + PF) % LDN][j] = load_row(j);
                bool ring_plane[TB + 1];
#pragma unroll
                for (int l = 1; l <= TB; ++l)
                    ring_plane[l] = (z_lo_ring && kappa - l == 0) || (z_hi_ring && kappa - l == g.td + 1);
                const int oplane = kappa - TB;
                const bool store_plane = q >= 2 * TB && oplane <= k1;
                T *outp = dst + (out_tile + (long long)oplane * g.plane + (long long)i0 * g.pitch);
#pragma unroll
                for (int j = 0; j < NRW; ++j) {
                    V d = ld[u % LDN][j];                    // newest plane of the level below, row j
#pragma unroll
                    for (int l = 1; l <= TB; ++l) {
                        if (j < l - 1 || j >= NRW - (l - 1)) break;     // row not carried at level l-1
                        const V zm = st[l - 1][p][j];
                        st[l - 1][p][j] = d;                 // the older plane is dead: its slot takes the newest
                        if (j < l || j >= NRW - l) break;    // row not produced at level l
                        const V c = st[l - 1][1 - p][j];
                        // Dirichlet cells keep their value (selects, not branches: see sweep2d_tp_kernel)
                        const bool frozen_all = ring_plane[l] || ring_row[j];
                        const V ym = st[l - 1][1 - p][j - 1], yp = st[l - 1][1 - p][j + 1];
                        const T left = from_prev_lane_or_zero(c[NV - 1]);
                        const T right = from_next_lane_or_zero(c[0]);
                        V nw;
#pragma unroll
                        for (int e = 0; e < NV; ++e) {
                            const T xx = (e == 0 ? left : c[e - 1]) + (e == NV - 1 ? right : c[e + 1]);
                            const T yy = ym[e] + yp[e];
                            const T zz = zm[e] + d[e];
                            const T sum = (xx + yy) + zz;
                            const bool frozen = frozen_all || (e == NV - 1 && kind == 1) || (e == 0 && kind == 2);
                            nw[e] = frozen ? c[e] : Coef<T>::sixth * sum;
                            if constexpr (MODE == MODE_BOTH) {
                                const int plane = kappa - 1, row = i0 - TB + j;
                                if (l == 1 && plane >= k0 && plane <= k1 && j >= TB && j < TB + RW && row <= g.th && owner) {
                                    const T res = sum - Coef<T>::six * c[e];
                                    const double rd = (double)res;
                                    acc += rd * rd;
                                }
                            }
                        }
                        d = nw;
                    }
                    // after TB levels `d` is u(t+TB) of plane kappa-TB for the owned rows
                    if (j >= TB && j < TB + RW) {
                        if (store_plane && i0 + (j - TB) <= g.th && owner)
                            __builtin_nontemporal_store(d, (V *)((char *)(outp + (long long)(j - TB) * g.pitch) + lane_bytes));
                    }
                }
            }
        }
    }
    if constexpr (MODE == MODE_BOTH) {
        const double tot = wg_sum(acc, red);
        if (threadIdx.x == 0) partial[lwg] = tot;
    }
}

// ------------------------------------------------------------------------------------
// 3-D, TB time steps per pass, pipelined along z, with the WPG wavefronts of a workgroup
// sharing one range of rows.  Wavefront w holds rows [w*NR, (w+1)*NR) of the workgroup's
// WPG*NR rows (per level two planes of them, in registers); the rows just above and below a
// wavefront's range belong to its neighbours in the workgroup, which publish their first and last
// row of every level's newest plane in LDS each step (double-buffered: one barrier per step).
// Only the workgroup as a whole carries TB ghost rows per side, so WPG*NR rows are loaded per
// WPG*NR - 2*TB rows stored.  Rows are counted along the whole column of tiles (a workgroup's rows
// may lie in two tiles).  Columns, planes, ring handling and addressing as in sweep3d_tp_kernel.
// Rows outside the shrinking range of a level are computed anyway (nothing valid reads them).
// Every workgroup of the grid has work and all its wavefronts take the same number of steps.
// Bit-identical to TB single steps.  Needs tw a multiple of the vector width and td >= TB.
// ------------------------------------------------------------------------------------
template <typename T, int MODE, int TB, int NR, int WPG, int MINW>
__global__ __launch_bounds__(WPG * WAVE, MINW) void sweep3d_tc_kernel(Geo g, StripParams sp, int nyg,
                                                              const T *__restrict__ src, T *__restrict__ dst,
                                                              double *__restrict__ partial)
{
    using V = typename Vec<T>::type;
    using G3 = TpGeometry<T, TB, 3>;
    constexpr int NV = Vec<T>::N;
    typedef T VU __attribute__((ext_vector_type(NV), aligned(sizeof(T))));
    constexpr int GL = G3::GHOST_LANES;
    constexpr int SEGW = G3::SEGW;
    constexpr int WROWS = WPG * NR;              // rows a workgroup (WPG wavefronts) holds
    constexpr int OWN = WROWS - 2 * TB;          // rows it stores
    static_assert(OWN >= 1, "ghost rows must leave something to own");
    static_assert(MODE != MODE_RESIDUAL, "stand-alone residual uses the single-step kernel");
    __shared__ V xch[2][TB][WPG][2][WAVE];   // [step parity][level][wavefront][first / last row][lane]
    __shared__ double red[WPG];

    const int lane = threadIdx.x % WAVE;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const long long lwg = xcd_logical_wg(sp.xcd_chunk);     // a work unit: the grid has exactly one workgroup each
    double acc = 0.0;

    // unit = z-layer of tiles -> plane block -> column segment -> row group
    const int per_layer = sp.nblk * sp.nseg * nyg;
    const int tz = (int)(lwg / per_layer);
    int rem = (int)(lwg - (long long)tz * per_layer);
    const int kb = rem / (sp.nseg * nyg);
    rem -= kb * sp.nseg * nyg;
    const int seg = rem / nyg, yg = rem - seg * nyg;
    const int k0 = 1 + kb * sp.R, k1 = min(g.td, k0 + sp.R - 1);
    const int nrows = g.Ty * g.th;               // rows 1..nrows along the column of tiles; 0 and nrows+1: ring
    const int y0 = 1 + yg * OWN;                 // first row this workgroup stores
    const long long tilerow = (long long)g.Tx * g.tile_stride;

    const TpLane L = tp_lane<T, NV, GL, SEGW>(g, seg, lane);
    const int kind = L.kind;
    const unsigned lane_bytes = L.bytes;
    const bool ring_lane = L.ring_lane, wave_has_ring = L.wave_has_ring, owner = L.owner;
    const bool z_lo_ring = tz == 0, z_hi_ring = tz == g.Tz - 1;

    // ---- this wavefront's rows j = 0..NR-1: row y0 - TB + wave*NR + j of the column of tiles
    long long row_base[NR];      // element offset of the row inside a z-layer of tiles
    int row_to_halo[NR];         // (x-halo entry of the row) - (first cell of the row), elements, plane part aside
    bool ring_row[NR], own_row[NR];
#pragma unroll
    for (int j = 0; j < NR; ++j) {
        const int gi = wave * NR + j;
        const int gy = y0 - TB + gi;
        int tyy, rr;
        ring_row[j] = false;
        if (gy <= 0) { tyy = 0; rr = 0; ring_row[j] = true; }
        else if (gy > nrows) { tyy = g.Ty - 1; rr = g.th + 1; ring_row[j] = true; }
        else { tyy = (gy - 1) / g.th; rr = gy - tyy * g.th; }
        own_row[j] = gi >= TB && gi < WROWS - TB && gy <= nrows;
        row_base[j] = (long long)tyy * tilerow + (long long)rr * g.pitch;
        row_to_halo[j] = rr - rr * g.pitch;
    }
    long long pl_cells;
    int pl_to_halo;
    auto locate_plane = [&](int kappa) {
        const TpPlane P = tp_locate_plane(g, tz, z_lo_ring, z_hi_ring, g.Ty * tilerow, kappa, TB);
        pl_cells = P.cells;
        pl_to_halo = P.to_halo;
    };
    auto load_row = [&](int j) -> V {
        const T *rowp = src + (pl_cells + row_base[j]);
        unsigned off = lane_bytes;
        if (wave_has_ring) off += ring_lane ? (unsigned)((pl_to_halo + row_to_halo[j]) * (int)sizeof(T)) : 0u;
        return *(const VU *)((const char *)rowp + off);
    };

    // The pipeline, compiled twice: with the selects that keep Dirichlet cells, and without them for the
    // wavefronts that can never produce one (no ring lane, no ring row among their rows, no ring plane within
    // reach of the unit's planes).  Both copies pass the same barriers, so the wavefronts of a workgroup may
    // run different ones.
    auto run_unit = [&](auto freeze) {
        constexpr bool FREEZE = decltype(freeze)::value;
        V st[TB][2][NR];                 // per level l-1: the two newest planes; roles swap each step
#pragma unroll
        for (int l = 0; l < TB; ++l)
#pragma unroll
            for (int j = 0; j < NR; ++j) st[l][0][j] = st[l][1][j] = V(0);

        const int nsteps = (k1 - k0 + 1) + 2 * TB;              // planes kappa = k0-TB .. k1+TB
        // The plane entering the pipeline, loaded one step ahead: as soon as a row has been taken, the load
        // of the same row of the next plane is issued in its place, so only ONE plane of loads is live.
        V ld[NR];
        locate_plane(k0 - TB);
#pragma unroll
        for (int j = 0; j < NR; ++j) ld[j] = load_row(j);

        // the first plane has to have arrived before the loop (its waits are placed for the longer-waiting entry)
#pragma unroll
        for (int j = 0; j < NR; ++j) asm volatile("" : "+v"(ld[j]));

        const long long out_layer = (long long)tz * g.Ty * tilerow;
        const unsigned tilerow_bytes = (unsigned)(tilerow * (long long)sizeof(T));      // below 2 GiB
        const int wave_up = max(wave - 1, 0), wave_dn = min(wave + 1, WPG - 1);

        for (int q0 = 0; q0 < nsteps; q0 += 2) {
#pragma unroll
            for (int p = 0; p < 2; ++p) {                        // p: slot holding the OLDER plane of every level
                const int q = q0 + p;
                if (q >= nsteps) break;
                const int kappa = k0 - TB + q;                   // plane of u(t) entering the pipeline
                locate_plane(kappa + 1);
                bool ring_plane[TB + 1];
#pragma unroll
                for (int l = 1; l <= TB; ++l)
                    ring_plane[l] = (z_lo_ring && kappa - l == 0) || (z_hi_ring && kappa - l == g.td + 1);
                const int oplane = kappa - TB;
                const bool store_plane = q >= 2 * TB && oplane <= k1;
                const long long out_plane = out_layer + (long long)oplane * g.plane;
#pragma unroll
                for (int j = 0; j < NR; ++j) {
                    V d = ld[j];                                 // newest plane of the level below, row j
                    ld[j] = load_row(j);                         // same row of the next plane, for the next step
#pragma unroll
                    for (int l = 1; l <= TB; ++l) {
                        const V zm = st[l - 1][p][j];
                        st[l - 1][p][j] = d;                     // the older plane is dead: its slot takes the newest
                        // the neighbouring wavefronts need this plane of our first and last row in the next step
                        if (j == 0) xch[1 - p][l - 1][wave][0][lane] = d;
                        if (j == NR - 1) xch[1 - p][l - 1][wave][1][lane] = d;
                        const V c = st[l - 1][1 - p][j];
                        V ym, yp;
                        if (j == 0) ym = xch[p][l - 1][wave_up][1][lane]; else ym = st[l - 1][1 - p][j - 1];
                        if (j == NR - 1) yp = xch[p][l - 1][wave_dn][0][lane]; else yp = st[l - 1][1 - p][j + 1];
                        const T left = from_prev_lane_or_zero(c[NV - 1]);
                        const T right = from_next_lane_or_zero(c[0]);
                        // Dirichlet cells keep their value: whole planes and rows (wave-uniform), and the one
                        // component of a ring lane that is the ring column.  Selects, not branches: branches
                        // made the compiler copy the whole vector around at every level.
                        const bool frozen_all = FREEZE && (ring_plane[l] || ring_row[j]);
                        V nw;
#pragma unroll
                        for (int e = 0; e < NV; ++e) {
                            const T xx = (e == 0 ? left : c[e - 1]) + (e == NV - 1 ? right : c[e + 1]);
                            const T yy = ym[e] + yp[e];
                            const T zz = zm[e] + d[e];
                            const T sum = (xx + yy) + zz;
                            const bool frozen = frozen_all || (e == NV - 1 && kind == 1) || (e == 0 && kind == 2);
                            nw[e] = FREEZE && frozen ? c[e] : Coef<T>::sixth * sum;
                            if constexpr (MODE == MODE_BOTH) {
                                const int plane = kappa - 1;
                                if (l == 1 && plane >= k0 && plane <= k1 && own_row[j] && owner) {
                                    const T res = sum - Coef<T>::six * c[e];
                                    const double rd = (double)res;
                                    acc += rd * rd;
                                }
                            }
                        }
                        d = nw;
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // after TB levels `d` is u(t+TB) of plane kappa-TB: one counted store per row, dropped where
                    // there is nothing to store (see buffer_store_stream)
                    buffer_store_stream(d, buffer_of(dst + (out_plane + row_base[j]), tilerow_bytes),
                                        store_plane && own_row[j] && owner ? lane_bytes : BUF_SKIP);
                    // keep the rows in program order: hoisting later rows' loads and LDS reads costs registers
                    __builtin_amdgcn_sched_barrier(0);
                }
                __syncthreads();                                 // next step reads what this one published
            }
        }
    };
    bool reaches_ring = wave_has_ring || (z_lo_ring && k0 <= 2 * TB) || (z_hi_ring && k1 + 2 * TB > g.td);
#pragma unroll
    for (int j = 0; j < NR; ++j) reaches_ring = reaches_ring || ring_row[j];
    if (reaches_ring) run_unit(std::true_type{});
    else run_unit(std::false_type{});
    if constexpr (MODE == MODE_BOTH) {
        const double tot = wg_sum(acc, red);
        if (threadIdx.x == 0) partial[lwg] = tot;
    }
}

}  // namespace jk
