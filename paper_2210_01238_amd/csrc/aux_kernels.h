// Device code used only by the host API translation unit: the final stage of the residual
// reduction, halo / boundary face copies, scatter / gather, and the plain copy probe.
#pragma once
#include "jacobi_kernels.h"

namespace jk {

// Final stage of the residual: one workgroup adds the per-workgroup partials in a fixed
// order (thread t takes t, t+1024, ... into eight running sums by turns, so that eight loads are in
// flight instead of one - 32768 partials took 17-35 us with a single sum -; then a fixed tree over the
// eight, the shuffle tree and LDS) and writes the sqrt.
__global__ __launch_bounds__(1024) void residual_final_kernel(const double *__restrict__ partial,
                                                              long long n, double *__restrict__ result)
{
    __shared__ double red[16];
    constexpr int U = 8;
    double acc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) acc[u] = 0.0;
    const long long step = blockDim.x;
    long long i = threadIdx.x;
    for (; i + (U - 1) * step < n; i += U * step) {
        double v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = partial[i + u * step];
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u] += v[u];
    }
#pragma unroll
    for (int u = 0; u < U - 1; ++u)                                   // fewer than U left
        if (i + u * step < n) acc[u] += partial[i + u * step];
    const double mine = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
    const double tot = wg_sum(mine, red);
    if (threadIdx.x == 0) *result = sqrt(tot);
}

// ------------------------------------------------------------------------------------
// Boundary copy.  A face of a tile is one of its 2*ndim halo faces (0: x-, 1: x+, 2: y-, 3: y+, 4: z-,
// 5: z+).  For every face that lies on the domain boundary, the Dirichlet halo cells are copied from the
// `src` grid to the `dst` grid - the full padded extent of the face, with its edges and corners, so that
// the destination carries the complete ring.  Work item = (tile, face, chunk of 4*WG cells); workgroups
// stride over the item list.
// ------------------------------------------------------------------------------------
constexpr int FACE_CHUNK = 4 * WG;

template <typename T>
__global__ __launch_bounds__(WG) void boundary_copy_kernel(Geo g, const T *__restrict__ src, T *__restrict__ dst,
                                                           int chunks_per_face, long long nitems)
{
    const int nfaces = 2 * g.ndim;
    for (long long item = blockIdx.x; item < nitems; item += gridDim.x) {
        const int chunk = (int)(item % chunks_per_face);
        const long long tf = item / chunks_per_face;
        const int face = (int)(tf % nfaces), t = (int)(tf / nfaces);
        const int axis = face >> 1, hi = face & 1;   // axis 0: x, 1: y, 2: z
        const int tz = t / (g.Ty * g.Tx), ty = (t / g.Tx) % g.Ty, tx = t % g.Tx;
        const int tc = axis == 0 ? tx : axis == 1 ? ty : tz;
        const int Tn = axis == 0 ? g.Tx : axis == 1 ? g.Ty : g.Tz;
        if (hi ? tc < Tn - 1 : tc > 0) continue;     // a neighbouring tile, not the boundary
        const long long tile = (long long)t * g.tile_stride;
        // face cells are indexed (a, b) with b fastest, over the padded extent
        const int nb = axis == 0 ? g.rows : g.tw;
        const int na = axis == 2 ? g.rows : g.nplanes;
        const long long n = (long long)na * nb;
        const long long base = (long long)chunk * FACE_CHUNK;
        for (int q = 0; q < 4; ++q) {
            const long long e = base + q * WG + threadIdx.x;
            if (e >= n) break;
            const int a = (int)(e / nb), b = (int)(e - (long long)a * nb);
            const long long off = axis == 0   ? (hi ? xp_off(g, a, b) : xm_off(g, a, b))      // (plane, row)
                                  : axis == 1 ? main_off(g, a, hi ? g.th + 1 : 0, b)          // (plane, column)
                                              : main_off(g, hi ? g.td + 1 : 0, a, b);         // (row, column)
            dst[tile + off] = src[tile + off];
        }
    }
}

// ------------------------------------------------------------------------------------
// Stand-alone halo exchange (paper Sec. VI-C: pack, transfer, unpack - one copy on one device): for every
// face of every tile that has a neighbour, halo cells <- the neighbour's edge cells, in place in one grid.
// y and z faces are rows of the neighbour (contiguous, cache-line aligned): copied as 16-byte vectors, whole
// vectors (the padding columns behind a row may hold anything and are overwritten with the source's).
// x faces, XSRC = 0: gathered from the neighbour's first / last column, one cell per row (one cell per cache
// line: 16 times the payload is read; always valid).  XSRC = 1: copied from the neighbour's dense x send
// arrays, which a FUSED_PACK update of that grid has just filled (dense to dense).
// Work item = (tile, face, chunk of 4*64 vectors or cells), one per WAVEFRONT (faces of small tiles are a few
// hundred bytes: a whole workgroup per face would idle most of its lanes); a lane issues its (up to) four
// loads before its stores.  Workgroups stride over the item list.
// ------------------------------------------------------------------------------------
constexpr int HALO_CHUNK = 4 * WAVE;

template <typename T, int XSRC>
__global__ __launch_bounds__(WG) void halo_exchange_kernel(Geo g, T *grid, int chunks_per_face, long long nitems)
{
    using V = typename Vec<T>::type;
    constexpr int NV = Vec<T>::N;
    const int nfaces = 2 * g.ndim;
    const int vrow = (g.tw + NV - 1) / NV;           // vectors per row (pitch is a multiple of NV)
    const int lane = threadIdx.x % WAVE, wave = threadIdx.x / WAVE;
    for (long long item = (long long)blockIdx.x * WAVES_PER_WG + wave; item < nitems; item += (long long)gridDim.x * WAVES_PER_WG) {
        const int chunk = (int)(item % chunks_per_face);
        const long long tf = item / chunks_per_face;
        const int face = (int)(tf % nfaces), t = (int)(tf / nfaces);
        const int axis = face >> 1, hi = face & 1;   // axis 0: x, 1: y, 2: z
        const int tz = t / (g.Ty * g.Tx), ty = (t / g.Tx) % g.Ty, tx = t % g.Tx;
        const int tc = axis == 0 ? tx : axis == 1 ? ty : tz;
        const int Tn = axis == 0 ? g.Tx : axis == 1 ? g.Ty : g.Tz;
        if (!(hi ? tc < Tn - 1 : tc > 0)) continue;   // no neighbour on this side
        const long long tstep = axis == 0 ? 1 : axis == 1 ? g.Tx : (long long)g.Ty * g.Tx;
        const T *stile = grid + ((long long)t + (hi ? tstep : -tstep)) * g.tile_stride;
        T *dtile = grid + (long long)t * g.tile_stride;
        // offsets inside a tile fit 32 bits (a tile has fewer than 2^31 elements): keeps the index arithmetic cheap
        const unsigned base = (unsigned)chunk * HALO_CHUNK;
        unsigned dofs[4];
        constexpr unsigned NONE = 0xffffffffu;
        if (axis == 0) {
            // cells (plane a, row b), b fastest: consecutive lanes write consecutive halo entries
            const unsigned n = (unsigned)g.td * (unsigned)g.th;
            const unsigned s0 = XSRC ? (unsigned)(g.xsend + (hi ? 0 : g.hpitch)) : (hi ? 0u : (unsigned)(g.tw - 1));
            const unsigned d0 = (unsigned)(g.xoff + (hi ? g.hpitch : 0));
            T v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned e = base + q * WAVE + lane;
                dofs[q] = NONE;
                if (e >= n) continue;
                const unsigned a = e / (unsigned)g.th, b = e - a * (unsigned)g.th;
                const unsigned k = g.z0 + a, i = 1 + b;
                const unsigned entry = k * (unsigned)g.rows + i;
                // my x+ halo <- the right neighbour's first column; my x- halo <- the left neighbour's last column
                v[q] = stile[XSRC ? s0 + entry : entry * (unsigned)g.pitch + s0];
                dofs[q] = d0 + entry;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (dofs[q] != NONE) dtile[dofs[q]] = v[q];
        } else {
            // vectors (row a of the face, vector b of the row): y faces have one row per plane, z faces th rows
            const unsigned na = axis == 1 ? g.td : g.th;
            const unsigned n = na * (unsigned)vrow;
            // element offset of face row a: y faces step by a plane, z faces by a row
            const unsigned step = axis == 1 ? (unsigned)g.plane : (unsigned)g.pitch;
            const unsigned first = axis == 1 ? (unsigned)g.z0 * (unsigned)g.plane : (unsigned)g.pitch;
            const unsigned d0 = first + (axis == 1 ? (hi ? (unsigned)(g.th + 1) * g.pitch : 0u)
                                                   : (hi ? (unsigned)(g.td + 1) * (unsigned)g.plane : 0u));
            const unsigned s0 = first + (axis == 1 ? (hi ? 1u : (unsigned)g.th) * g.pitch
                                                   : (hi ? 1u : (unsigned)g.td) * (unsigned)g.plane);
            V v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned e = base + q * WAVE + lane;
                dofs[q] = NONE;
                if (e >= n) continue;
                const unsigned a = e / (unsigned)vrow, c = (e - a * (unsigned)vrow) * NV;
                v[q] = *(const V *)(stile + (s0 + a * step + c));
                dofs[q] = d0 + a * step + c;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (dofs[q] != NONE) *(V *)(dtile + dofs[q]) = v[q];
        }
    }
}

// ------------------------------------------------------------------------------------
// Scatter / gather between a padded global array and the tile-major grid.
// Work item = (padded row of a tile: tile, plane, row; chunk of 64*Q padded columns), one per WAVEFRONT.  A lane
// moves Q cells 64 columns apart - column index cc in [-1, tw]: the two x halo cells live in the dense arrays -
// and issues its Q loads before its Q stores.  Consecutive lanes move consecutive cells on both sides.
// ------------------------------------------------------------------------------------
template <typename T, bool GATHER, int Q>
__global__ __launch_bounds__(WG) void scatter_gather_kernel(Geo g, const T *__restrict__ from, T *__restrict__ to,
                                                            long long GP, long long GQ, unsigned nchunks,
                                                            unsigned nitems)
{
    const unsigned w = blockIdx.x * WAVES_PER_WG + threadIdx.x / WAVE;      // the host keeps nitems below 2^32 - 4
    if (w >= nitems) return;
    const unsigned chunk = w % nchunks;
    const unsigned item = w / nchunks;                   // (tile, plane, row)
    const int i = (int)(item % (unsigned)g.rows);
    const unsigned rest = item / (unsigned)g.rows;
    const int k = (int)(rest % (unsigned)g.nplanes), t = (int)(rest / (unsigned)g.nplanes);
    const int tz = t / (g.Ty * g.Tx), ty = (t / g.Tx) % g.Ty, tx = t % g.Tx;
    const long long tbase = (long long)t * g.tile_stride;
    const long long row = tbase + main_off(g, k, i, 0), xm = tbase + xm_off(g, k, i), xp = tbase + xp_off(g, k, i);
    const long long gk = g.ndim == 3 ? (long long)tz * g.td + k : 0;
    const long long grow = gk * GQ + ((long long)ty * g.th + i) * GP + (long long)tx * g.tw + 1;   // of tile column 0
    // gather: a padded cell of the tile is written back if it is interior to the tile or lies on the domain
    // boundary; the tile's copies of neighbouring tiles' cells are skipped
    const bool in_k = g.ndim == 2 || (k >= 1 && k <= g.td) || (k == 0 && tz == 0) || (k == g.td + 1 && tz == g.Tz - 1);
    const bool in_i = (i >= 1 && i <= g.th) || (i == 0 && ty == 0) || (i == g.th + 1 && ty == g.Ty - 1);
    if (GATHER && !(in_k && in_i)) return;
    T v[Q];
    long long dst[Q];
    bool ok[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const int cc = ((int)chunk * Q + q) * WAVE + (int)(threadIdx.x % WAVE) - 1;
        ok[q] = cc <= g.tw;
        const long long toff = cc < 0 ? xm : cc == g.tw ? xp : row + cc;
        const long long goff = grow + cc;
        if (GATHER) ok[q] = ok[q] && ((cc >= 0 && cc < g.tw) || (cc < 0 && tx == 0) || (cc == g.tw && tx == g.Tx - 1));
        dst[q] = GATHER ? goff : toff;
        v[q] = ok[q] ? from[GATHER ? toff : goff] : T(0);
    }
#pragma unroll
    for (int q = 0; q < Q; ++q)
        if (ok[q]) to[dst[q]] = v[q];
}

// Plain streaming copy, 16 bytes per lane, one element per thread, workgroups in memory
// order (the fastest simple copy on this chip): the practical bandwidth ceiling the update
// kernel is compared with, and the known-size dispatch used to calibrate HBM counters.
__global__ __launch_bounds__(WG) void stream_copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                         long long n16)
{
    const long long i = (long long)blockIdx.x * WG + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

}  // namespace jk
