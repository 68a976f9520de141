// Device code used only by the host API translation unit: the final stage of the residual
// reduction, halo / boundary face copies, scatter / gather, and the plain copy probe.
#pragma once
#include "jacobi_kernels.h"

namespace jk {

// Final stage of the residual: one workgroup adds the per-workgroup partials in a fixed
// order (thread t takes t, t+1024, ...; then shuffle tree + LDS) and writes the sqrt.
__global__ __launch_bounds__(1024) void residual_final_kernel(const double *__restrict__ partial,
                                                              long long n, double *__restrict__ result)
{
    __shared__ double red[16];
    double acc = 0.0;
    for (long long i = threadIdx.x; i < n; i += blockDim.x) acc += partial[i];
    const double tot = wg_sum(acc, red);
    if (threadIdx.x == 0) *result = sqrt(tot);
}

// ------------------------------------------------------------------------------------
// Face copies.  A face of a tile is one of its 2*ndim halo faces (0: x-, 1: x+, 2: y-,
// 3: y+, 4: z-, 5: z+), interior extent only (edges/corners are never read by the
// stencils).  EXCHANGE: for faces with a neighbouring tile, halo <- neighbour's edge cells
// (pack + transfer + unpack in one gather-scatter copy), within one grid.  BOUNDARY: for
// faces on the domain boundary, copy the Dirichlet halo cells from `src` grid to `dst` grid.
// Work item = (tile, face, chunk of 4*WG cells); workgroups stride over the item list.
// ------------------------------------------------------------------------------------
enum FaceMode { FACE_EXCHANGE = 0, FACE_BOUNDARY = 1 };
constexpr int FACE_CHUNK = 4 * WG;

template <typename T, int FMODE>
__global__ __launch_bounds__(WG) void face_copy_kernel(Geo g, const T *__restrict__ src, T *__restrict__ dst,
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
        const bool has_nbr = hi ? tc < Tn - 1 : tc > 0;
        if ((FMODE == FACE_EXCHANGE) != has_nbr) continue;

        const long long tstep = axis == 0 ? 1 : axis == 1 ? g.Tx : (long long)g.Ty * g.Tx;
        const T *stile = src + ((long long)t + (FMODE == FACE_EXCHANGE ? (hi ? tstep : -tstep) : 0)) * g.tile_stride;
        T *dtile = dst + (long long)t * g.tile_stride;

        // face cells are indexed (a, b) with b fastest.  EXCHANGE copies the interior extent of
        // the face; BOUNDARY the full padded extent (face plus its edges and corners), so the
        // destination grid carries the complete Dirichlet ring.
        constexpr int X = FMODE == FACE_BOUNDARY ? 1 : 0;   // extend by the halo cells
        const int nb = axis == 0 ? g.th + 2 * X : g.tw;
        const int na = axis == 2 ? g.th + 2 * X : (X ? g.nplanes : g.td);
        const int k_first = X ? 0 : g.z0, i_first = X ? 0 : 1;
        const long long n = (long long)na * nb;
        const long long base = (long long)chunk * FACE_CHUNK;
        for (int q = 0; q < 4; ++q) {
            const long long e = base + q * WG + threadIdx.x;
            if (e >= n) break;
            const int a = (int)(e / nb), b = (int)(e - (long long)a * nb);
            long long so, dofs;
            if (axis == 0) {          // (a, b) = (plane, row)
                const int k = k_first + a, i = i_first + b;
                dofs = hi ? xp_off(g, k, i) : xm_off(g, k, i);
                so = FMODE == FACE_BOUNDARY ? dofs : main_off(g, k, i, hi ? 0 : g.tw - 1);
            } else if (axis == 1) {   // (a, b) = (plane, column)
                const int k = k_first + a;
                dofs = main_off(g, k, hi ? g.th + 1 : 0, b);
                so = FMODE == FACE_BOUNDARY ? dofs : main_off(g, k, hi ? 1 : g.th, b);
            } else {                  // (a, b) = (row, column)
                const int i = i_first + a;
                dofs = main_off(g, hi ? g.td + 1 : 0, i, b);
                so = FMODE == FACE_BOUNDARY ? dofs : main_off(g, hi ? 1 : g.td, i, b);
            }
            dtile[dofs] = stile[so];
        }
    }
}

// ------------------------------------------------------------------------------------
// Scatter / gather between a padded global array and the tile-major grid.
// Work item = (tile, padded plane, padded row, chunk of WG columns); one thread per padded
// cell, column index cc in [-1, tw].  Workgroups stride over the item list.
// ------------------------------------------------------------------------------------
template <typename T, bool GATHER>
__global__ __launch_bounds__(WG) void scatter_gather_kernel(Geo g, const T *__restrict__ from, T *__restrict__ to,
                                                            long long GP, long long GQ, int chunks_per_row,
                                                            long long nitems)
{
    for (long long item = blockIdx.x; item < nitems; item += gridDim.x) {
        const int chunk = (int)(item % chunks_per_row);
        long long rest = item / chunks_per_row;
        const int i = (int)(rest % g.rows);
        rest /= g.rows;
        const int k = (int)(rest % g.nplanes), t = (int)(rest / g.nplanes);
        const int tz = t / (g.Ty * g.Tx), ty = (t / g.Tx) % g.Ty, tx = t % g.Tx;
        const int cc = chunk * WG + (int)threadIdx.x - 1;
        if (cc > g.tw) continue;
        const long long toff = (long long)t * g.tile_stride +
                               (cc < 0 ? xm_off(g, k, i) : cc == g.tw ? xp_off(g, k, i) : main_off(g, k, i, cc));
        const long long gk = g.ndim == 3 ? (long long)tz * g.td + k : 0;
        const long long gi = (long long)ty * g.th + i, gj = (long long)tx * g.tw + cc + 1;
        const long long goff = gk * GQ + gi * GP + gj;
        if constexpr (!GATHER) {
            to[toff] = from[goff];
        } else {
            // a padded cell of the tile is written back if it is interior to the tile, or lies on
            // the domain boundary; copies of neighbouring tiles' cells are skipped
            const bool in_k = g.ndim == 2 || (k >= 1 && k <= g.td) || (k == 0 && tz == 0) ||
                              (k == g.td + 1 && tz == g.Tz - 1);
            const bool in_i = (i >= 1 && i <= g.th) || (i == 0 && ty == 0) || (i == g.th + 1 && ty == g.Ty - 1);
            const bool in_c = (cc >= 0 && cc < g.tw) || (cc < 0 && tx == 0) || (cc == g.tw && tx == g.Tx - 1);
            if (in_k && in_i && in_c) to[goff] = from[toff];
        }
    }
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
