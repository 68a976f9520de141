// Small 2-D grids: ALL iterations of a jacobi_sweep call in ONE kernel launch.
//
// A grid of a few hundred rows is updated in about a microsecond, so a launch per iteration (paper
// Sec. VI-C: exchange, then update, every iteration) leaves the chip waiting for the host: the runtime
// the paper describes exists to overlap exactly that sequencing (Sec. IV-B, VI-A).  On one device the
// remedy is to not return to the host at all: the grid stays in registers, the iterations run inside
// the kernel, and the workgroups meet at a barrier in device memory every `d` iterations only.
//
// Decomposition.  Rows are counted along the whole column of tiles (1 .. Ny; 0 and Ny+1 are the
// Dirichlet ring), columns along the whole row of tiles (0 .. Nx-1).  Workgroup b owns B consecutive
// rows and HOLDS HR = B + 2d: d ghost rows on either side, which the neighbouring workgroups own and
// this one recomputes (a ghost row is exact for as many iterations as its distance to the end of the
// held range, so after d iterations they are refreshed).  The 16 wavefronts of a workgroup split the
// held rows: wavefront w keeps rows [w*RW, (w+1)*RW) in registers, full width (NSEG segments of 64
// lanes x 16 bytes).  Every iteration each wavefront publishes its first and last row in LDS
// (double-buffered by iteration parity: one barrier per iteration), reads the rows next to its range
// from its neighbours, and updates its rows in place, top to bottom.  The x neighbours come from the
// adjacent lanes (DPP wave shifts), across a segment seam from the other segment's end lane
// (v_readlane), beside the first / last column from the Dirichlet values loaded once.
//
// Phases.  The iterations are cut into phases of at most d.  After a phase every workgroup stores its
// OWNED rows to the destination grid, all workgroups meet at a grid barrier (one arrival counter in
// device memory, agent-scope release / acquire around it so the other XCDs' L2s see the rows), each
// reloads only its ghost rows from that grid, and the two grids swap roles: exactly the ping-pong of
// the launch-per-pass path, with the owned rows never leaving the registers.  A plan of at most HR - 2
// rows runs in a single workgroup with no barrier at all.
//
// The barrier needs all workgroups resident at once: the host launches at most one per CU.  Its wait
// is bounded (spin_limit polls): a workgroup that gives up sets a flag, every workgroup that sees the
// flag stops waiting, and all of them write NaN instead of results, so a launch always drains and a
// failed one cannot be mistaken for a good one.
//
// One launch is the whole call.  The kernel carries the Dirichlet ring to the other grid itself (the ring
// rows and the cells beside each row are in its registers anyway), it can deliver the residual norm of the
// grid it produced (one more exchange of border rows; the last workgroup to finish adds the workgroups'
// partial sums in index order), and that last workgroup also puts the barrier words back to zero for the
// next launch: a workgroup counts itself as finished after its last barrier and nobody waits for that
// count, so this needs no further synchronisation and also cleans up after a barrier that gave up.
//
// Every value is formed by the single-step expression 0.25*((W+E)+(S+N)): bit-identical to the
// launch-per-iteration path.  Needs tw a multiple of the vector width and Nx <= NSEG*64 vectors.
#pragma once
#include "launchers.h"

namespace jk {

// All workgroups of the grid wait for each other.  `target` = arrivals expected so far.  Returns false if
// this workgroup gave up waiting (or saw that another one had).  The cache maintenance that makes one XCD's
// stores visible to the others (write back the L2's dirty lines before arriving, drop its clean lines after
// the wait) is done ONCE per workgroup, by thread 0: the wavefronts of a workgroup share their CU's L1 and
// their XCD's L2, every wavefront's stores have completed when it passes the first barrier below, and none
// of them loads before the second.  (All 16 wavefronts doing it cost 7 us per barrier.)
__device__ __forceinline__ bool resident_grid_barrier(unsigned *sync, unsigned target, unsigned spin_limit, int *lds_flag)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");      // this wavefront's stores have completed
    __syncthreads();
    if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __hip_atomic_fetch_add(&sync[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool ok = false;
        for (unsigned n = 0; n <= spin_limit; ++n) {
            if (__hip_atomic_load(&sync[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) { ok = true; break; }
            if (__hip_atomic_load(&sync[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
            __builtin_amdgcn_s_sleep(2);
        }
        if (!ok) __hip_atomic_store(&sync[1], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        *lds_flag = ok ? 1 : 0;
    }
    __syncthreads();
    return *lds_flag != 0;
}

// Column layout: a lane holds NSEG consecutive 16-byte vectors of a row (lane l: columns [l*NSEG*NV,
// (l+1)*NSEG*NV)), so only the first and the last of its cells have their x neighbour in another lane.
template <typename T, int NSEG, int RW>
__global__ __launch_bounds__(RES_WAVES * WAVE) void resident2d_kernel(Geo g, ResidentParams rp, T *ga, T *gb)
{
    using V = typename Vec<T>::type;
    constexpr int NV = Vec<T>::N;
    static_assert(NSEG >= 1 && NSEG <= RES_MAX_SEG && RW >= 1 && RW <= RES_MAX_RW, "variant out of range");
    __shared__ V xch[2][RES_WAVES][2][NSEG][WAVE];      // [parity][wavefront][first / last row][vector][lane]
    __shared__ int barrier_ok;

    const int lane = threadIdx.x % WAVE;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int Ny = g.Ty * g.th, Nx = g.Tx * g.tw;
    const int own_lo = 1 + (int)blockIdx.x * rp.B;
    const int own_hi = min(Ny, own_lo + rp.B - 1);
    const bool single = gridDim.x == 1;

    // ---- this wavefront's rows j = 0..RW-1: row own_lo - d + wave*RW + j, clamped onto the ring rows
    long long row_off[RW];       // element offset of the row's first cell (first tile of its row of tiles)
    bool ring_row[RW], own_row[RW];
    T edge_w[RW], edge_e[RW];    // Dirichlet values beside the row's first and last column
    bool wave_has_ring = false;
#pragma unroll
    for (int j = 0; j < RW; ++j) {
        int gy = own_lo - rp.d + wave * RW + j;
        gy = max(0, min(gy, Ny + 1));
        ring_row[j] = gy == 0 || gy == Ny + 1;
        wave_has_ring = wave_has_ring || ring_row[j];
        own_row[j] = gy >= own_lo && gy <= own_hi;
        const int ty = gy == 0 ? 0 : gy == Ny + 1 ? g.Ty - 1 : (gy - 1) / g.th;
        const int rr = gy - ty * g.th;                       // 0 .. th+1
        const long long tile_row = (long long)ty * g.Tx * g.tile_stride;
        row_off[j] = tile_row + (long long)rr * g.pitch;
        edge_w[j] = ga[tile_row + xm_off(g, 0, rr)];
        edge_e[j] = ga[tile_row + (long long)(g.Tx - 1) * g.tile_stride + xp_off(g, 0, rr)];
    }
    // ---- this lane's vectors: s-th vector = columns gc .. gc+NV-1 along the row of tiles
    long long col_off[NSEG];
    bool active[NSEG], has_last[NSEG];
#pragma unroll
    for (int s = 0; s < NSEG; ++s) {
        const int gc = (lane * NSEG + s) * NV;
        active[s] = gc < Nx;
        has_last[s] = active[s] && gc + NV == Nx;            // Nx is a multiple of NV
        const int tx = active[s] ? gc / g.tw : 0, c = active[s] ? gc - tx * g.tw : 0;
        col_off[s] = (long long)tx * g.tile_stride + c;
    }
    const bool ragged = Nx != WAVE * NSEG * NV;              // the last column is not the last lane's last cell

    V A[RW][NSEG], Bv[RW][NSEG];
    auto load_row = [&](const T *grid, int j) {
#pragma unroll
        for (int s = 0; s < NSEG; ++s)
            A[j][s] = active[s] ? *(const V *)(grid + row_off[j] + col_off[s]) : V(0);
    };
#pragma unroll
    for (int j = 0; j < RW; ++j) load_row(ga, j);

    if (rp.copy_ring) {
        // the other grid gets the ring: the two ring rows from the workgroups that own the rows next to them,
        // the cells beside a row (the corners beside the ring rows) from whoever owns or copies that row
#pragma unroll
        for (int j = 0; j < RW; ++j) {
            const int gy = max(0, min(own_lo - rp.d + wave * RW + j, Ny + 1));
            const bool mine = own_row[j] || (gy == 0 && own_lo == 1) || (gy == Ny + 1 && own_hi == Ny);
            if (!mine) continue;
            if (ring_row[j]) {
#pragma unroll
                for (int s = 0; s < NSEG; ++s)
                    if (active[s]) *(V *)(gb + row_off[j] + col_off[s]) = A[j][s];
            }
            if (lane == 0) {
                const int ty = gy == 0 ? 0 : gy == Ny + 1 ? g.Ty - 1 : (gy - 1) / g.th;
                const int rr = gy - ty * g.th;
                const long long tile_row = (long long)ty * g.Tx * g.tile_stride;
                gb[tile_row + xm_off(g, 0, rr)] = edge_w[j];
                gb[tile_row + (long long)(g.Tx - 1) * g.tile_stride + xp_off(g, 0, rr)] = edge_e[j];
            }
        }
    }

    const int wave_up = max(wave - 1, 0), wave_dn = min(wave + 1, RES_WAVES - 1);

    // One iteration: rows `a` -> rows `b`.  RING: some row of this wavefront is a Dirichlet row (keeps its value);
    // RAGGED: the cell right of the last column is not the next lane's first cell.
    auto step = [&](V (&a)[RW][NSEG], V (&b)[RW][NSEG], int parity, auto ring, auto rag) {
        constexpr bool RING = decltype(ring)::value, RAGGED = decltype(rag)::value;
#pragma unroll
        for (int s = 0; s < NSEG; ++s) {
            xch[parity][wave][0][s][lane] = a[0][s];
            xch[parity][wave][1][s][lane] = a[RW - 1][s];
        }
        __syncthreads();
        V above[NSEG], below[NSEG];
#pragma unroll
        for (int s = 0; s < NSEG; ++s) {
            above[s] = xch[parity][wave_up][1][s][lane];
            below[s] = xch[parity][wave_dn][0][s][lane];
        }
#pragma unroll
        for (int j = 0; j < RW; ++j) {
            const T left = from_prev_lane(a[j][NSEG - 1][NV - 1], edge_w[j]);     // lane 0 keeps the W ring value
            const T right = from_next_lane(a[j][0][0], edge_e[j]);                // lane 63 keeps the E ring value
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                const V up = j == 0 ? above[s] : a[j == 0 ? 0 : j - 1][s];
                const V dn = j == RW - 1 ? below[s] : a[j == RW - 1 ? j : j + 1][s];
#pragma unroll
                for (int e = 0; e < NV; ++e) {
                    const T w = e > 0 ? a[j][s][e - 1] : s > 0 ? a[j][s > 0 ? s - 1 : 0][NV - 1] : left;
                    T ea = e < NV - 1 ? a[j][s][e + 1] : s < NSEG - 1 ? a[j][s < NSEG - 1 ? s + 1 : s][0] : right;
                    if (RAGGED && e == NV - 1) ea = has_last[s] ? edge_e[j] : ea;
                    const T val = Coef<T>::quarter * ((w + ea) + (up[e] + dn[e]));
                    b[j][s][e] = RING && ring_row[j] ? a[j][s][e] : val;
                }
            }
        }
    };
    // `depth` iterations on A (result back in A); the two register sets take turns
    auto iterate = [&](int depth, auto ring, auto rag) {
        int it = 0;
        for (; it + 2 <= depth; it += 2) {
            step(A, Bv, 0, ring, rag);
            step(Bv, A, 1, ring, rag);
        }
        if (it < depth) {
            step(A, Bv, 0, ring, rag);
            __syncthreads();        // the next use of parity 0 may follow at once: everyone has read this one
#pragma unroll
            for (int j = 0; j < RW; ++j)
#pragma unroll
                for (int s = 0; s < NSEG; ++s) A[j][s] = Bv[j][s];
        }
    };

    bool healthy = true;
    T *src = ga, *dst = gb;
    for (int ph = 0; ph < rp.nphase; ++ph) {
        const int depth = rp.depth + (ph < rp.n_deep ? 1 : 0);
        if (ph > 0) {
            // the ghost rows went stale during the last phase: their owners have just stored them
#pragma unroll
            for (int j = 0; j < RW; ++j)
                if (!own_row[j] && !ring_row[j]) load_row(src, j);
        }
        if (ragged) {
            if (wave_has_ring) iterate(depth, std::true_type{}, std::true_type{});
            else iterate(depth, std::false_type{}, std::true_type{});
        } else {
            if (wave_has_ring) iterate(depth, std::true_type{}, std::false_type{});
            else iterate(depth, std::false_type{}, std::false_type{});
        }
        const bool last_phase = ph + 1 == rp.nphase;
        if (last_phase && !single)
            healthy = healthy && __hip_atomic_load(&rp.sync[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u;
#pragma unroll
        for (int j = 0; j < RW; ++j) {
            if (!own_row[j]) continue;
#pragma unroll
            for (int s = 0; s < NSEG; ++s)
                if (active[s]) {
                    V out = A[j][s];
                    if (!healthy) {
#pragma unroll
                        for (int e = 0; e < NV; ++e) out[e] = __builtin_nan("");
                    }
                    *(V *)(dst + row_off[j] + col_off[s]) = out;
                }
        }
        if (!last_phase)
            healthy = resident_grid_barrier(rp.sync, (unsigned)(ph + 1) * gridDim.x, rp.spin_limit, &barrier_ok) && healthy;
        T *t = src; src = dst; dst = t;
    }
    if (single && !rp.residual) return;

    // ---- residual norm of the grid just produced (A): sum over the owned rows of (W+E+S+N - 4u)^2.  The rows
    // next to the owned ones are exact: the host gives d one more than the deepest phase when it asks for this.
    __shared__ double red[RES_WAVES];
    double tot = 0.0;
    if (rp.residual) {
        __syncthreads();                            // the last iteration's border rows have been read
#pragma unroll
        for (int s = 0; s < NSEG; ++s) {
            xch[0][wave][0][s][lane] = A[0][s];
            xch[0][wave][1][s][lane] = A[RW - 1][s];
        }
        __syncthreads();
        double acc = 0.0;
#pragma unroll
        for (int j = 0; j < RW; ++j) {
            if (!own_row[j]) continue;              // wave-uniform
            const T left = from_prev_lane(A[j][NSEG - 1][NV - 1], edge_w[j]);
            const T right = from_next_lane(A[j][0][0], edge_e[j]);
#pragma unroll
            for (int s = 0; s < NSEG; ++s) {
                const V up = j == 0 ? xch[0][wave_up][1][s][lane] : A[j == 0 ? 0 : j - 1][s];
                const V dn = j == RW - 1 ? xch[0][wave_dn][0][s][lane] : A[j == RW - 1 ? j : j + 1][s];
#pragma unroll
                for (int e = 0; e < NV; ++e) {
                    const T w = e > 0 ? A[j][s][e - 1] : s > 0 ? A[j][s > 0 ? s - 1 : 0][NV - 1] : left;
                    T ea = e < NV - 1 ? A[j][s][e + 1] : s < NSEG - 1 ? A[j][s < NSEG - 1 ? s + 1 : s][0] : right;
                    if (e == NV - 1) ea = has_last[s] ? edge_e[j] : ea;
                    const T res = ((w + ea) + (up[e] + dn[e])) - Coef<T>::four * A[j][s][e];
                    const double rd = (double)res;
                    if (active[s]) acc += rd * rd;
                }
            }
        }
        tot = wg_sum(acc, red);                     // valid in thread 0
    }
    if (single) {
        if (threadIdx.x == 0) *rp.residual = sqrt(tot);
        return;
    }
    // ---- this workgroup has finished; the last one to say so closes the launch
    if (threadIdx.x == 0) {
        if (rp.residual) {
            __hip_atomic_store(&rp.partial[blockIdx.x], healthy ? tot : __builtin_nan(""), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        }
        const unsigned before = __hip_atomic_fetch_add(&rp.sync[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool last = before == gridDim.x - 1;
        if (last && rp.residual) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");     // before the others' sums are read
        barrier_ok = last ? 1 : 0;
    }
    __syncthreads();
    if (!barrier_ok) return;
    if (rp.residual) {
        double v = 0.0;
        for (unsigned i = threadIdx.x; i < gridDim.x; i += blockDim.x)
            v += __hip_atomic_load(&rp.partial[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const double sum = wg_sum(v, red);
        if (threadIdx.x == 0) *rp.residual = sqrt(sum);
    }
    if (threadIdx.x < 3) __hip_atomic_store(&rp.sync[threadIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace jk
