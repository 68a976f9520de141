// Internal interface between the host API (jacobi.hip) and the translation units that hold
// the compiled variants of the update kernels.  The variants are spread over several files
// only so that they compile in parallel; each launcher picks the instantiation for its
// arguments, launches it and returns hipGetLastError() (hipErrorInvalidValue if the requested
// variant is not compiled).
#pragma once
#include "jacobi_kernels.h"
#include <mutex>

namespace jk {

struct LaunchArgs {
    unsigned nwg;        // workgroups (grid size); block size is always WG
    hipStream_t st;
    Geo g;
    StripParams sp;
    const void *src;     // element type is given by the f64 flag of the call
    void *dst;
    double *partial;     // per-workgroup partial sums (residual modes), else unused
    int aux = 0;         // kernel-specific extra (3-D blocked pass: row groups per tile)
    // Workgroup limit: `lds` bytes of dynamic LDS that nobody touches are requested with the launch so that at
    // most `per_cu` workgroups share a CU (0: no limit).  The request only goes out if the occupancy query
    // confirms that it has this effect for the kernel at hand (lds_for_launch); if not, the launch runs
    // without a limit and *limit_failed is set.
    unsigned lds = 0;
    int per_cu = 0;
    int64_t *limit_failed = nullptr;
};

// Dynamic LDS to pass to the launch of KERNEL (a __global__ function; the template argument makes the cache
// below one per compiled variant): a.lds if the runtime confirms that a workgroup of `block_threads` threads
// asking for it leaves room for at most a.per_cu workgroups on a CU, else 0.  Requests above 64 KiB are
// allowed for the kernel first (once per kernel and device).  Checked once per kernel, device and size.
template <auto KERNEL>
inline hipError_t lds_for_launch(const LaunchArgs &a, int block_threads, unsigned *lds)
{
    struct Cache { unsigned allowed = 65536, checked = 0; bool ok = false; };
    constexpr int MAX_DEV = 64;
    static Cache cache[MAX_DEV];
    static std::mutex lock;
    *lds = 0;
    if (a.lds == 0 || a.per_cu <= 0) return hipSuccess;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    bool ok = false;
    if (dev >= 0 && dev < MAX_DEV) {
        std::lock_guard<std::mutex> hold(lock);
        Cache &c = cache[dev];
        if (c.checked != a.lds) {
            if (a.lds > c.allowed) {
                e = hipFuncSetAttribute((const void *)KERNEL, hipFuncAttributeMaxDynamicSharedMemorySize, (int)a.lds);
                if (e != hipSuccess) return e;
                c.allowed = a.lds;
            }
            int nb = 0;
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, KERNEL, block_threads, a.lds);
            if (e != hipSuccess) (void)hipGetLastError();
            c.ok = e == hipSuccess && nb >= 1 && nb <= a.per_cu;
            c.checked = a.lds;
        }
        ok = c.ok;
    }
    if (ok) *lds = a.lds;
    else if (a.limit_failed) *a.limit_failed = 1;
    return hipSuccess;
}

// single-step update / residual (mode: Mode; unroll 1,2,4,8,16; nt: 0 or 2)
hipError_t launch_sweep2d_f64(int mode, int unroll, int nt, const LaunchArgs &a);
hipError_t launch_sweep2d_f32(int mode, int unroll, int nt, const LaunchArgs &a);
// rows_per_wave 1,2,4; unroll 1,2,4
hipError_t launch_sweep3d_f64(int mode, int rows_per_wave, int unroll, int nt, const LaunchArgs &a);
hipError_t launch_sweep3d_f32(int mode, int rows_per_wave, int unroll, int nt, const LaunchArgs &a);
// 2-D residual pass with the wavefronts of a workgroup stacked (rows 8 per wavefront, waves 4 or 8 per
// workgroup); a.nwg = work units (tile x band x column segment), a.sp.nblk = bands per tile
hipError_t launch_stack_f64(int rows, int waves, const LaunchArgs &a);
hipError_t launch_stack_f32(int rows, int waves, const LaunchArgs &a);
// two iterations per pass (8-row strips); mode MODE_UPDATE or MODE_BOTH
constexpr int T2_ROWS = 8;
hipError_t launch_t2(bool f64, int mode, const LaunchArgs &a);
// TP_MIN..TP_MAX iterations per pass, pipelined down tall strips (overlapped wavefronts)
constexpr int TP_MIN = 3, TP_MAX = 12;
hipError_t launch_tp_f64(int depth, int mode, const LaunchArgs &a);
hipError_t launch_tp_f32(int depth, int mode, const LaunchArgs &a);

// 3-D: passes of depth 2 (2 or 4 rows per wavefront) or 3 (2 rows), pipelined along z
constexpr int TP3D_MIN = 2, TP3D_MAX = 3;
hipError_t launch_tp3d_f64(int depth, int rows_per_wave, int mode, const LaunchArgs &a);
hipError_t launch_tp3d_f32(int depth, int rows_per_wave, int mode, const LaunchArgs &a);

// 3-D, workgroup-cooperative blocked passes: rows one wavefront holds at each depth (a workgroup stores
// TC3D_WAVES * rows - 2 * depth rows per plane)
constexpr int TC3D_MIN = 2, TC3D_MAX = 4;
constexpr int TC3D_WAVES = 8;   // wavefronts per workgroup (one workgroup per CU at 2 wavefronts per SIMD)
constexpr int tc3d_rows_per_wave(int depth) { return depth == 2 ? 8 : depth == 3 ? 6 : 5; }
hipError_t launch_tc3d_f64(int depth, int mode, const LaunchArgs &a);
hipError_t launch_tc3d_f32(int depth, int mode, const LaunchArgs &a);

// All iterations of a call in one launch (small 2-D grids; resident_kernel.h).  nseg 1 or 2 column segments per
// wavefront, 1..4 rows per wavefront.  With more than one workgroup a one-wavefront kernel that zeroes the
// barrier words is launched first.
constexpr int RES_WAVES = 16;                // wavefronts per workgroup (1024 threads: one workgroup per CU)
constexpr int RES_MAX_SEG = 2;               // column segments a wavefront holds (rows of at most 2 KiB)
constexpr int RES_MAX_RW = 4;                // rows per wavefront
struct ResidentParams {
    int B;                 // rows a workgroup owns
    int d;                 // ghost rows per side
    int nphase;            // phases; the first n_deep of them run depth + 1 iterations, the others depth
    int depth, n_deep;
    unsigned spin_limit;   // polls a workgroup waits at a grid barrier before it gives up
    unsigned *sync;        // [0]: arrivals, [1]: failure flag, [2]: workgroups that have finished.  All zero between
                           // launches (the last workgroup to finish clears them); unused with one workgroup
    int copy_ring;         // also carry the Dirichlet ring from the source grid to the other one
    double *partial;       // per-workgroup sums of the residual terms (one per workgroup; unused if residual is null)
    double *residual;      // if not null: the residual norm of the final grid goes here (then d > deepest phase)
};
struct ResidentLaunch {
    unsigned nwg;
    hipStream_t st;
    Geo g;
    ResidentParams rp;
    void *in, *out;
};
hipError_t launch_resident(bool f64, int nseg, int rows_per_wave, const ResidentLaunch &a);

}  // namespace jk
