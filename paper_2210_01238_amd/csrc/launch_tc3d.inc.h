// Dispatch over the compiled variants of the workgroup-cooperative 3-D temporal-blocking kernel
// (sweep3d_tc_kernel) for one element type.  Included by launch_tc3d_f64.hip / _f32.hip.
#include "launchers.h"

namespace jk {

template <typename T>
static hipError_t tc3d_dispatch(int depth, int mode, const LaunchArgs &a)
{
    const dim3 grid(a.nwg), block(TC3D_WAVES * WAVE);
    const T *src = (const T *)a.src;
    T *dst = (T *)a.dst;
    // template arguments after the mode: depth, rows per wavefront (tc3d_rows_per_wave), wavefronts per
    // workgroup, and the occupancy the compiler must fit (wavefronts per SIMD)
#define JK_L(MODE_, TB_) \
    hipLaunchKernelGGL((sweep3d_tc_kernel<T, MODE_, TB_, tc3d_rows_per_wave(TB_), TC3D_WAVES, 2>), grid, block, 0, a.st, a.g, a.sp, a.aux, src, dst, a.partial)
#define JK_V(MODE_)                              \
    do {                                         \
        if (depth == 2) JK_L(MODE_, 2);          \
        else if (depth == 3) JK_L(MODE_, 3);     \
        else if (depth == 4) {                   \
            /* fp32 passes stop at depth 3 */      \
            if constexpr (sizeof(T) == 8) JK_L(MODE_, 4); \
            else return hipErrorInvalidValue;    \
        } else return hipErrorInvalidValue;      \
    } while (0)
    if (mode == MODE_UPDATE) JK_V(MODE_UPDATE);
    else if (mode == MODE_BOTH) JK_V(MODE_BOTH);
    else return hipErrorInvalidValue;
#undef JK_V
#undef JK_L
    return hipGetLastError();
}

}  // namespace jk
