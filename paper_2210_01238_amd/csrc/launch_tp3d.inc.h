// Dispatch over the compiled variants of the 3-D pipelined temporal-blocking kernel
// (sweep3d_tp_kernel) for one element type.  Included by launch_tp3d_f64.hip / _f32.hip.
#include "launchers.h"

namespace jk {

template <typename T>
static hipError_t tp3d_dispatch(int depth, int rows_per_wave, int mode, const LaunchArgs &a)
{
    const dim3 grid(a.nwg), block(WG);
    const T *src = (const T *)a.src;
    T *dst = (T *)a.dst;
    // template arguments after the mode: depth, rows per wavefront, planes loaded ahead, and the occupancy
    // the compiler must fit (wavefronts per SIMD; chosen so that nothing spills)
#define JK_L(MODE_, TB_, RW_, PF_, MINW_) \
    hipLaunchKernelGGL((sweep3d_tp_kernel<T, MODE_, TB_, RW_, PF_, MINW_>), grid, block, 0, a.st, a.g, a.sp, a.aux, src, dst, a.partial)
#define JK_V(MODE_)                                                        \
    do {                                                                   \
        if (depth == 2 && rows_per_wave == 2) JK_L(MODE_, 2, 2, 1, 3);     \
        else if (depth == 2 && rows_per_wave == 4) JK_L(MODE_, 2, 4, 1, 2);\
        else if (depth == 3 && rows_per_wave == 2) {                       \
            /* fp32 passes of this kernel stop at depth 2 */                 \
            if constexpr (sizeof(T) == 8) JK_L(MODE_, 3, 2, 1, 2);         \
            else return hipErrorInvalidValue;                              \
        }                                                                  \
        else return hipErrorInvalidValue;                                  \
    } while (0)
    if (mode == MODE_UPDATE) JK_V(MODE_UPDATE);
    else if (mode == MODE_BOTH) JK_V(MODE_BOTH);
    else return hipErrorInvalidValue;
#undef JK_V
#undef JK_L
    return hipGetLastError();
}

}  // namespace jk
