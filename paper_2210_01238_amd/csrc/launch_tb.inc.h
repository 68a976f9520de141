// One depth of the overlapped-wavefront temporal-blocking kernel (sweep2d_tb_kernel), both
// element types, with and without the residual of the source grid.  Included by
// launch_tb_d<k>.hip with JK_TB_DEPTH = k; one file per depth so they compile in parallel.
//
// JK_TB_MINW_*: minimum wavefronts per SIMD the compiler must fit - the largest occupancy the
// variant reaches without register spills (found by compiling each setting).
#include "launchers.h"

#ifndef JK_TB_DEPTH
#error "define JK_TB_DEPTH before including launch_tb.inc.h"
#endif

namespace jk {

template <typename T, int MINW>
static hipError_t tb_dispatch(int mode, const LaunchArgs &a)
{
    const dim3 grid(a.nwg), block(WG);
    const T *src = (const T *)a.src;
    T *dst = (T *)a.dst;
    if (mode == MODE_UPDATE)
        hipLaunchKernelGGL((sweep2d_tb_kernel<T, MODE_UPDATE, JK_TB_DEPTH, TB_ROWS, 2, MINW>), grid, block, 0, a.st, a.g,
                           a.sp, src, dst, a.partial);
    else if (mode == MODE_BOTH)
        hipLaunchKernelGGL((sweep2d_tb_kernel<T, MODE_BOTH, JK_TB_DEPTH, TB_ROWS, 2, MINW>), grid, block, 0, a.st, a.g,
                           a.sp, src, dst, a.partial);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

#define JK_TB_CAT2(a, b) a##b
#define JK_TB_CAT(a, b) JK_TB_CAT2(a, b)
hipError_t JK_TB_CAT(launch_tb_d, JK_TB_DEPTH)(bool f64, int mode, const LaunchArgs &a)
{
    return f64 ? tb_dispatch<double, JK_TB_MINW_F64>(mode, a) : tb_dispatch<float, JK_TB_MINW_F32>(mode, a);
}

}  // namespace jk
