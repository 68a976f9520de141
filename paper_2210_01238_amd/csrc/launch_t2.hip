// Two iterations per pass (sweep2d_t2_kernel), 8-row strips, streaming stores.
#include "launchers.h"

namespace jk {

template <typename T>
static hipError_t t2_dispatch(int mode, const LaunchArgs &a)
{
    const dim3 grid(a.nwg), block(WG);
    const T *src = (const T *)a.src;
    T *dst = (T *)a.dst;
    if (mode == MODE_UPDATE)
        hipLaunchKernelGGL((sweep2d_t2_kernel<T, MODE_UPDATE, T2_ROWS, 2>), grid, block, 0, a.st, a.g, a.sp, src, dst, a.partial);
    else if (mode == MODE_BOTH)
        hipLaunchKernelGGL((sweep2d_t2_kernel<T, MODE_BOTH, T2_ROWS, 2>), grid, block, 0, a.st, a.g, a.sp, src, dst, a.partial);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_t2(bool f64, int mode, const LaunchArgs &a)
{
    return f64 ? t2_dispatch<double>(mode, a) : t2_dispatch<float>(mode, a);
}

}  // namespace jk
