// Dispatch over the compiled variants of residual2d_stack_kernel (2-D read-only residual pass, the wavefronts
// of a workgroup stacked and exchanging border rows through LDS) for one element type.  Included by
// launch_stack_f64.hip / _f32.hip.
#include "launchers.h"

namespace jk {

template <typename T>
static hipError_t stack_dispatch(int rows, int waves, const LaunchArgs &a)
{
    const dim3 grid(a.nwg);
    const T *src = (const T *)a.src;
#define JK_K(R_, NW_) \
    hipLaunchKernelGGL((residual2d_stack_kernel<T, R_, NW_>), grid, dim3(NW_ * WAVE), 0, a.st, a.g, a.sp, src, a.partial)
    // 16 rows per wavefront were measured too: slower than 8 in every shape
    if (rows == 8 && waves == 4) JK_K(8, 4);
    else if (rows == 8 && waves == 8) JK_K(8, 8);
    else return hipErrorInvalidValue;
#undef JK_K
    return hipGetLastError();
}

}  // namespace jk
