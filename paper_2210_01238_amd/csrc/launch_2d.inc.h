// Dispatch over the compiled variants of sweep2d_kernel for one element type.
// Included by launch_2d_f64.hip and launch_2d_f32.hip.
#include "launchers.h"

namespace jk {

template <typename T>
static hipError_t sweep2d_dispatch(int mode, int unroll, int nt, const LaunchArgs &a)
{
    const dim3 grid(a.nwg), block(WG);
    const T *src = (const T *)a.src;
    T *dst = (T *)a.dst;
    // the read-only residual pass always pulls (no variant of it reads halo cells); updates in either way
#define JK_K(MODE_, U_, NT_, PULL_) \
    hipLaunchKernelGGL((sweep2d_kernel<T, MODE_, U_, NT_, PULL_>), grid, block, 0, a.st, a.g, a.sp, src, dst, a.partial)
#define JK_L(MODE_, U_, NT_)                                          \
    do {                                                              \
        if (MODE_ == MODE_RESIDUAL || a.sp.pull) JK_K(MODE_, U_, NT_, true); \
        else if constexpr (MODE_ != MODE_RESIDUAL) JK_K(MODE_, U_, NT_, false); \
    } while (0)
#define JK_NT(MODE_, U_)                      \
    do {                                      \
        if (nt & 2) JK_L(MODE_, U_, 2);       \
        else        JK_L(MODE_, U_, 0);       \
    } while (0)
#define JK_U(MODE_)                           \
    switch (unroll) {                         \
    case 1: JK_NT(MODE_, 1); break;           \
    case 2: JK_NT(MODE_, 2); break;           \
    case 4: JK_NT(MODE_, 4); break;           \
    case 8: JK_NT(MODE_, 8); break;           \
    case 16: JK_NT(MODE_, 16); break;         \
    default: return hipErrorInvalidValue;     \
    }
    switch (mode) {
    case MODE_UPDATE: JK_U(MODE_UPDATE); break;
    case MODE_RESIDUAL: JK_U(MODE_RESIDUAL); break;
    case MODE_BOTH: JK_U(MODE_BOTH); break;
    default: return hipErrorInvalidValue;
    }
#undef JK_U
#undef JK_NT
#undef JK_L
#undef JK_K
    return hipGetLastError();
}

}  // namespace jk
