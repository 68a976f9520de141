// Dispatch over the depths of the pipelined temporal-blocking kernel (sweep2d_tp_kernel) for
// one element type.  Included by launch_tp_f64.hip and launch_tp_f32.hip.
#include "launchers.h"

namespace jk {

template <typename T>
static hipError_t tp_dispatch(int depth, int mode, const LaunchArgs &a)
{
    const dim3 grid(a.nwg), block(WG);
    const T *src = (const T *)a.src;
    T *dst = (T *)a.dst;
    // Template arguments after the depth: rows loaded ahead (4; 8 measured no faster), and the
    // wavefronts per SIMD the compiler has to fit the kernel's registers into: 3 up to depth 8 (150
    // VGPRs at depth 8, about 18 more with the residual), 2 beyond (215 at depth 12).  On large grids the
    // launch lets only 2 per SIMD run (see the LDS request in launch_tp).
#define JK_MINW(TB_) ((TB_) >= 9 ? 2 : 3)
    // a.lds (it only limits the workgroups per CU) is checked, and allowed for the kernel if above 64 KiB, by lds_for_launch
#define JK_L(MODE_, TB_)                                                                                           \
    do {                                                                                                           \
        unsigned lds_ = 0;                                                                                         \
        const hipError_t e_ = lds_for_launch<sweep2d_tp_kernel<T, MODE_, TB_, 4, JK_MINW(TB_)>>(a, WG, &lds_);     \
        if (e_ != hipSuccess) return e_;                                                                           \
        hipLaunchKernelGGL((sweep2d_tp_kernel<T, MODE_, TB_, 4, JK_MINW(TB_)>), grid, block, lds_, a.st, a.g,      \
                           a.sp, src, dst, a.partial);                                                             \
    } while (0)
#define JK_D(MODE_)                         \
    switch (depth) {                        \
    case 3: JK_L(MODE_, 3); break;          \
    case 4: JK_L(MODE_, 4); break;          \
    case 5: JK_L(MODE_, 5); break;          \
    case 6: JK_L(MODE_, 6); break;          \
    case 7: JK_L(MODE_, 7); break;          \
    case 8: JK_L(MODE_, 8); break;          \
    case 9: JK_L(MODE_, 9); break;          \
    case 10: JK_L(MODE_, 10); break;        \
    case 11: JK_L(MODE_, 11); break;        \
    case 12: JK_L(MODE_, 12); break;        \
    default: return hipErrorInvalidValue;   \
    }
    if (mode == MODE_UPDATE) { JK_D(MODE_UPDATE) }
    else if (mode == MODE_BOTH) { JK_D(MODE_BOTH) }
    else return hipErrorInvalidValue;
#undef JK_D
#undef JK_L
#undef JK_MINW
    return hipGetLastError();
}

}  // namespace jk
