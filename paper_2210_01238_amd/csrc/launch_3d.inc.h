// Dispatch over the compiled variants of sweep3d_kernel for one element type.
// Included by launch_3d_f64.hip and launch_3d_f32.hip.  Streaming loads are never useful in
// 3-D (every row is re-read as somebody's neighbour), so only the store bit of nt is honoured.
#include "launchers.h"

namespace jk {

template <typename T>
static hipError_t sweep3d_dispatch(int mode, int rows_per_wave, int unroll, int nt, const LaunchArgs &a)
{
    const dim3 grid(a.nwg), block(WG);
    const T *src = (const T *)a.src;
    T *dst = (T *)a.dst;
#define JK_P(MODE_, RW_, U_, NT_, PULL_, NVEC_)                                                                     \
    do {                                                                                                            \
        unsigned lds_ = 0;                                                                                          \
        const hipError_t e_ = lds_for_launch<sweep3d_kernel<T, MODE_, RW_, U_, NT_, PULL_, NVEC_>>(a, WG, &lds_);   \
        if (e_ != hipSuccess) return e_;                                                                            \
        hipLaunchKernelGGL((sweep3d_kernel<T, MODE_, RW_, U_, NT_, PULL_, NVEC_>), grid, block, lds_, a.st, a.g,    \
                           a.sp, src, dst, a.partial);                                                              \
    } while (0)
    // the read-only residual pass always pulls (no variant of it reads halo cells); updates in either way
#define JK_K(MODE_, RW_, U_, NT_, NVEC_)                                                                            \
    do {                                                                                                            \
        if (MODE_ == MODE_RESIDUAL || a.sp.pull) JK_P(MODE_, RW_, U_, NT_, true, NVEC_);                            \
        else if constexpr (MODE_ != MODE_RESIDUAL) JK_P(MODE_, RW_, U_, NT_, false, NVEC_);                         \
    } while (0)
    // a.aux = 1: fp32 rows of at most 128 elements, 2 elements per lane (4 rows per wavefront only)
#define JK_L(MODE_, RW_, U_, NT_)                                                                                   \
    do {                                                                                                            \
        if constexpr (sizeof(T) == 4 && RW_ == 4) {                                                                 \
            if (a.aux == 1) JK_K(MODE_, RW_, U_, NT_, 2);                                                           \
            else JK_K(MODE_, RW_, U_, NT_, Vec<T>::N);                                                              \
        } else {                                                                                                    \
            if (a.aux == 1) return hipErrorInvalidValue;                                                            \
            JK_K(MODE_, RW_, U_, NT_, Vec<T>::N);                                                                   \
        }                                                                                                           \
    } while (0)
#define JK_NT(MODE_, RW_, U_)                 \
    do {                                      \
        if (nt & 2) JK_L(MODE_, RW_, U_, 2);  \
        else        JK_L(MODE_, RW_, U_, 0);  \
    } while (0)
#define JK_U(MODE_, RW_)                      \
    switch (unroll) {                         \
    case 1: JK_NT(MODE_, RW_, 1); break;      \
    case 2: JK_NT(MODE_, RW_, 2); break;      \
    case 4: JK_NT(MODE_, RW_, 4); break;      \
    default: return hipErrorInvalidValue;     \
    }
#define JK_RW(MODE_)                          \
    switch (rows_per_wave) {                  \
    case 1: JK_U(MODE_, 1); break;            \
    case 2: JK_U(MODE_, 2); break;            \
    case 4: JK_U(MODE_, 4); break;            \
    default: return hipErrorInvalidValue;     \
    }
    switch (mode) {
    case MODE_UPDATE: JK_RW(MODE_UPDATE); break;
    case MODE_RESIDUAL: JK_RW(MODE_RESIDUAL); break;
    case MODE_BOTH: JK_RW(MODE_BOTH); break;
    default: return hipErrorInvalidValue;
    }
#undef JK_RW
#undef JK_U
#undef JK_NT
#undef JK_L
#undef JK_K
#undef JK_P
    return hipGetLastError();
}

}  // namespace jk
