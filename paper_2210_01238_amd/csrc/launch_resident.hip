// Compiled variants of resident2d_kernel (all iterations of a call in one launch, small 2-D grids).
#include "resident_kernel.h"

namespace jk {

template <typename T>
static hipError_t resident_dispatch(int nseg, int rows_per_wave, const ResidentLaunch &a)
{
    const dim3 grid(a.nwg), block(RES_WAVES * WAVE);
    T *ga = (T *)a.in, *gb = (T *)a.out;
#define JK_L(NSEG_, RW_) \
    hipLaunchKernelGGL((resident2d_kernel<T, NSEG_, RW_>), grid, block, 0, a.st, a.g, a.rp, ga, gb)
    // two register sets of rows x vectors: 4 rows of 2 vectors would not fit the 128 registers of a 1024-thread workgroup
    if (nseg == 1) {
        switch (rows_per_wave) {
        case 1: JK_L(1, 1); break;
        case 2: JK_L(1, 2); break;
        case 3: JK_L(1, 3); break;
        case 4: JK_L(1, 4); break;
        default: return hipErrorInvalidValue;
        }
    } else if (nseg == 2) {
        switch (rows_per_wave) {
        case 1: JK_L(2, 1); break;
        case 2: JK_L(2, 2); break;
        case 3: JK_L(2, 3); break;
        default: return hipErrorInvalidValue;
        }
    } else return hipErrorInvalidValue;
#undef JK_L
    return hipGetLastError();
}

hipError_t launch_resident(bool f64, int nseg, int rows_per_wave, const ResidentLaunch &a)
{
    return f64 ? resident_dispatch<double>(nseg, rows_per_wave, a) : resident_dispatch<float>(nseg, rows_per_wave, a);
}

}  // namespace jk
