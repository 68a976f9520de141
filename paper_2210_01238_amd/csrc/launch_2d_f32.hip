#include "launch_2d.inc.h"
namespace jk {
hipError_t launch_sweep2d_f32(int mode, int unroll, int nt, const LaunchArgs &a) { return sweep2d_dispatch<float>(mode, unroll, nt, a); }
}
