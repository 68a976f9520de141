#include "launch_2d.inc.h"
namespace jk {
hipError_t launch_sweep2d_f64(int mode, int unroll, int nt, const LaunchArgs &a) { return sweep2d_dispatch<double>(mode, unroll, nt, a); }
}
