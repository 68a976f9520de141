#include "launch_3d.inc.h"
namespace jk {
hipError_t launch_sweep3d_f32(int mode, int rows_per_wave, int unroll, int nt, const LaunchArgs &a) { return sweep3d_dispatch<float>(mode, rows_per_wave, unroll, nt, a); }
}
