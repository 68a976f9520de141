#include "launch_tp3d.inc.h"
namespace jk {
hipError_t launch_tp3d_f32(int depth, int rows_per_wave, int mode, const LaunchArgs &a) { return tp3d_dispatch<float>(depth, rows_per_wave, mode, a); }
}
