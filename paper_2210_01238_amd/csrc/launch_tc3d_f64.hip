#include "launch_tc3d.inc.h"
namespace jk {
hipError_t launch_tc3d_f64(int depth, int mode, const LaunchArgs &a) { return tc3d_dispatch<double>(depth, mode, a); }
}
