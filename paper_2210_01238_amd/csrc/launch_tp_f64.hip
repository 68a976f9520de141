#include "launch_tp.inc.h"
namespace jk {
hipError_t launch_tp_f64(int depth, int mode, const LaunchArgs &a) { return tp_dispatch<double>(depth, mode, a); }
}
