#include "launch_stack.inc.h"
namespace jk {
hipError_t launch_stack_f64(int rows, int waves, const LaunchArgs &a) { return stack_dispatch<double>(rows, waves, a); }
}
