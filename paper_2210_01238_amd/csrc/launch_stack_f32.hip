#include "launch_stack.inc.h"
namespace jk {
hipError_t launch_stack_f32(int rows, int waves, const LaunchArgs &a) { return stack_dispatch<float>(rows, waves, a); }
}
