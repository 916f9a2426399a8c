// cos_kernels_f32.hip -- the kernels instantiated for logits stored as float.
#include "cos_launch.h"

namespace cosv {
cos_status_t run_f32(const Params& p, const LaunchPlan& lp) { return run_kernels<float>(p, lp); }
}  // namespace cosv
