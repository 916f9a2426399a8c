// cos_kernels_f16.hip -- the kernels instantiated for logits stored as _Float16.
#include "cos_launch.h"

namespace cosv {
cos_status_t run_f16(const Params& p, const LaunchPlan& lp) { return run_kernels<_Float16>(p, lp); }
}  // namespace cosv
