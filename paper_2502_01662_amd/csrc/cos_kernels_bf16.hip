// cos_kernels_bf16.hip -- the kernels instantiated for logits stored as uint16_t.
#include "cos_launch.h"

namespace cosv {
cos_status_t run_bf16(const Params& p, const LaunchPlan& lp) { return run_kernels<uint16_t>(p, lp); }
}  // namespace cosv
