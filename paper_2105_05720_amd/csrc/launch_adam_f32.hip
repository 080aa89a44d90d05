// Launches of the fused Adam kernels for fp32 gradient slices.
#include "launch_adam.inc.hpp"

namespace ccf {

void launch_fused_adam_f32(const cc_plan *p, const StepScalars &s, int32_t *flag, hipStream_t st, int mode)
{
    launch_fused_adam<true>(p, s, flag, st, mode);
}

}  // namespace ccf
