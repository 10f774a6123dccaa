// FUSED path: placeholder until the single-kernel LDS path lands.
#include "tb_kernels.h"

namespace tb {

bool plan_fused(int64_t, int64_t, int, FusedPlan*) { return false; }

hipError_t launch_fused(const Problem&, const FusedPlan&, const StatPtrs&, const ScoreParams&,
                        float*, hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace tb
