// The fused rollout / evaluation kernel for the 3 x 3 view (one translation unit per view size keeps the build parallel).
#include "rollout_fused.h"

namespace marl {

int32_t launch_rollout_fused_v3(int H, bool eval, const RolloutFusedArgs& a, hipStream_t s) {
  return launch_rollout_fused_tu<3>(H, eval, a, s);
}

}  // namespace marl
