// Planar articulated body kernels — not built yet: the launchers report "not supported".
#include "body_kernels.hpp"

namespace envk {

hipError_t launch_body_reset(uint32_t*, int64_t, uint64_t, uint64_t, float*, hipStream_t) {
  return hipErrorNotSupported;
}
hipError_t launch_body_rollout(const BodyLaunch&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace envk
