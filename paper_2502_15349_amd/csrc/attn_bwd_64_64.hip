// Backward kernel instantiations for D_qk = 64, D_v = 64.
#include "bwd_launch.hpp"

namespace ae {
hipError_t launch_backward_64_64(const BwdParams& p, const DecayTable& dt, int norm, int causal, hipStream_t stream) {
  return launch_dims<64, 64>(p, dt, norm, causal, stream);
}
}  // namespace ae
