// Backward kernel instantiations for D_qk = 128, D_v = 256.
#include "bwd_launch.hpp"

namespace ae {
hipError_t launch_backward_128_256(const BwdParams& p, const DecayTable& dt, int norm, int causal, hipStream_t stream) {
  return launch_dims<128, 256>(p, dt, norm, causal, stream);
}
}  // namespace ae
