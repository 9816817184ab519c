// Backward pass: what ae_attn.hip needs to know of attn_bwd.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "attn_bwd_kernel.hpp"

namespace ae {
// True if kernels exist for this combination (norm: NORM_SOFTMAX, NORM_SIGMOID, NORM_NONE or BWD_NORM_NONE_RELU).
bool backward_supported(int dqk, int dv, int norm);
// Launches delta (softmax), the key-side kernel (dK, dV) and the query-side kernel (dQ) on the stream.
hipError_t launch_backward(const BwdParams& p, int dqk, int dv, int norm, int causal, hipStream_t stream);
}  // namespace ae
