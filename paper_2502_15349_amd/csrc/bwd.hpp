// Backward pass: what ae_attn.hip needs to know of attn_bwd.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "attn_bwd_kernel.hpp"

namespace ae {
// True if kernels exist for this combination (norm: a NORM_* value or BWD_NORM_NONE_RELU).
bool backward_supported(int dqk, int dv, int norm);
// Launches delta (softmax), the key-side kernel (dK, dV) and the query-side kernel (dQ) on the stream.
// dt: log2 of the per-q-head decay rates (abs-sum family with head decay; zeros otherwise).
hipError_t launch_backward(const BwdParams& p, const DecayTable& dt, int dqk, int dv, int norm, int causal, hipStream_t stream);
}  // namespace ae
