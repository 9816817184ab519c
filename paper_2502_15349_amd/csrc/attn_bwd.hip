// Launch of the backward pass (see attn_bwd_kernel.hpp): the delta kernel and the dispatch to the per-head-dim
// instantiation files.
#include "bwd.hpp"

namespace ae {
namespace {

// delta_i = dO_i . O_i, one wavefront per row.  Abs-sum family: what the main kernels subtract is
// delta_i only where the normalizer is above its clamp (r_i > 1), with the sign of the row sum for the
// |sum| normalizer (norm: NORM_*).
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const BwdParams p, int D_v, int norm) {
  const int64_t rows = (int64_t)p.B * p.H_q * p.L_q;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int lane = threadIdx.x & 63;
  const int i = (int)(r % p.L_q), hq = (int)((r / p.L_q) % p.H_q), b = (int)(r / ((int64_t)p.L_q * p.H_q));
  const int64_t ob = b * p.os[0] + hq * p.os[1] + (int64_t)i * p.os[2];
  float acc = 0.f;
  for (int d = lane; d < D_v; d += 64) {
    const float o = p.o_bf16 ? (float)static_cast<const __bf16*>(p.O)[ob + d] : static_cast<const float*>(p.O)[ob + d];
    acc += o * (float)p.dO[r * D_v + d];
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) acc += __shfl_xor(acc, s);
  if (norm == NORM_ABSSUM || norm == NORM_ABS_OF_SUM) {
    const float st = p.lse[r];
    acc = fabsf(st) > 1.f ? (norm == NORM_ABS_OF_SUM && st < 0.f ? -acc : acc) : 0.f;
  }
  if (lane == 0) p.delta[r] = acc;
}

}  // namespace

hipError_t launch_backward_64_64(const BwdParams&, const DecayTable&, int, int, hipStream_t);
hipError_t launch_backward_128_128(const BwdParams&, const DecayTable&, int, int, hipStream_t);
hipError_t launch_backward_192_128(const BwdParams&, const DecayTable&, int, int, hipStream_t);
hipError_t launch_backward_128_256(const BwdParams&, const DecayTable&, int, int, hipStream_t);

bool backward_supported(int dqk, int dv, int norm) {
  const bool dims = (dqk == 64 && dv == 64) || (dqk == 128 && dv == 128) || (dqk == 192 && dv == 128) || (dqk == 128 && dv == 256);
  return dims && (norm == NORM_SOFTMAX || norm == NORM_SIGMOID || norm == NORM_ABSSUM || norm == NORM_ABS_OF_SUM ||
                  norm == NORM_NONE || norm == BWD_NORM_NONE_RELU);
}

hipError_t launch_backward(const BwdParams& p, const DecayTable& dt, int dqk, int dv, int norm, int causal, hipStream_t stream) {
  if (norm == NORM_SOFTMAX || norm == NORM_ABSSUM || norm == NORM_ABS_OF_SUM) {
    const int64_t rows = (int64_t)p.B * p.H_q * p.L_q;
    hipLaunchKernelGGL(attn_bwd_delta_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, p, dv, norm);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (dqk == 64 && dv == 64) return launch_backward_64_64(p, dt, norm, causal, stream);
  if (dqk == 128 && dv == 128) return launch_backward_128_128(p, dt, norm, causal, stream);
  if (dqk == 192 && dv == 128) return launch_backward_192_128(p, dt, norm, causal, stream);
  if (dqk == 128 && dv == 256) return launch_backward_128_256(p, dt, norm, causal, stream);
  return hipErrorInvalidValue;
}

}  // namespace ae
