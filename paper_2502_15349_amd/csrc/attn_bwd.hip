// Kernel instantiations and launch of the backward pass (see attn_bwd_kernel.hpp).
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

template <int DQK, int DV, int NORM, bool CAUSAL, int OUT, bool BIAS>
hipError_t launch_one(const BwdParams& p, const DecayTable& dt, hipStream_t s) {
  typedef BwdCfg<DQK, DV, NORM, CAUSAL, OUT, BIAS> C;
  const int heads = C::KV_SIDE ? p.H_kv : p.H_q, L = C::KV_SIDE ? p.L_k : p.L_q;
  hipLaunchKernelGGL(attn_bwd_kernel<C>, dim3((unsigned)(p.B * heads * ((L + C::OWN - 1) / C::OWN))), dim3(C::THREADS), 0, s, p, dt);
  return hipGetLastError();
}

template <int DQK, int DV, int NORM, bool CAUSAL>
hipError_t launch_pair(const BwdParams& p, const DecayTable& dt, hipStream_t s) {
  // the bias tensor comes with softmax, sigmoid and no normalization, and not with head dims 128/256
  constexpr bool kBiasBuilt = (NORM == NORM_SOFTMAX || NORM == NORM_SIGMOID || NORM == NORM_NONE) && !(DQK == 128 && DV == 256);
  if (p.bias != nullptr) {
    if constexpr (kBiasBuilt) {
      const hipError_t e = launch_one<DQK, DV, NORM, CAUSAL, BWD_DKV, true>(p, dt, s);
      if (e != hipSuccess) return e;
      return launch_one<DQK, DV, NORM, CAUSAL, BWD_DQ, true>(p, dt, s);
    } else {
      return hipErrorInvalidValue;
    }
  }
  const hipError_t e = launch_one<DQK, DV, NORM, CAUSAL, BWD_DKV, false>(p, dt, s);
  if (e != hipSuccess) return e;
  return launch_one<DQK, DV, NORM, CAUSAL, BWD_DQ, false>(p, dt, s);
}

template <int DQK, int DV, int NORM>
hipError_t launch_norm(const BwdParams& p, const DecayTable& dt, int causal, hipStream_t s) {
  return causal ? launch_pair<DQK, DV, NORM, true>(p, dt, s) : launch_pair<DQK, DV, NORM, false>(p, dt, s);
}

template <int DQK, int DV>
hipError_t launch_dims(const BwdParams& p, const DecayTable& dt, int norm, int causal, hipStream_t s) {
  switch (norm) {
    case NORM_SOFTMAX: return launch_norm<DQK, DV, NORM_SOFTMAX>(p, dt, causal, s);
    case NORM_SIGMOID: return launch_norm<DQK, DV, NORM_SIGMOID>(p, dt, causal, s);
    case NORM_ABSSUM: return launch_norm<DQK, DV, NORM_ABSSUM>(p, dt, causal, s);
    case NORM_ABS_OF_SUM: return launch_norm<DQK, DV, NORM_ABS_OF_SUM>(p, dt, causal, s);
    case NORM_NONE: return launch_norm<DQK, DV, NORM_NONE>(p, dt, causal, s);
    case BWD_NORM_NONE_RELU: return launch_norm<DQK, DV, BWD_NORM_NONE_RELU>(p, dt, causal, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

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
  if (dqk == 64 && dv == 64) return launch_dims<64, 64>(p, dt, norm, causal, stream);
  if (dqk == 128 && dv == 128) return launch_dims<128, 128>(p, dt, norm, causal, stream);
  if (dqk == 192 && dv == 128) return launch_dims<192, 128>(p, dt, norm, causal, stream);
  if (dqk == 128 && dv == 256) return launch_dims<128, 256>(p, dt, norm, causal, stream);
  return hipErrorInvalidValue;
}

}  // namespace ae
