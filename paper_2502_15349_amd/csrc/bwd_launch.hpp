// Launch templates of the backward kernels, shared by the per-head-dim instantiation files
// (attn_bwd_<D_qk>_<D_v>.hip), each of which defines one launch_backward_<D_qk>_<D_v>().
#pragma once
#include "bwd.hpp"

namespace ae {
namespace {

template <int DQK, int DV, int NORM, bool CAUSAL, int OUT, bool BIAS>
hipError_t launch_one(const BwdParams& p, const DecayTable& dt, hipStream_t s) {
  typedef BwdCfg<DQK, DV, NORM, CAUSAL, OUT, BIAS> C;
  // whole sets of `together` groups per XCD (the kernel's mapping): sets x together x 8 XCDs x workgroups per group
  const int L = C::KV_SIDE ? p.L_k : p.L_q;
  const int64_t per_group = (int64_t)((L + C::OWN - 1) / C::OWN) * (C::KV_SIDE ? 1 : p.g);
  const int64_t rounds = ((int64_t)p.B * p.H_kv + 7) / 8, tg = p.together[C::KV_SIDE ? 1 : 0];
  const int64_t grid = ((rounds + tg - 1) / tg) * tg * 8 * per_group;
  if (tg < 1 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attn_bwd_kernel<C>, dim3((unsigned)grid), dim3(C::THREADS), 0, s, p, dt);
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
}  // namespace ae
