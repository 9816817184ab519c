// Launch of the backward pass (see attn_bwd_kernel.hpp): the delta kernel and the dispatch to the per-head-dim
// instantiation files.
#include "bwd.hpp"

namespace ae {
namespace {

// delta_i = dO_i . O_i.  Abs-sum family: what the main kernels subtract is delta_i only where the normalizer is
// above its clamp (r_i > 1), with the sign of the row sum for the |sum| normalizer (norm: NORM_*).
// A group of D_v / 8 lanes owns a row and every lane 8 consecutive columns (16 bytes of dO, 32 or 16 of O), a
// wavefront 64 / (D_v / 8) rows per pass and kDeltaPasses passes, all loads of which are issued before the first
// is used: the kernel only streams, and what it needs is bytes in flight.
constexpr int kDeltaPasses = 4;
template <int DV>
__global__ __launch_bounds__(256) void attn_bwd_delta_kernel(const BwdParams p, int norm) {
  constexpr int LPR = DV / 8, RPP = 64 / LPR, RPW = RPP * kDeltaPasses;  // lanes per row, rows per pass / per wavefront
  const int64_t rows = (int64_t)p.B * p.H_q * p.L_q;
  const int lane = threadIdx.x & 63, sub = lane % LPR;
  const int64_t r0 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / LPR;
  bf16x8 g[kDeltaPasses];
  f32x4 o[kDeltaPasses][2];
#pragma unroll
  for (int k = 0; k < kDeltaPasses; ++k) {
    const int64_t r = r0 + k * RPP < rows ? r0 + k * RPP : rows - 1;
    const int i = (int)(r % p.L_q), hq = (int)((r / p.L_q) % p.H_q), b = (int)(r / ((int64_t)p.L_q * p.H_q));
    const int64_t ob = b * p.os[0] + hq * p.os[1] + (int64_t)i * p.os[2] + 8 * sub;
    g[k] = *reinterpret_cast<const bf16x8*>(p.dO + r * DV + 8 * sub);
    if (p.o_bf16) {
      // (O's strides are multiples of 4 elements: 8-byte pieces)
      const bf16x4 lo = *reinterpret_cast<const bf16x4*>(static_cast<const __bf16*>(p.O) + ob);
      const bf16x4 hi = *reinterpret_cast<const bf16x4*>(static_cast<const __bf16*>(p.O) + ob + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        o[k][0][e] = (float)lo[e];
        o[k][1][e] = (float)hi[e];
      }
    } else {
      o[k][0] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p.O) + ob);
      o[k][1] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(p.O) + ob + 4);
    }
  }
#pragma unroll
  for (int k = 0; k < kDeltaPasses; ++k) {
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc += o[k][e / 4][e % 4] * (float)g[k][e];
#pragma unroll
    for (int s = LPR / 2; s >= 1; s >>= 1) acc += __shfl_xor(acc, s);
    const int64_t r = r0 + k * RPP;
    if (r < rows && sub == 0) {
      if (norm == NORM_ABSSUM || norm == NORM_ABS_OF_SUM) {
        const float st = p.lse[r];
        acc = fabsf(st) > 1.f ? (norm == NORM_ABS_OF_SUM && st < 0.f ? -acc : acc) : 0.f;
      }
      p.delta[r] = acc;
    }
  }
}

template <int DV>
hipError_t launch_delta(const BwdParams& p, int norm, hipStream_t stream) {
  constexpr int RPW = 64 / (DV / 8) * kDeltaPasses;
  const int64_t rows = (int64_t)p.B * p.H_q * p.L_q, grid = (rows + 4 * RPW - 1) / (4 * RPW);
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attn_bwd_delta_kernel<DV>, dim3((unsigned)grid), dim3(256), 0, stream, p, norm);
  return hipGetLastError();
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
    const hipError_t e = dv == 64 ? launch_delta<64>(p, norm, stream) : dv == 128 ? launch_delta<128>(p, norm, stream)
                                                                                   : launch_delta<256>(p, norm, stream);
    if (e != hipSuccess) return e;
  }
  if (dqk == 64 && dv == 64) return launch_backward_64_64(p, dt, norm, causal, stream);
  if (dqk == 128 && dv == 128) return launch_backward_128_128(p, dt, norm, causal, stream);
  if (dqk == 192 && dv == 128) return launch_backward_192_128(p, dt, norm, causal, stream);
  if (dqk == 128 && dv == 256) return launch_backward_128_256(p, dt, norm, causal, stream);
  return hipErrorInvalidValue;
}

}  // namespace ae
