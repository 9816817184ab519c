// Measurement aid: the rate at which this GPU sustains bf16 MFMAs when nothing
// else is in the way -- operands in registers, four independent accumulator
// chains per wave, two waves per SIMD -- with operand values that toggle like
// real data (constant operands draw less power and clock higher).  The figure
// puts the attention kernel's TFLOP/s next to what the matrix pipes deliver
// under the board's power limit rather than next to the nominal peak only.
#include "../../include/ae_attn.h"

#include <hip/hip_runtime.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kThreads = 512, kMfmaPerIter = 16;

__global__ __launch_bounds__(kThreads) void calib_mfma_kernel(float* sink, int iters, unsigned seed) {
  // operand bits from a per-lane integer hash: values in (-1, 1), all mantissa bits in play
  unsigned h = (blockIdx.x * kThreads + threadIdx.x) * 2654435761u + seed;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      h = h * 1664525u + 1013904223u;
      a[j][e] = (__bf16)((float)(int)(h >> 8) * (1.0f / 8388608.f) - 1.0f);
      h = h * 1664525u + 1013904223u;
      b[j][e] = (__bf16)((float)(int)(h >> 8) * (1.0f / 8388608.f) - 1.0f);
    }
  f32x16 c[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) c[n][r] = 0.f;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int r = 0; r < kMfmaPerIter; ++r)
      c[r & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r & 3], b[(r >> 2) & 3], c[r & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c[n][r];
  sink[blockIdx.x * kThreads + threadIdx.x] = s;
}

}  // namespace

extern "C" ae_status_t ae_calib_mfma_bf16(void* sink, size_t sink_bytes, int32_t workgroups, int32_t iters,
                                          double* flop, hipStream_t stream) {
  if (!sink || workgroups <= 0 || iters <= 0 || sink_bytes < (size_t)workgroups * kThreads * sizeof(float))
    return AE_ERR_INVALID_ARG;
  hipLaunchKernelGGL(calib_mfma_kernel, dim3(workgroups), dim3(kThreads), 0, static_cast<hipStream_t>(stream),
                     static_cast<float*>(sink), iters, 12345u);
  if (hipGetLastError() != hipSuccess) return AE_ERR_HIP;
  // 8 waves per workgroup, 32*32*16*2 flop per MFMA
  if (flop) *flop = (double)workgroups * (kThreads / 64) * (double)iters * kMfmaPerIter * 32768.0;
  return AE_OK;
}
