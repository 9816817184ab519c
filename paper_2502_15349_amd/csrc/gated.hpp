// Recurrent pattern with per-token gates: what ae_attn.hip needs to know of gated_recurrent.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_kernel.hpp"  // DecayTable

namespace ae {
struct GatedParams {
  const __bf16* Q;          // [B, H_qk, L, D_qk]
  const __bf16* K;          // [B, H_qk, L, D_qk]
  const __bf16* V;          // [B, H, L, D_v]
  const float* log_decay;   // [B, H, L]: ln a_t <= 0; null: one constant decay per head, from the table passed beside
  const float* key_gate;    // [B, H, L] or null (ones)
  const float* h_in;        // [B, H, D_qk, D_v] fp32 or null (zero)
  float* h_out;             // the same layout, or null
  void* O;                  // [B, H, L, D_v] fp32, or bf16 if out_bf16
  int B, H, H_qk, L;
  float scale;
  int out_bf16;
};
bool gated_supported(int dqk, int dv);
// dt: log2 of the per-head decay, read only where p.log_decay is null
hipError_t launch_gated_recurrent(const GatedParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream);
}  // namespace ae
