// Recurrent-pattern retention, chunk-parallel: what ae_attn.hip needs to know of retention_recurrent.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "attn_kernel.hpp"

namespace ae {
// One (batch, head) pair after the other is cut into chunks of `chunk` tokens (a multiple of 64); the last one may
// be short.  S and HT hold one [D_v][D_qk] matrix per (batch, head, chunk but the last): the chunk's own
// contribution to the state (fp32) and the state in front of the NEXT chunk (bf16).
struct RecParams {
  const __bf16 *Q, *K, *V;  // contiguous [B, H, L, D]
  float* O;                 // contiguous [B, H, L, D_v]; holds the intra-chunk part when the read-out kernel runs
  float* S;                 // [B*H, n_chunks - 1, D_v, D_qk]
  __bf16* HT;               // [B*H, n_chunks - 1, D_v, D_qk]
  int B, H, L, chunk, n_chunks;
  float scale;
};
bool recurrent_supported(int dqk, int dv);
// chunk states, scan over chunks, read-out of the carried state added to O; n_chunks >= 2
hipError_t launch_recurrent_inter(const RecParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream);
}  // namespace ae
