// Recurrent-pattern retention, chunk-parallel: what ae_attn.hip needs to know of retention_recurrent.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "attn_kernel.hpp"

namespace ae {
// Every (batch, head) sequence is cut into chunks of `chunk` tokens (a multiple of 64); the last one may be short.
// HT holds one bf16 matrix [D_v][D_qk] per (batch, head, chunk but the last): the state after that chunk,
// transposed, which the chunk behind it starts from.
struct RecParams {
  const __bf16 *K, *V;  // contiguous [B, H, L, D]
  __bf16* HT;           // [B*H, n_chunks - 1, D_v, D_qk]
  int B, H, L, chunk, n_chunks;
};
bool recurrent_supported(int dqk, int dv);
// The states after chunks 0 .. n_chunks-2 (n_chunks >= 2).
hipError_t launch_recurrent_states(const RecParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream);
}  // namespace ae
