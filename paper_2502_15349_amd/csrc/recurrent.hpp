// Recurrent-pattern retention, chunk-parallel: what ae_attn.hip needs to know of retention_recurrent.hip.
#pragma once
#include <hip/hip_runtime.h>

#include "attn_kernel.hpp"

namespace ae {
// Every (batch, head) sequence is cut into chunks of `chunk` tokens (a multiple of 64); the last one may be short.
// HT holds one bf16 matrix [D_v][D_qk] per (batch, head, chunk): the state in front of that chunk, transposed
// (slot 0 is written only when the caller hands in a state).
struct RecParams {
  const __bf16 *K, *V;  // contiguous [B, H, L, D]
  __bf16* HT;           // [B*H, n_chunks, D_v, D_qk]
  const float* h_in;    // optional [B, H, D_qk, D_v]: the state in front of the first token (null: zero)
  float* h_out;         // optional [B, H, D_qk, D_v]: the state after the last token
  int B, H, L, chunk, n_chunks;
};
bool recurrent_supported(int dqk, int dv);
// The states in front of chunks 1 .. n_chunks-1 (and 0, from h_in), and the final state if asked for.
hipError_t launch_recurrent_states(const RecParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream);
// One token: state = gamma * state + k^T v (fp32 [B, H, D_qk, D_v], in place), o = scale * q state (fp32 [B, H, D_v]);
// q, k bf16 [B, H, D_qk], v bf16 [B, H, D_v].
struct RecStepParams {
  const __bf16 *q, *k, *v;
  float* state;
  float* o;
  int B, H;
  float scale;
};
hipError_t launch_recurrent_step(const RecStepParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream);
}  // namespace ae
