// Recurrent pattern with per-token gates: what ae_attn.hip needs to know of gated_recurrent.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_kernel.hpp"  // DecayTable

namespace ae {
struct GatedParams {
  const __bf16* Q;          // [B, H_qk, L, D_qk]
  const __bf16* K;          // [B, H_qk, L, D_qk]
  const __bf16* V;          // [B, H_v, L, D_v] (H_v = H unless the backward pass swaps the roles of the operands)
  const float* log_decay;   // [B, H, L]: ln a_t <= 0; null: one constant decay per head, from the table passed beside
  const float* key_gate;    // [B, H, L] or null (ones): the factor g_t on the key -- or, with gate_on_output, on the
                            // output row of token t instead (the two never occur together)
  const float* h_in;        // [B, H, D_qk, D_v] fp32 or null (zero)
  float* h_out;             // the same layout, or null
  void* O;                  // [B, H, L, D_v] fp32, or bf16 if out_bf16
  int B, H, H_qk, L;
  float scale;
  int out_bf16;
  int H_v = 0;         // heads of V (0: H): H, or a divisor of it (contiguous groups of H / H_v heads read the same V head)
  int gate_on_output = 0;  // key_gate multiplies o_t, not k_t
  // Walk the tokens from the last to the first: the recurrence runs over tau = L - 1 - t, token tau's decay is
  // log_decay[t + 1] (0 for the last token of the sequence, which is the first of the walk).  Only the memory
  // addresses change.  This is the form the sums over later tokens of the backward pass take.
  int reverse = 0;
  // Segments: the walk of a (batch, head) cut into nseg pieces of seg_len tokens (a multiple of 64; the last may be
  // shorter), one workgroup each.  h_in / h_out are then [B, H, nseg, D_qk, D_v]: every segment starts from its
  // own slot and leaves its final state in its own slot -- unless h_out_last_only, where h_out is [B, H, D_qk, D_v]
  // and only the last segment writes.  nseg = 1: the whole sequence, the layouts above.
  int nseg = 1;
  int seg_len = 0;
  int h_out_last_only = 0;
  // state_only: no outputs -- only the state update is walked (O is not touched); seg_decay, if set, receives the
  // sum of the segment's log-decays, fp32 [B, H, nseg]
  int state_only = 0;
  float* seg_decay = nullptr;
};
// In place on buf [B, H, nseg, D_qk x D_v] (the segments' final states from a zero start, as a state_only walk
// leaves them): slot s becomes the state in front of segment s, given the state in front of the sequence (h_in,
// [B, H, D_qk x D_v], or null for zero) and the segments' decays.
hipError_t launch_gated_combine_segments(float* buf, const float* seg_decay, const float* h_in, int BH, int nseg, int state_elems,
                                         hipStream_t stream);
// Epilogue of the backward pass (see ae_gated_backward): per q/k head and token, over the value heads of its group,
//   dB[h, t] = q_t . dQu[h, t] - g[h, t] (k_t . X[h, t]),   dkey_gate[h, t] = k_t . X[h, t],
//   dQ[t] = sum_h dQu[h, t],   dK[t] = sum_h g[h, t] X[h, t]
// and then dlog_decay[h, t] = sum_{i >= t} dB[h, i].  dQu / X may be dQ / dK themselves where H = H_qk.
struct GatedBwdEpilogueParams {
  const __bf16* Q;      // [B, H_qk, L, D_qk]
  const __bf16* K;
  const float* dQu;     // [B, H, L, D_qk]: gradient of q per value head
  const float* X;       // [B, H, L, D_qk]: gradient of the gated key per value head
  const float* key_gate;  // [B, H, L] or null
  float* dQ;            // [B, H_qk, L, D_qk]
  float* dK;
  float* dkey_gate;     // [B, H, L] or null
  float* dB;            // [B, H, L] workspace
  float* dlog_decay;    // [B, H, L]
  int B, H, H_qk, L;
};
hipError_t launch_gated_backward_epilogue(const GatedBwdEpilogueParams& p, int dqk, hipStream_t stream);
bool gated_supported(int dqk, int dv);
// dt: log2 of the per-head decay, read only where p.log_decay is null
hipError_t launch_gated_recurrent(const GatedParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream);
}  // namespace ae
