// Decoding shapes with split keys: what ae_attn.hip needs to know of attn_decode.hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ae {
struct DecodeParams {
  const __bf16* Q;       // one row per (batch, q head): element strides qs[] = {batch, head}
  const __bf16* K;       // element strides ks[] = {batch, head, row}; rows 16-byte aligned
  const __bf16* V;
  float* ws_o;           // [n_splits, rows, D_v]: normalised partial rows
  float* ws_lse;         // [n_splits, rows]: their log-sum-exp (natural logarithm; -inf for a range without keys)
  int64_t qs[2], ks[3], vs[3];
  int64_t rows;          // B * H_q
  int H_q, g, L_k;       // g = H_q / H_kv
  int n_splits, split_keys;  // key range c: [c * split_keys, (c + 1) * split_keys)
  float c;               // scale * log2(e)
  float b2;              // constant bias * log2(e)
};
// softmax with a plain or constant-bias modification, one query row per head, every key visible
bool decode_supported(int dqk, int dv);
hipError_t launch_decode(const DecodeParams& p, int dqk, int dv, hipStream_t stream);
}  // namespace ae
