// Decoding shapes with split keys (paper Table 2, the decoding row: one query row per head against thousands of
// keys; Section 4.1, online row-norm interface: the state of two key blocks is combined by the rule of the online
// softmax).  One query row has no use for matrix units or for a 256-row tile: the work is reading K and V once, so
// the kernel is a stream.  A workgroup owns one (batch, q head, key range) and its four wavefronts take the range's
// keys four at a time; 16 lanes share a key, each holding D / 16 consecutive elements of its row (one 16-byte load
// per lane for 128 elements, an 8-byte one more for 192), so every load instruction of a wavefront reads four whole
// rows, contiguous in memory.  The dot product is D / 16 multiply-adds and four data-parallel-primitive adds inside
// the row of 16 lanes; every group of 16 lanes keeps an online softmax state of its own (reference, sum, D_v / 16
// output columns), and the 16 states of a workgroup are combined through LDS at the end into one normalised partial
// row and its log-sum-exp, which attn_merge_kernel combines over the key ranges.  Loads run one block of
// kDecodeDepth steps ahead of the arithmetic (registers only, no LDS tiles, no barrier inside the loop).
#include <hip/hip_runtime.h>

#include "attn_decode.hpp"

namespace ae {
namespace {

constexpr int kDecodeDepth = 4;  // steps (of 4 keys per wavefront) loaded ahead

template <int N>
struct RowPiece {  // N bf16 elements of a row, N = 4, 8 or 12
  uint32_t w[N / 2];
};

template <int N>
__device__ __forceinline__ RowPiece<N> load_piece(const __bf16* row, int sub) {
  RowPiece<N> r;
  if constexpr (N == 4) {
    const uint2 a = *reinterpret_cast<const uint2*>(row + 4 * sub);
    r.w[0] = a.x, r.w[1] = a.y;
  } else {
    const uint4 a = *reinterpret_cast<const uint4*>(row + 8 * sub);
    r.w[0] = a.x, r.w[1] = a.y, r.w[2] = a.z, r.w[3] = a.w;
    if constexpr (N == 12) {
      const uint2 b = *reinterpret_cast<const uint2*>(row + 128 + 4 * sub);
      r.w[4] = b.x, r.w[5] = b.y;
    }
  }
  return r;
}

// element e of a piece as fp32 (bf16 is the upper half of an fp32)
template <int N>
__device__ __forceinline__ float elem(const RowPiece<N>& r, int e) {
  const uint32_t w = r.w[e / 2];
  return __builtin_bit_cast(float, (e & 1) ? (w & 0xffff0000u) : (w << 16));
}

// sum over the 16 lanes of a row, left in every one of them
__device__ __forceinline__ float row16_sum(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xb1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4e, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xf, 0xf, false));  // row_half_mirror
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xf, 0xf, false));  // row_mirror
  return x;
}

constexpr float kNone = -1e30f;  // "no key yet": finite, so that differences of references stay finite

template <int DQK, int DV>
__global__ __launch_bounds__(256) void attn_decode_kernel(const DecodeParams p) {
  constexpr int NK = DQK / 16, NV = DV / 16;
  __shared__ float red[16][DV + 2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, grp = lane >> 4, sub = lane & 15;
  const int c = blockIdx.x % p.n_splits;                 // key range
  const int64_t row = blockIdx.x / p.n_splits;           // (batch, q head)
  const int b = (int)(row / p.H_q), hq = (int)(row % p.H_q), hk = hq / p.g;
  const int j_begin = c * p.split_keys, j_end = min(p.L_k, j_begin + p.split_keys);
  const __bf16* Kh = p.K + b * p.ks[0] + hk * p.ks[1];
  const __bf16* Vh = p.V + b * p.vs[0] + hk * p.vs[1];

  // the query row, in log2 units: scale * log2(e) * q, fp32
  float q[NK];
  {
    const RowPiece<NK> qp = load_piece<NK>(p.Q + b * p.qs[0] + hq * p.qs[1], sub);
#pragma unroll
    for (int e = 0; e < NK; ++e) q[e] = elem(qp, e) * p.c;
  }
  float m = kNone, l = 0.f, acc[NV];
#pragma unroll
  for (int e = 0; e < NV; ++e) acc[e] = 0.f;

  // step s of this wavefront: keys j_begin + (4 s + wave) * 4 + grp
  const int n_steps = (j_end - j_begin + 15) / 16;
  auto key_of = [&](int s) { return j_begin + (4 * s + wave) * 4 + grp; };
  RowPiece<NK> kbuf[2][kDecodeDepth];
  RowPiece<NV> vbuf[2][kDecodeDepth];
  auto issue = [&](int s0, int which) {
#pragma unroll
    for (int u = 0; u < kDecodeDepth; ++u) {
      const int j = min(key_of(s0 + u), p.L_k - 1);  // (keys past the end are read as the last key and get weight 0)
      kbuf[which][u] = load_piece<NK>(Kh + (int64_t)j * p.ks[2], sub);
      vbuf[which][u] = load_piece<NV>(Vh + (int64_t)j * p.vs[2], sub);
    }
  };
  auto work = [&](int s0, int which) {
#pragma unroll
    for (int u = 0; u < kDecodeDepth; ++u) {
      float x = 0.f;
#pragma unroll
      for (int e = 0; e < NK; ++e) x = __builtin_fmaf(q[e], elem(kbuf[which][u], e), x);
      x = row16_sum(x) + p.b2;
      const bool live = key_of(s0 + u) < j_end;
      x = live ? x : kNone;
      const float mn = fmaxf(m, x);
      const float alpha = __builtin_amdgcn_exp2f(m - mn);          // 1 while the reference stands
      const float w = live ? __builtin_amdgcn_exp2f(x - mn) : 0.f;
      m = mn;
      l = l * alpha + w;
#pragma unroll
      for (int e = 0; e < NV; ++e) acc[e] = __builtin_fmaf(w, elem(vbuf[which][u], e), acc[e] * alpha);
    }
  };
  // blocks of kDecodeDepth steps, the loads of block n + 1 in flight while block n is worked on
  const int n_blocks = (n_steps + kDecodeDepth - 1) / kDecodeDepth;
  if (n_blocks > 0) issue(0, 0);
  for (int n = 0; n < n_blocks; n += 2) {
    if (n + 1 < n_blocks) issue((n + 1) * kDecodeDepth, 1);
    work(n * kDecodeDepth, 0);
    if (n + 1 < n_blocks) {
      if (n + 2 < n_blocks) issue((n + 2) * kDecodeDepth, 0);
      work((n + 1) * kDecodeDepth, 1);
    }
  }

  // ---- the 16 states of the workgroup (4 wavefronts x 4 rows of lanes) into one ----
  {
    float* mine = red[4 * wave + grp];
#pragma unroll
    for (int e = 0; e < NV; ++e) mine[NV * sub + e] = acc[e];
    if (sub == 0) {
      mine[DV] = m;
      mine[DV + 1] = l;
    }
  }
  __syncthreads();
  if (threadIdx.x < DV) {
    const int d = threadIdx.x;
    float M = kNone;
#pragma unroll
    for (int s = 0; s < 16; ++s) M = fmaxf(M, red[s][DV]);
    float L = 0.f, o = 0.f;
#pragma unroll
    for (int s = 0; s < 16; ++s) {
      const float f = __builtin_amdgcn_exp2f(red[s][DV] - M);
      L += f * red[s][DV + 1];
      o += f * red[s][d];
    }
    const bool any = L > 0.f;
    p.ws_o[((int64_t)c * p.rows + row) * DV + d] = any ? o / L : 0.f;
    if (d == 0) p.ws_lse[(int64_t)c * p.rows + row] = any ? (M + __builtin_amdgcn_logf(L)) * 0.6931471805599453f : -INFINITY;
  }
}

template <int DQK, int DV>
hipError_t launch(const DecodeParams& p, hipStream_t s) {
  const int64_t grid = p.rows * p.n_splits;
  if (grid > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_decode_kernel<DQK, DV>), dim3((unsigned)grid), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace

bool decode_supported(int dqk, int dv) { return (dqk == 64 && dv == 64) || (dqk == 128 && dv == 128) || (dqk == 192 && dv == 128); }

hipError_t launch_decode(const DecodeParams& p, int dqk, int dv, hipStream_t s) {
  if (p.n_splits < 1 || p.split_keys < 1 || p.rows < 1) return hipErrorInvalidValue;
  if (dqk == 64 && dv == 64) return launch<64, 64>(p, s);
  if (dqk == 128 && dv == 128) return launch<128, 128>(p, s);
  if (dqk == 192 && dv == 128) return launch<192, 128>(p, s);
  return hipErrorInvalidValue;
}

}  // namespace ae
