// Layout pre-pass for the workspace entry point: V [L_k, D_v] per (batch, kv head)
// -> V^T [D_v, ldvt] (ldvt = L_k rounded up to 64, zero filled), so that the
// attention kernel can read aggregation fragments (one output column, eight
// consecutive keys) with a single 128-bit LDS load.  Bandwidth-bound; the
// operator itself (scoring, modification, normalization, aggregation) stays in
// attn_fwd_kernel.
#include "dispatch.hpp"

namespace ae {

// One workgroup transposes a 64-key x 64-column tile through LDS.
__global__ __launch_bounds__(256) void transpose_v_kernel(const __bf16* __restrict__ V, __bf16* __restrict__ Vt, int H_kv,
                                                          int L_k, int D_v, int ldvt, int64_t vs_b, int64_t vs_h,
                                                          int64_t vs_r) {
  __shared__ uint16_t tile[64][64 + 2];  // +2 elements: rows land on different banks when read by column
  const int bh = blockIdx.z, b = bh / H_kv, h = bh % H_kv;
  const int j0 = blockIdx.x * 64, d0 = blockIdx.y * 64;
  const uint16_t* src = reinterpret_cast<const uint16_t*>(V) + b * vs_b + h * vs_h;
  uint16_t* dst = reinterpret_cast<uint16_t*>(Vt) + (int64_t)bh * D_v * ldvt;
  const int tid = threadIdx.x;
  {
    // 64 keys x 4 pieces of 16 columns
    const int key = tid >> 2, c0 = (tid & 3) * 16;
    u32x4 a = {0u, 0u, 0u, 0u}, bq = {0u, 0u, 0u, 0u};
    if (j0 + key < L_k) {
      const u32x4* g = reinterpret_cast<const u32x4*>(src + (int64_t)(j0 + key) * vs_r + d0 + c0);
      a = g[0];
      bq = g[1];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      tile[key][c0 + 2 * e] = (uint16_t)(a[e] & 0xffffu);
      tile[key][c0 + 2 * e + 1] = (uint16_t)(a[e] >> 16);
      tile[key][c0 + 8 + 2 * e] = (uint16_t)(bq[e] & 0xffffu);
      tile[key][c0 + 8 + 2 * e + 1] = (uint16_t)(bq[e] >> 16);
    }
  }
  __syncthreads();
  {
    // 64 columns x 4 pieces of 16 keys
    const int d = tid >> 2, k0 = (tid & 3) * 16;
    u32x4 a, bq;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      a[e] = (uint32_t)tile[k0 + 2 * e][d] | ((uint32_t)tile[k0 + 2 * e + 1][d] << 16);
      bq[e] = (uint32_t)tile[k0 + 8 + 2 * e][d] | ((uint32_t)tile[k0 + 8 + 2 * e + 1][d] << 16);
    }
    u32x4* o = reinterpret_cast<u32x4*>(dst + (int64_t)(d0 + d) * ldvt + j0 + k0);
    o[0] = a;
    o[1] = bq;
  }
}

hipError_t launch_transpose_v(const __bf16* V, __bf16* Vt, int B, int H_kv, int L_k, int D_v, int ldvt,
                              const int64_t (&vs)[3], hipStream_t s) {
  const dim3 grid(ldvt / 64, D_v / 64, B * H_kv);
  hipLaunchKernelGGL(transpose_v_kernel, grid, dim3(256), 0, s, V, Vt, H_kv, L_k, D_v, ldvt, vs[0], vs[1], vs[2]);
  return hipGetLastError();
}

}  // namespace ae
