// Recurrent pattern (Section 4.1: K@V first, then Q@h over a compressed state), chunk-parallel so that the
// matrix units do the work (Section 4.2, kernel templates for recurrent patterns): retention with a constant
// decay per head,  h_t = gamma h_{t-1} + k_t^T v_t,  o_t = scale q_t h_t.
//
// With the sequence cut into chunks of C tokens and H_c the state after chunk c:
//   o_i  = [intra-chunk part: causal decay-masked attention inside the chunk, the parallel-pattern kernel]
//        + scale gamma^(i+1) q_i H_{c-1}                         (i: position inside the chunk)   "read-out"
//   H_c  = gamma^C H_{c-1} + sum_j gamma^(C-1-j) k_j^T v_j                                        "state" + "scan"
// Three kernels here: the per-chunk sums (one MFMA contraction over the chunk's tokens), the scan over chunks
// (elementwise, fp32), and the read-out (one MFMA contraction over D_qk, added to O).  States are kept
// transposed, [D_v][D_qk], so that both contractions read their operands in 16-byte pieces.
// Every decay factor is a power of gamma with a non-negative exponent: nothing can overflow.
#include "recurrent.hpp"

namespace ae {
namespace {

constexpr int kPad = 72;  // LDS row: 64 tokens + 8 (rows stay 16-byte aligned, 144-byte stride spreads the banks)

// S_c^T[dv][dk] = sum_j V[j][dv] * gamma^(C-1-j) K[j][dk]  for the full chunks 0 .. n_chunks-2.
// One workgroup (4 waves) per (batch*head, chunk); wave w owns the (w>>1) half of dv and the (w&1) half of dk.
template <int DK, int DV>
__global__ __launch_bounds__(256) void rec_state_kernel(const RecParams p, const DecayTable dt) {
  __shared__ __attribute__((aligned(16))) __bf16 VT[DV][kPad];
  __shared__ __attribute__((aligned(16))) __bf16 KT[DK][kPad];
  constexpr int MT = DV / 64, NT = DK / 64;
  const int nc1 = p.n_chunks - 1;
  const int c = blockIdx.x % nc1, bh = blockIdx.x / nc1;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const float lg = dt.log2_gamma[bh % p.H];
  const int64_t row0 = (int64_t)bh * p.L + (int64_t)c * p.chunk;
  const __bf16* Kc = p.K + row0 * DK;
  const __bf16* Vc = p.V + row0 * DV;
  const int m0 = (w >> 1) * (DV / 2), n0 = (w & 1) * (DK / 2);

  f32x16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;

  for (int jb = 0; jb < p.chunk; jb += 64) {
    if (jb) __syncthreads();
#pragma unroll
    for (int it = 0; it < DK / 32; ++it) {
      const int piece = tid + it * 256, row = piece / (DK / 8), c8 = piece % (DK / 8);
      const bf16x8 x = *reinterpret_cast<const bf16x8*>(Kc + (int64_t)(jb + row) * DK + c8 * 8);
      const float decay = exp2f(lg * (float)(p.chunk - 1 - (jb + row)));
#pragma unroll
      for (int t = 0; t < 8; ++t) KT[c8 * 8 + t][row] = (__bf16)((float)x[t] * decay);
    }
#pragma unroll
    for (int it = 0; it < DV / 32; ++it) {
      const int piece = tid + it * 256, row = piece / (DV / 8), c8 = piece % (DV / 8);
      const bf16x8 x = *reinterpret_cast<const bf16x8*>(Vc + (int64_t)(jb + row) * DV + c8 * 8);
#pragma unroll
      for (int t = 0; t < 8; ++t) VT[c8 * 8 + t][row] = x[t];
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int k0 = ks * 16 + 8 * (lane >> 5);
      bf16x8 a[MT], b[NT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) a[mt] = *reinterpret_cast<const bf16x8*>(&VT[m0 + mt * 32 + (lane & 31)][k0]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[nt] = *reinterpret_cast<const bf16x8*>(&KT[n0 + nt * 32 + (lane & 31)][k0]);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mt], b[nt], acc[mt][nt], 0, 0, 0);
    }
  }
  float* S = p.S + ((int64_t)bh * nc1 + c) * (DV * DK);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + mt * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        S[row * DK + n0 + nt * 32 + (lane & 31)] = acc[mt][nt][r];
      }
}

// HT[c] = state in front of chunk c+1 (bf16 of the fp32 running state):  h = gamma^C h + S[c],  c = 0 .. n_chunks-2.
// One thread per four state elements of a (batch, head); every thread walks the chunks in order.
__global__ __launch_bounds__(256) void rec_scan_kernel(const RecParams p, const DecayTable dt, int quads) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (gid >= (int64_t)p.B * p.H * quads) return;
  const int bh = (int)(gid / quads), e = (int)(gid % quads);
  const int nc1 = p.n_chunks - 1;
  const float g = exp2f(dt.log2_gamma[bh % p.H] * (float)p.chunk);
  const float4* S = reinterpret_cast<const float4*>(p.S) + (int64_t)bh * nc1 * quads + e;
  bf16x4* HT = reinterpret_cast<bf16x4*>(p.HT) + (int64_t)bh * nc1 * quads + e;
  float4 h = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int c = 0; c < nc1; ++c) {
    const float4 s = S[(int64_t)c * quads];
    h.x = g * h.x + s.x;
    h.y = g * h.y + s.y;
    h.z = g * h.z + s.z;
    h.w = g * h.w + s.w;
    bf16x4 o;
    o[0] = (__bf16)h.x;
    o[1] = (__bf16)h.y;
    o[2] = (__bf16)h.z;
    o[3] = (__bf16)h.w;
    HT[(int64_t)c * quads] = o;
  }
}

// O[i][dv] += scale gamma^(i+1) sum_dk Q[i][dk] HT[c-1][dv][dk]  for the rows of chunks 1 .. n_chunks-1.
// One workgroup (4 waves) per (batch*head, chunk, 64 rows); wave w owns rows 32 (w>>1) .. and the (w&1) half of dv.
template <int DK, int DV>
__global__ __launch_bounds__(256) void rec_readout_kernel(const RecParams p, const DecayTable dt) {
  constexpr int NT = DV / 64;
  const int blocks_per_chunk = p.chunk / 64, nc1 = p.n_chunks - 1;
  const int rb = blockIdx.x % blocks_per_chunk, c = 1 + (blockIdx.x / blocks_per_chunk) % nc1;
  const int bh = blockIdx.x / (blocks_per_chunk * nc1);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int i0 = rb * 64 + (w >> 1) * 32;            // first row of the wave, inside the chunk
  const int t0 = c * p.chunk + i0;                   // and inside the sequence
  if (t0 >= p.L) return;                             // (whole wave; no barrier in this kernel)
  const float lg = dt.log2_gamma[bh % p.H];
  const int n0 = (w & 1) * (DV / 2);
  const int arow = min(t0 + (lane & 31), p.L - 1);   // rows past the end read the last row and are not stored
  const __bf16* q = p.Q + ((int64_t)bh * p.L + arow) * DK + 8 * (lane >> 5);
  const __bf16* ht = p.HT + ((int64_t)bh * nc1 + (c - 1)) * (DV * DK) + (int64_t)(n0 + (lane & 31)) * DK + 8 * (lane >> 5);

  f32x16 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < DK / 16; ++ks) {
    const bf16x8 a = *reinterpret_cast<const bf16x8*>(q + ks * 16);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const bf16x8 b = *reinterpret_cast<const bf16x8*>(ht + (int64_t)nt * 32 * DK + ks * 16);
      acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[nt], 0, 0, 0);
    }
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int ri = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
    if (t0 + ri < p.L) {
      const float f = p.scale * exp2f(lg * (float)(i0 + ri + 1));
      float* o = p.O + ((int64_t)bh * p.L + t0 + ri) * DV + n0 + (lane & 31);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) o[nt * 32] += f * acc[nt][r];
    }
  }
}

template <int DK, int DV>
hipError_t launch_dims(const RecParams& p, const DecayTable& dt, hipStream_t stream) {
  const int nc1 = p.n_chunks - 1, bh = p.B * p.H, quads = DK * DV / 4;
  rec_state_kernel<DK, DV><<<dim3(bh * nc1), dim3(256), 0, stream>>>(p, dt);
  rec_scan_kernel<<<dim3((unsigned)(((int64_t)bh * quads + 255) / 256)), dim3(256), 0, stream>>>(p, dt, quads);
  rec_readout_kernel<DK, DV><<<dim3(bh * nc1 * (p.chunk / 64)), dim3(256), 0, stream>>>(p, dt);
  return hipGetLastError();
}

}  // namespace

bool recurrent_supported(int dqk, int dv) { return (dqk == 64 && dv == 64) || (dqk == 128 && dv == 128); }

hipError_t launch_recurrent_inter(const RecParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream) {
  if (p.n_chunks < 2 || p.chunk % 64 != 0) return hipErrorInvalidValue;
  if (dqk == 64 && dv == 64) return launch_dims<64, 64>(p, dt, stream);
  if (dqk == 128 && dv == 128) return launch_dims<128, 128>(p, dt, stream);
  return hipErrorInvalidValue;
}

}  // namespace ae
