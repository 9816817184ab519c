// Recurrent pattern (Section 4.1: K@V first, then Q@h over a compressed state), chunk-parallel so that the
// matrix units do the work (Section 4.2, kernel templates for recurrent patterns): retention with a constant
// decay per head,  h_t = gamma h_{t-1} + k_t^T v_t,  o_t = scale q_t h_t.
//
// With the sequence cut into chunks of C tokens and H_c the state after chunk c:
//   o_i  = scale gamma^(i+1) q_i H_{c-1}          (i: position inside the chunk)      read-out of the carried state
//        + causal decay-masked attention inside the chunk                              parallel pattern
//   H_c  = gamma^C H_{c-1} + sum_j gamma^(C-1-j) k_j^T v_j                            this file
// The read-out is the prologue of the parallel-pattern kernel (attn_kernel.hpp, Params::state), which then walks
// the chunk's own keys on top of it: O is written once.  The kernel here produces the states: one workgroup per
// (batch, head, 32 columns of D_v) walks the sequence chunk by chunk with its slice of the state in MFMA
// accumulators (fp32) and stores it, rounded to bf16 and transposed ([D_v][D_qk]: the layout the read-out takes
// 16 bytes at a time), after every chunk but the last.
// Every decay factor is a power of gamma with a non-negative exponent: nothing can overflow.
#include "recurrent.hpp"

#include <type_traits>

namespace ae {
namespace {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// MFMA operand with the contraction index along the ROWS of a row-major LDS tile: the transposing read hands
// each lane of a 16-lane block column (lane % 16) of the 4 rows whose addresses the block's lanes supply
// (lane i: row i / 4, columns 4 (i % 4) .. +3).  lo / hi: this lane's address for tokens 0..3 / 4..7 of its eight.
__device__ __forceinline__ bf16x8 read_tr(uint32_t lo, uint32_t hi) {
  const s16x4 x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)lo);
  const s16x4 y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)hi);
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(x, y, 0, 1, 2, 3, 4, 5, 6, 7));
}

// H^T[dv][dk] += sum_j gamma^(C-1-j) V[j][dv] K[j][dk]: the contraction runs over the tokens, the slow index of
// both operands.  The 64-token blocks are stored to LDS as they come (16 bytes per lane, the decay applied to V
// on the way) and read with the transposing LDS read.  Row strides of 16 or 48 (mod 64) words keep the four
// rows x two column groups that half a wave reads at once on different banks.
// A workgroup owns NSL slices of 32 D_v columns, NSL * DK/32 waves; a wave owns one 32 x 32 tile (slice, dk block).
// NSL = D_v / 32: one workgroup per (batch, head), K staged once for all slices (many (batch, head) pairs);
// NSL = 1: a workgroup per slice, four times the workgroups (few pairs: the walk is sequential per workgroup).
template <int DK, int DV, int NSL>
__global__ __launch_bounds__(2 * DK * NSL) void rec_state_kernel(const RecParams p, const DecayTable dt) {
  constexpr int THREADS = 2 * DK * NSL, NS = DV / (32 * NSL);  // NS workgroups per (batch, head)
  constexpr int KP = (64 * (DK / 8) + THREADS - 1) / THREADS;  // 16-byte pieces of a K block per thread
  constexpr int VPIECES = 64 * 4 * NSL, VP = (VPIECES + THREADS - 1) / THREADS;  // and of the V slices
  constexpr int KS = DK * 2 + 64;                               // bytes per K row in LDS: 80 / 48 words
  constexpr int VS = NSL == 1 ? 64 : 64 * NSL + 64;             // 16 words, or 80 / 48
  static_assert((KS / 4) % 64 == 16 || (KS / 4) % 64 == 48, "K row stride");
  static_assert((VS / 4) % 64 == 16 || (VS / 4) % 64 == 48, "V row stride");
  static_assert(64 * (DK / 8) % THREADS == 0 && VPIECES % THREADS == 0, "every thread copies the same number of pieces");
  __shared__ __attribute__((aligned(16))) char Ks[64 * KS];
  __shared__ __attribute__((aligned(16))) char Vs[64 * VS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int w = wave % (DK / 32), sl = wave / (DK / 32);  // dk block and slice of this wave
  // The workgroups of one (batch, head) read the same K: they go to one XCD (workgroups are dealt to the 8 XCDs
  // round-robin by id), next to each other in time, so that its L2 serves the repeats.
  const int bhs = p.B * p.H;
  int bh, slice;  // slice: the first one of the workgroup, then this wave's
  if (bhs % 8 == 0) {
    const int x = blockIdx.x % 8, k = blockIdx.x / 8;
    bh = (k / NS) * 8 + x;
    slice = k % NS;
  } else {
    bh = blockIdx.x / NS;
    slice = blockIdx.x % NS;
  }
  const int slice0 = slice * NSL;
  slice = slice0 + sl;
  const float lg = dt.log2_gamma[bh % p.H];
  const float g_chunk = exp2f(lg * (float)p.chunk);
  const __bf16* Kb = p.K + (int64_t)bh * p.L * DK;
  const __bf16* Vb = p.V + (int64_t)bh * p.L * DV + slice0 * 32;
  __bf16* HTb = p.HT + (int64_t)bh * p.n_chunks * (DV * DK) + (int64_t)slice * 32 * DK;  // slot c: the state in front of chunk c

  // fragment addresses of contraction step 0: tokens 8 (lane / 32) + (lane % 16) / 4, column 16 ((lane / 16) % 2) + 4 (lane % 4)
  const int i16 = lane & 15, q = lane >> 4;
  const int frow = 8 * (q >> 1) + (i16 >> 2), fcol = 16 * (q & 1) + 4 * (i16 & 3);
  const uint32_t ks0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)Ks);
  const uint32_t vs0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)Vs);
  const uint32_t ka = ks0 + frow * KS + (w * 32 + fcol) * 2;
  const uint32_t va = vs0 + frow * VS + (sl * 32 + fcol) * 2;

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  if (p.h_in != nullptr) {  // start from the caller's state ([D_qk][D_v] fp32); chunk 0 reads it from slot 0
    const float* hin = p.h_in + (int64_t)bh * (DK * DV) + (int64_t)(w * 32 + (lane & 31)) * DV + slice * 32;
    __bf16* ht = HTb + w * 32 + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      acc[r] = hin[row];
      ht[row * DK] = (__bf16)acc[r];
      acc[r] *= exp2f(lg * (float)min(p.chunk, p.L));  // aged by the first chunk's length before its tokens are added
    }
  }

  // Without a final state to hand back the last chunk is not walked; every chunk but the last is a full one.
  const int n_blocks = p.h_out != nullptr ? (p.L + 63) / 64 : (p.n_chunks - 1) * (p.chunk / 64);
  // Block loads run two blocks ahead of the MFMAs, in two register sets used in turn: a workgroup's own MFMAs
  // are far too short to cover a memory latency, and only four workgroups share a CU.
  bf16x8 kreg[2][KP], vreg[2][VP];
  auto fetch = [&](auto setc, int blk) {
    constexpr int S = decltype(setc)::value;
    if (blk >= n_blocks) return;
    const int t0 = blk * 64;  // tokens past the end (last block of a short last chunk) read the last one, with weight 0
#pragma unroll
    for (int it = 0; it < KP; ++it) {
      const int piece = tid + it * THREADS, row = piece / (DK / 8), c8 = piece % (DK / 8);
      kreg[S][it] = *reinterpret_cast<const bf16x8*>(Kb + (int64_t)min(t0 + row, p.L - 1) * DK + c8 * 8);
    }
#pragma unroll
    for (int it = 0; it < VP; ++it) {
      const int piece = tid + it * THREADS, row = piece / (4 * NSL), c8 = piece % (4 * NSL);
      vreg[S][it] = *reinterpret_cast<const bf16x8*>(Vb + (int64_t)min(t0 + row, p.L - 1) * DV + c8 * 8);
    }
  };
  auto process = [&](auto setc, int blk) {
    constexpr int S = decltype(setc)::value;
    if (blk >= n_blocks) return;          // (uniform over the workgroup)
    const int j0 = (blk * 64) % p.chunk;  // position of the block inside its chunk
    const int c = (blk * 64) / p.chunk;
    const int len = min(p.chunk, p.L - c * p.chunk);  // tokens of this chunk (the last one may be short)
    __syncthreads();                      // the fragments of the previous block have been read
#pragma unroll
    for (int it = 0; it < KP; ++it) {
      const int piece = tid + it * THREADS, row = piece / (DK / 8), c8 = piece % (DK / 8);
      *reinterpret_cast<bf16x8*>(Ks + row * KS + c8 * 16) = kreg[S][it];
    }
    // the token's decay goes onto its V row: the slice has a quarter of the K block's elements (at 128/128)
#pragma unroll
    for (int it = 0; it < VP; ++it) {
      const int piece = tid + it * THREADS, row = piece / (4 * NSL), c8 = piece % (4 * NSL);
      {
        const float decay = j0 + row < len ? exp2f(lg * (float)(len - 1 - (j0 + row))) : 0.f;
        bf16x8 x;
#pragma unroll
        for (int t = 0; t < 8; ++t) x[t] = (__bf16)((float)vreg[S][it][t] * decay);
        *reinterpret_cast<bf16x8*>(Vs + row * VS + c8 * 16) = x;
      }
    }
    __syncthreads();
    fetch(setc, blk + 2);  // this set is free again
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8 a = read_tr(va + ks * 16 * VS, va + (ks * 16 + 4) * VS);
      const bf16x8 b = read_tr(ka + ks * 16 * KS, ka + (ks * 16 + 4) * KS);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
    if (j0 + 64 >= len) {  // end of a chunk
      if (c + 1 < p.n_chunks) {  // store the state for the next chunk, then age it by that chunk's length
        const float g_next = c + 2 < p.n_chunks ? g_chunk : exp2f(lg * (float)(p.L - (c + 1) * p.chunk));
        __bf16* ht = HTb + (int64_t)(c + 1) * (DV * DK) + w * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          ht[row * DK] = (__bf16)acc[r];
          acc[r] *= g_next;
        }
      } else {  // the state after the last token, [D_qk][D_v] fp32 (only walked when asked for)
        float* hout = p.h_out + (int64_t)bh * (DK * DV) + (int64_t)(w * 32 + (lane & 31)) * DV + slice * 32;
#pragma unroll
        for (int r = 0; r < 16; ++r) hout[8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)] = acc[r];
      }
    }
  };
  using Set0 = std::integral_constant<int, 0>;
  using Set1 = std::integral_constant<int, 1>;
  fetch(Set0{}, 0);
  fetch(Set1{}, 1);
  for (int blk = 0; blk < n_blocks; blk += 2) {
    process(Set0{}, blk);
    process(Set1{}, blk + 1);
  }
}

// One step of the recurrence as the paper's recurrent pattern states it (K@V into the state, then Q@h): a pass over
// the state, which is all the traffic there is (8 bytes per state element).  One workgroup per (batch, head);
// a thread owns four columns of D_v in every (256 / (D_v / 4))-th row; the partial read-outs meet in LDS.
template <int DK, int DV>
__global__ __launch_bounds__(256) void rec_step_kernel(const RecStepParams p, const DecayTable dt) {
  constexpr int CG = DV / 4, RG = 256 / CG;  // column groups, row groups
  __shared__ float4 part[RG][CG];
  const int bh = blockIdx.x, tid = threadIdx.x, cg = tid % CG, rg = tid / CG;
  const float g = exp2f(dt.log2_gamma[bh % p.H]);
  const __bf16* q = p.q + (int64_t)bh * DK;
  const __bf16* k = p.k + (int64_t)bh * DK;
  const bf16x4 vb = *reinterpret_cast<const bf16x4*>(p.v + (int64_t)bh * DV + 4 * cg);
  const float v0 = (float)vb[0], v1 = (float)vb[1], v2 = (float)vb[2], v3 = (float)vb[3];
  float4* st = reinterpret_cast<float4*>(p.state + (int64_t)bh * (DK * DV)) + cg;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
  for (int r = rg; r < DK; r += RG) {
    float4 h = st[(int64_t)r * CG];
    const float kr = (float)k[r], qr = (float)q[r];
    h.x = g * h.x + kr * v0;
    h.y = g * h.y + kr * v1;
    h.z = g * h.z + kr * v2;
    h.w = g * h.w + kr * v3;
    st[(int64_t)r * CG] = h;
    acc.x += qr * h.x;
    acc.y += qr * h.y;
    acc.z += qr * h.z;
    acc.w += qr * h.w;
  }
  part[rg][cg] = acc;
  __syncthreads();
  if (tid < CG) {
    float4 s = part[0][tid];
#pragma unroll
    for (int i = 1; i < RG; ++i) {
      const float4 x = part[i][tid];
      s.x += x.x;
      s.y += x.y;
      s.z += x.z;
      s.w += x.w;
    }
    s.x *= p.scale;
    s.y *= p.scale;
    s.z *= p.scale;
    s.w *= p.scale;
    reinterpret_cast<float4*>(p.o + (int64_t)bh * DV)[tid] = s;
  }
}

template <int DK, int DV>
hipError_t launch_dims(const RecParams& p, const DecayTable& dt, hipStream_t stream) {
  // enough (batch, head) pairs to give every CU a workgroup: all slices in one workgroup, K staged once
  if (p.B * p.H >= 256) rec_state_kernel<DK, DV, DV / 32><<<dim3(p.B * p.H), dim3(2 * DK * (DV / 32)), 0, stream>>>(p, dt);
  else rec_state_kernel<DK, DV, 1><<<dim3(p.B * p.H * (DV / 32)), dim3(2 * DK), 0, stream>>>(p, dt);
  return hipGetLastError();
}

}  // namespace

bool recurrent_supported(int dqk, int dv) { return (dqk == 64 && dv == 64) || (dqk == 128 && dv == 128); }

hipError_t launch_recurrent_step(const RecStepParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream) {
  if (dqk == 64 && dv == 64) rec_step_kernel<64, 64><<<dim3(p.B * p.H), dim3(256), 0, stream>>>(p, dt);
  else if (dqk == 128 && dv == 128) rec_step_kernel<128, 128><<<dim3(p.B * p.H), dim3(256), 0, stream>>>(p, dt);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_recurrent_states(const RecParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t stream) {
  if (p.chunk % 64 != 0 || (p.n_chunks < 2 && !p.h_in && !p.h_out)) return hipErrorInvalidValue;
  if (dqk == 64 && dv == 64) return launch_dims<64, 64>(p, dt, stream);
  if (dqk == 128 && dv == 128) return launch_dims<128, 128>(p, dt, stream);
  return hipErrorInvalidValue;
}

}  // namespace ae
