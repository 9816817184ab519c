// Fused parallel-pattern attention forward kernel for gfx950 (CDNA4).
//
// One workgroup owns BLOCK_M = 32*QB*WAVES query rows of one (batch, q-head)
// and walks the visible key/value tiles of BLOCK_N = 64 keys.  Per tile:
//   relevance scoring   S^T = K_tile Q^T          (bf16 MFMA 32x32x16, fp32 acc)
//   modification        scale / bias / decay / relu / mask, in registers
//   online row-norm     per-row running state (max+sum, or abs-sum), registers
//   aggregation         O^T += V_tile^T P^T       (bf16 MFMA, fp32 acc)
// (paper Section 4.1: parallel pattern with the online row-norm interface).
//
// Why the transposed products: in the 32x32 accumulator layout a lane owns ONE
// column and 16 rows.  With S^T (rows = keys, columns = queries) every value a
// lane holds belongs to a single query, so the row reductions of the
// normalization are in-lane plus one exchange between lane l and lane l^32, the
// per-row rescale of O is a per-lane scalar, and the accumulator registers of
// S^T are, with no data movement, the B operand of the second MFMA: the order
// in which keys are contracted is free, so V is read from LDS in the key order
// that the accumulator layout dictates (ds_read_b64_tr_b16 does the transpose).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ae {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

enum : int { NORM_SOFTMAX = 0, NORM_SIGMOID = 1, NORM_ABSSUM = 2, NORM_ABS_OF_SUM = 3, NORM_NONE = 4 };
enum : int { MOD_PLAIN = 0, MOD_DECAY = 1, MOD_RELU = 2 };  // PLAIN carries a runtime bias (0 for "none")

constexpr int kMaxDecayHeads = 256;

struct Params {
  const __bf16* Q;
  const __bf16* K;
  const __bf16* V;
  float* O;
  int B, H_q, H_kv, L_q, L_k;
  int g;        // H_q / H_kv
  int n_qtiles; // ceil(L_q / BLOCK_M)
  int n_groups; // B * H_kv
  int64_t qs[3], ks[3], vs[3], os[3];  // element strides {batch, head, row}
  float c;      // |scale| * log2(e)  (softmax, sigmoid)  or |scale| (others)
  float b2;     // bias * log2(e)     (softmax, sigmoid)  or bias (others)
  int neg_q;    // scale < 0: the sign is moved onto Q (exact for bf16)
};

struct DecayTable {
  float log2_gamma[kMaxDecayHeads];
};

template <int DQK_, int DV_, int NORM_, int MOD_, bool CAUSAL_, int WAVES_, int QB_>
struct Cfg {
  static constexpr int DQK = DQK_, DV = DV_, NORM = NORM_, MOD = MOD_, WAVES = WAVES_, QB = QB_;
  static constexpr bool CAUSAL = CAUSAL_;
  static constexpr int BLOCK_N = 64;
  static constexpr int BLOCK_M = 32 * QB * WAVES;
  static constexpr int THREADS = 64 * WAVES;
  // LDS row strides in bytes.  K is read with 128-bit loads by 16 lanes at a
  // time, one row each: +16 B per row spreads them over all banks.  V is read
  // with 64-bit transposing loads, 32 lanes covering 4 rows x 64 B: +64 B per
  // row does the same.
  static constexpr int KSTRIDE = DQK * 2 + 16;
  static constexpr int VSTRIDE = DV * 2 + 64;
  static constexpr int K_BYTES = BLOCK_N * KSTRIDE;
  static constexpr int V_BYTES = BLOCK_N * VSTRIDE;
  static constexpr int LDS_BYTES = 2 * (K_BYTES + V_BYTES);
  static constexpr int K_CHUNKS = BLOCK_N * DQK / 8;  // 16-byte chunks per tile
  static constexpr int V_CHUNKS = BLOCK_N * DV / 8;
  static constexpr int K_PER_THREAD = (K_CHUNKS + THREADS - 1) / THREADS;
  static constexpr int V_PER_THREAD = (V_CHUNKS + THREADS - 1) / THREADS;
  static_assert(DQK % 16 == 0 && DV % 32 == 0, "head dims must fit the MFMA tile");
  static_assert(LDS_BYTES <= 160 * 1024, "tile does not fit LDS");
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// The other 16 keys of a query row live in lane l^32.  v_permlane32_swap
// exchanges the upper half of its first operand with the lower half of its
// second: fed the same value twice it returns (x[l%32], x[l%32 + 32]) in every
// lane.  (The results are copied to scalars before the bit cast: a bit cast
// applied directly to a vector element reads element 0 with this compiler.)
__device__ __forceinline__ void swap_halves(float x, float& lo, float& hi) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  lo = __builtin_bit_cast(float, r0);
  hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float max_halves(float x) {
  float lo, hi;
  swap_halves(x, lo, hi);
  return fmaxf(lo, hi);
}
__device__ __forceinline__ float sum_halves(float x) {
  float lo, hi;
  swap_halves(x, lo, hi);
  return lo + hi;
}
constexpr float kLazyLog2 = 8.0f;

template <class C>
__device__ __forceinline__ void stage_load(const Params& p, const __bf16* kbase, const __bf16* vbase,
                                           int j0, u32x4 (&kreg)[C::K_PER_THREAD], u32x4 (&vreg)[C::V_PER_THREAD]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < C::K_PER_THREAD; ++i) {
    const int c = tid + i * C::THREADS;
    const int row = c / (C::DQK / 8), col = c % (C::DQK / 8);
    u32x4 v = {0u, 0u, 0u, 0u};
    if ((C::K_CHUNKS % C::THREADS == 0 || c < C::K_CHUNKS) && j0 + row < p.L_k)
      v = *reinterpret_cast<const u32x4*>(kbase + (int64_t)(j0 + row) * p.ks[2] + col * 8);
    kreg[i] = v;
  }
#pragma unroll
  for (int i = 0; i < C::V_PER_THREAD; ++i) {
    const int c = tid + i * C::THREADS;
    const int row = c / (C::DV / 8), col = c % (C::DV / 8);
    u32x4 v = {0u, 0u, 0u, 0u};
    if ((C::V_CHUNKS % C::THREADS == 0 || c < C::V_CHUNKS) && j0 + row < p.L_k)
      v = *reinterpret_cast<const u32x4*>(vbase + (int64_t)(j0 + row) * p.vs[2] + col * 8);
    vreg[i] = v;
  }
}

template <class C>
__device__ __forceinline__ void stage_store(char* ksm, char* vsm, const u32x4 (&kreg)[C::K_PER_THREAD],
                                            const u32x4 (&vreg)[C::V_PER_THREAD]) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < C::K_PER_THREAD; ++i) {
    const int c = tid + i * C::THREADS;
    const int row = c / (C::DQK / 8), col = c % (C::DQK / 8);
    if (C::K_CHUNKS % C::THREADS == 0 || c < C::K_CHUNKS)
      *reinterpret_cast<u32x4*>(ksm + row * C::KSTRIDE + col * 16) = kreg[i];
  }
#pragma unroll
  for (int i = 0; i < C::V_PER_THREAD; ++i) {
    const int c = tid + i * C::THREADS;
    const int row = c / (C::DV / 8), col = c % (C::DV / 8);
    if (C::V_CHUNKS % C::THREADS == 0 || c < C::V_CHUNKS)
      *reinterpret_cast<u32x4*>(vsm + row * C::VSTRIDE + col * 16) = vreg[i];
  }
}

// Per-wave running state of the online row normalization.
template <class C>
struct RowState {
  float m[C::QB];  // softmax: running row max (log2 domain); others unused
  float l[C::QB];  // softmax: running sum of exp; abs-sum family: running sum
  f32x16 o[C::QB][C::DV / 32];
};

// One key/value tile: scores, modification, online normalization, aggregation.
// MASKED selects the variant that tests visibility per element (tiles that
// cross the causal diagonal or the end of the key sequence).
template <class C, bool MASKED>
__device__ __forceinline__ void tile_compute(const Params& p, const char* ksm, const char* vsm,
                                             const bf16x8 (&qf)[C::QB][C::DQK / 16], RowState<C>& st,
                                             int j0, int iw0, int off, float g2) {
  const int lane = threadIdx.x & 63;
  const int ql = lane & 31, half = lane >> 5;

  // ---- relevance scoring: S^T[key, query] ---------------------------------
  f32x16 s[C::QB][2];
#pragma unroll
  for (int qb = 0; qb < C::QB; ++qb)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) s[qb][kb][r] = 0.f;

#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    const char* krow = ksm + (kb * 32 + ql) * C::KSTRIDE + half * 16;
#pragma unroll
    for (int t = 0; t < C::DQK / 16; ++t) {
      const bf16x8 kf = *reinterpret_cast<const bf16x8*>(krow + t * 32);
#pragma unroll
      for (int qb = 0; qb < C::QB; ++qb)
        s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][t], s[qb][kb], 0, 0, 0);
    }
  }

  // ---- modification + online row-norm, producing P^T as bf16 B operands ----
  // Register r of key block kb is key j0 + 32*kb + 8*(r/4) + 4*half + (r%4).
  bf16x8 pf[C::QB][4];
#pragma unroll
  for (int qb = 0; qb < C::QB; ++qb) {
    const int i = iw0 + qb * 32 + ql;  // this lane's query row
    const int jlim = MASKED ? min(C::CAUSAL ? i + off : p.L_k - 1, p.L_k - 1) - j0 - 4 * half : 0;
    // visible  <=>  32*kb + 8*(r/4) + (r%4) <= jlim
    float x[2][16];

    if constexpr (C::NORM == NORM_SOFTMAX) {
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = s[qb][kb][r];
          if (MASKED && (32 * kb + 8 * (r / 4) + (r % 4) > jlim)) v = -INFINITY;
          x[kb][r] = v;
          mx = fmaxf(mx, v);
        }
      mx = max_halves(mx);
      // Lazy reference maximum: the running reference m only moves when the
      // tile's row max exceeds it by more than kLazyLog2 (weights then stay
      // below 2^kLazyLog2, harmless in bf16/fp32), so the rescale of l and O
      // is skipped for almost every tile after the first.
      const float xm = __builtin_fmaf(mx, p.c, p.b2);  // c > 0
      const bool moved = xm > st.m[qb] + kLazyLog2;
      if (__builtin_amdgcn_ballot_w64(moved) != 0) {
        const float m_new = moved ? xm : st.m[qb];
        const float alpha = moved ? fast_exp2(st.m[qb] - m_new) : 1.f;
        st.m[qb] = m_new;
        st.l[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < C::DV / 32; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) st.o[qb][db][r] *= alpha;
      }
      const float k0 = p.b2 - ((st.m[qb] == -INFINITY) ? 0.f : st.m[qb]);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) x[kb][r] = fast_exp2(__builtin_fmaf(x[kb][r], p.c, k0));
    } else {
      // decay exponent base for this lane: log2(gamma) * (i + off - j) with
      // j = j0 + 4*half + const(kb, r); log2|scale| is folded in as well.
      float dbase = 0.f;
      if constexpr (C::MOD == MOD_DECAY) dbase = g2 * (float)(i + off - j0 - 4 * half);
      float sum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float raw = s[qb][kb][r];
          float v;
          if constexpr (C::NORM == NORM_SIGMOID) {
            // 1 / (1 + 2^(-(s*c + b2)))
            v = fast_rcp(1.f + fast_exp2(__builtin_fmaf(raw, -p.c, -p.b2)));
          } else {
            if constexpr (C::MOD == MOD_DECAY) {
              const float w = fast_exp2(__builtin_fmaf(-g2, (float)(32 * kb + 8 * (r / 4) + (r % 4)), dbase));
              v = raw * p.c * w;
            } else {
              v = __builtin_fmaf(raw, p.c, p.b2);
              if constexpr (C::MOD == MOD_RELU) v = fmaxf(v, 0.f);
            }
          }
          if (MASKED && (32 * kb + 8 * (r / 4) + (r % 4) > jlim)) v = 0.f;
          x[kb][r] = v;
          if constexpr (C::NORM == NORM_ABSSUM) sum += fabsf(v);
          if constexpr (C::NORM == NORM_ABS_OF_SUM) sum += v;
        }
      if constexpr (C::NORM == NORM_ABSSUM || C::NORM == NORM_ABS_OF_SUM) st.l[qb] += sum;
    }

    // P -> bf16 pairs (hardware RNE pack); for softmax the row sum is taken
    // over the rounded weights, two per v_dot2c_f32_bf16.
    float psum = 0.f;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      u32x4 pk;
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        bf16x2 pr;
        pr[0] = (__bf16)x[t >> 1][8 * (t & 1) + 2 * e2];
        pr[1] = (__bf16)x[t >> 1][8 * (t & 1) + 2 * e2 + 1];
        if constexpr (C::NORM == NORM_SOFTMAX) {
          const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
          psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
        }
        pk[e2] = __builtin_bit_cast(uint32_t, pr);
      }
      pf[qb][t] = __builtin_bit_cast(bf16x8, pk);
    }
    if constexpr (C::NORM == NORM_SOFTMAX) st.l[qb] += psum;
  }

  // ---- aggregation: O^T[d, query] += V^T P^T --------------------------------
  // Transposing LDS read: within each 16-lane block, lane i supplies the
  // address of row (i/4), columns 4*(i%4)..+3 and receives column i of the 4
  // rows.  Blocks 0/1 of the wave cover d 0..15 / 16..31 for key half 0,
  // blocks 2/3 the same for key half 1.
  const int li = lane & 15;
  const char* vlane = vsm + ((li >> 2) + 4 * half) * C::VSTRIDE + (16 * ((lane >> 4) & 1) + 4 * (li & 3)) * 2;
#pragma unroll
  for (int db = 0; db < C::DV / 32; ++db) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const char* a0 = vlane + (16 * t) * C::VSTRIDE + db * 64;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(a0));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(a0 + 8 * C::VSTRIDE));
      const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
      for (int qb = 0; qb < C::QB; ++qb)
        st.o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb][t], st.o[qb][db], 0, 0, 0);
    }
  }
}

template <class C>
__global__ __launch_bounds__(C::THREADS) void attn_fwd_kernel(const Params p, const DecayTable dt) {
  __shared__ __attribute__((aligned(16))) char smem[C::LDS_BYTES];

  // ---- workgroup -> (batch, kv head, q head, q tile) ------------------------
  // Workgroups are handed to the 8 XCDs round-robin by id.  All q tiles and
  // all q heads of one (batch, kv head) group are mapped to ONE XCD so that
  // the group's K/V stays in that XCD's L2; within a group the causal tiles
  // with the most key tiles are issued first.
  const int w = blockIdx.x;
  const int per_group = p.n_qtiles * p.g;
  const int slot = w >> 3;
  const int group = (slot / per_group) * 8 + (w & 7);
  if (group >= p.n_groups) return;
  const int t = slot % per_group;
  const int b = group / p.H_kv, hkv = group % p.H_kv;
  const int hq = hkv * p.g + (t % p.g);
  const int qt_lin = t / p.g;
  const int qtile = C::CAUSAL ? (p.n_qtiles - 1 - qt_lin) : qt_lin;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ql = lane & 31, half = lane >> 5;
  const int off = p.L_k - p.L_q;
  const int i_wg = qtile * C::BLOCK_M;
  const int iw0 = i_wg + wave * 32 * C::QB;

  const __bf16* qbase = p.Q + b * p.qs[0] + hq * p.qs[1];
  const __bf16* kbase = p.K + b * p.ks[0] + hkv * p.ks[1];
  const __bf16* vbase = p.V + b * p.vs[0] + hkv * p.vs[1];
  float* obase = p.O + b * p.os[0] + hq * p.os[1];

  // ---- Q fragments (B operand of S^T = K Q^T), resident for the whole kernel -
  bf16x8 qf[C::QB][C::DQK / 16];
#pragma unroll
  for (int qb = 0; qb < C::QB; ++qb) {
    const int i = iw0 + qb * 32 + ql;
#pragma unroll
    for (int tt = 0; tt < C::DQK / 16; ++tt) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (i < p.L_q) v = *reinterpret_cast<const u32x4*>(qbase + (int64_t)i * p.qs[2] + tt * 16 + half * 8);
      if (p.neg_q) v ^= (u32x4){0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
      qf[qb][tt] = __builtin_bit_cast(bf16x8, v);
    }
  }

  RowState<C> st;
#pragma unroll
  for (int qb = 0; qb < C::QB; ++qb) {
    st.m[qb] = -INFINITY;
    st.l[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < C::DV / 32; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st.o[qb][db][r] = 0.f;
  }

  float g2 = 0.f;
  if constexpr (C::MOD == MOD_DECAY) g2 = dt.log2_gamma[hq];

  // number of key tiles this workgroup visits
  int kmax = p.L_k;
  if (C::CAUSAL) kmax = max(0, min(p.L_k, i_wg + C::BLOCK_M + off));
  const int n_tiles = (kmax + C::BLOCK_N - 1) / C::BLOCK_N;

  // LDS: [K buf 0][K buf 1][V buf 0][V buf 1]
  char* const ksm0 = smem;
  char* const vsm0 = smem + 2 * C::K_BYTES;

  u32x4 kreg[C::K_PER_THREAD], vreg[C::V_PER_THREAD];
  if (n_tiles > 0) {
    stage_load<C>(p, kbase, vbase, 0, kreg, vreg);
    stage_store<C>(ksm0, vsm0, kreg, vreg);
  }
  __syncthreads();

  for (int jt = 0; jt < n_tiles; ++jt) {
    const int j0 = jt * C::BLOCK_N;
    const int cur = jt & 1;
    const bool more = jt + 1 < n_tiles;
    if (more) stage_load<C>(p, kbase, vbase, j0 + C::BLOCK_N, kreg, vreg);

    // wave-uniform: does this wave see any key of the tile / need the mask?
    const int iw_last = iw0 + 32 * C::QB - 1;
    const bool any_visible = !C::CAUSAL || (j0 <= iw_last + off);
    if (any_visible) {
      const bool need_mask = (j0 + C::BLOCK_N > p.L_k) || (C::CAUSAL && (j0 + C::BLOCK_N - 1 > iw0 + off));
      if (need_mask)
        tile_compute<C, true>(p, ksm0 + cur * C::K_BYTES, vsm0 + cur * C::V_BYTES, qf, st, j0, iw0, off, g2);
      else
        tile_compute<C, false>(p, ksm0 + cur * C::K_BYTES, vsm0 + cur * C::V_BYTES, qf, st, j0, iw0, off, g2);
    }

    if (more) stage_store<C>(ksm0 + (cur ^ 1) * C::K_BYTES, vsm0 + (cur ^ 1) * C::V_BYTES, kreg, vreg);
    __syncthreads();
  }

  // ---- online_epilogue + store ------------------------------------------------
#pragma unroll
  for (int qb = 0; qb < C::QB; ++qb) {
    float inv = 1.f;
    if constexpr (C::NORM == NORM_SOFTMAX) {
      const float l = sum_halves(st.l[qb]);
      inv = l > 0.f ? 1.f / l : 0.f;
    } else if constexpr (C::NORM == NORM_ABSSUM) {
      const float l = sum_halves(st.l[qb]);
      inv = 1.f / fmaxf(l, 1.f);
    } else if constexpr (C::NORM == NORM_ABS_OF_SUM) {
      const float l = sum_halves(st.l[qb]);
      inv = 1.f / fmaxf(fabsf(l), 1.f);
    }
    const int i = iw0 + qb * 32 + ql;
    if (i < p.L_q) {
      float* orow = obase + (int64_t)i * p.os[2];
#pragma unroll
      for (int db = 0; db < C::DV / 32; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = st.o[qb][db][4 * r4 + e] * inv;
          *reinterpret_cast<f32x4*>(orow + db * 32 + r4 * 8 + half * 4) = v;
        }
    }
  }
}

}  // namespace ae
