// Backward pass of fused parallel-pattern attention for gfx950 (CDNA4): the gradients
// of O = normalization(modification(Q K^T)) V with respect to Q, K and V, for a given
// upstream gradient dO, with the weights recomputed from the row statistic that the
// forward pass keeps (paper Section 4.1, online row-norm interface: the backward graph
// is derived from the same definition and reads the final row scales).
//
//   P   = exp(S' - lse_i)  (softmax)   |  sigmoid(S')            S' = scale * Q K^T + bias
//   dV  = P^T dO                          dP = dO V^T
//   dS' = P * (dP - delta_i), delta_i = dO_i . O_i  (softmax)   |  dP * P * (1 - P)  (sigmoid)
//   no normalization: P = S' or max(S', 0) on visible entries, dS' = dP or dP * [S' > 0]
//   abs-sum family (retention): S' = scale * Q K^T * decay, P = S' / n_i, n_i = max(r_i, 1), r_i = sum_j |S'| or
//     |sum_j S'| (the forward row statistic); dS' = (dP - g * [r_i > 1] * delta_i) / n_i with g = sign(S') or
//     sign(sum_j S'); the gradient of the raw score is dS' * decay
//   dQ  = scale * dS' K                   dK = scale * dS'^T Q
//
// Two kernels of one shape, no atomics, every output written once:
//   * key side (KV_SIDE): a workgroup owns 128 keys of one k/v head and walks the query tiles of
//     the q heads that share it: dK and dV;
//   * query side: a workgroup owns 128 query rows of one q head and walks the key tiles: dQ.
// The key-side kernel holds two accumulators and two resident operands; from D 128/128 on that
// is more than the 256 registers of a two-waves-per-SIMD kernel, and it then runs one workgroup
// per CU with up to 512 (a variant squeezed into 256 spilled in its inner loop and was 1.5 x
// slower; separate dK and dV kernels at two waves per SIMD recompute the scores once more and
// were 15-25 % slower than the fused one).  Both kernels run against the board's power limit:
// the clock under load is 1.4-1.7 GHz.
// In both a wavefront owns 32 rows ("own" side) whose two operand matrices it keeps in
// registers as MFMA B fragments (K, V | Q, dO), and the tiles of the other side (Q, dO |
// K, V; 64 rows, double buffered) arrive in LDS by global_load_lds.  Per 32-row sub-tile
//   S  [other x own] = Y1 X1^T      dP [other x own] = Y2 X2^T        (bf16 MFMA 32x32x16)
// put a lane's 16 accumulator values in one own column; after the elementwise step they
// are, packed to bf16 and with no data movement, the B operands of
//   dQ^T, dK^T [D_qk x own] += Y1^T dS       dV^T [D_v x own] += Y2^T P
// whose A operands are the same LDS tiles read through the transposing LDS load, in the
// row order that the accumulator layout dictates.
#pragma once
#include "attn_kernel.hpp"

namespace ae {

struct BwdParams {
  const __bf16* Q;
  const __bf16* K;
  const __bf16* V;
  const __bf16* dO;    // [B, H_q, L_q, D_v] contiguous
  const void* O;       // as the forward pass wrote it (softmax only): fp32, or bf16 if o_bf16
  const float* lse;    // [B, H_q, L_q] row statistic of the forward pass (softmax; abs-sum family: r or the signed sum)
  float* delta;        // [B, H_q, L_q] workspace (softmax; abs-sum family: delta where r > 1, signed for |sum|, else 0)
  float* dQ;           // [B, H_q, L_q, D_qk] contiguous fp32
  float* dK;           // [B, H_kv, L_k, D_qk]
  float* dV;           // [B, H_kv, L_k, D_v]
  int B, H_q, H_kv, L_q, L_k, g;
  int o_bf16;
  int64_t qs[3], ks[3], vs[3], os[3];  // element strides {batch, head, row} of Q, K, V, O
  float c2;     // scale * log2(e)
  float b2;     // bias * log2(e)
  float scale;
  // bias-tensor kernels: additive bias per (query, key), bf16, element strides bs[] = {batch, head, row};
  // bunit: log2(e) where the scores are kept in powers of two (softmax, sigmoid), else 1
  const __bf16* bias;
  int64_t bs[3];
  float bunit;
  // optional gradient of the bias tensor, bf16 [B, H_q, L_q, dbias_ld] (per batch and head, not summed over
  // sharers); written by the query-side kernel for the sub-tiles it visits
  __bf16* dbias;
  int64_t dbias_ld;
  // causal kernels: key j is also hidden from query i if j <= i + (L_k - L_q) - window (sliding
  // window); L_q + L_k for the plain causal mask, which hides nothing more
  int window;
  // the handle has a per-head decay: only then is the decay table read (it holds AE_MAX_DECAY_HEADS entries, and
  // handles without decay may have more heads than that)
  int has_decay;
  // (batch, k/v head) groups that one XCD walks together, per kernel ([0]: query side, [1]: key side); see the
  // mapping at the top of attn_bwd_kernel
  int together[2];
};

// Chunk swizzle of the backward tiles.  A tile row is read both ways -- 128-bit row
// fragments, 16 lanes = 16 consecutive rows at a time, and 64-bit transposing loads, 32
// lanes = 4 consecutive rows x 4 chunks at a time -- so the XOR pattern takes 16 values
// over 16 consecutive rows (rows of 128 or 384 bytes alternate between the halves of the
// 256-byte bank window, which supplies one of the four bits) and its upper bits change
// within every aligned group of 4 rows.
template <int CPR>
__device__ __forceinline__ int bswz(int row) {
  return CPR % 16 == 0 ? ((4 * (row & 3)) | ((row >> 2) & 3)) : ((4 * ((row >> 1) & 1)) | ((row >> 2) & 3));
}

// no normalization with the ReLU modification (the forward kernels carry the modification as a
// parameter of its own; here the pair is one more value of the NORM parameter)
constexpr int BWD_NORM_NONE_RELU = 5;
enum : int { BWD_DQ = 0, BWD_DKV = 1 };  // the query-side kernel (dQ), the key-side kernel (dK and dV)

#ifndef AE_BWD_OCC2_REGS
#define AE_BWD_OCC2_REGS 176
#endif
template <int DQK_, int DV_, int NORM_, bool CAUSAL_, int OUT_, bool BIAS_ = false>
struct BwdCfg {
  static constexpr bool BIAS = BIAS_;  // S' = scale * S + bias[b, h_q, i, j]
  static constexpr int DQK = DQK_, DV = DV_, NORM = NORM_, OUT = OUT_;
  static constexpr bool CAUSAL = CAUSAL_, KV_SIDE = OUT_ == BWD_DKV;
  static constexpr int WAVES = 4, THREADS = 256, OWN = 128;  // own rows per workgroup
  static constexpr int T1 = DQK / 16, T2 = DV / 16;
  static constexpr int DB = DQK / 32;  // 32-row blocks of the transposed result dQ^T / dK^T
  static constexpr bool HAS2 = KV_SIDE;               // key side: a second result, dV^T
  static constexpr int DB2 = HAS2 ? DV / 32 : 0;
  // Two workgroups per CU (two waves per SIMD, 256 registers each) where the accumulators, the
  // resident operands and the two score tiles leave room for the rest; one (512 registers) otherwise.
  // bias tensor: per stage the block of it that the tile meets, 16 KB: [128 own queries][64 keys] on the query
  // side, [64 queries][128 own keys] on the key side
  static constexpr int BIAS_BYTES = BIAS_ ? 16384 : 0;
  // (row quantities pass through LDS on the key side only, see ROW_BYTES)
  static constexpr bool OCC2 = 16 * (DB + DB2) + 4 * T1 + 4 * T2 + 32 + (BIAS_ ? 8 : 0) <= AE_BWD_OCC2_REGS &&
                               2 * 64 * (DQK + DV) * 2 + (KV_SIDE ? 1024 : 0) + 2 * BIAS_BYTES <= 80 * 1024;
  // one workgroup per CU: the LDS fragments of a step are read as a batch ahead of its MFMAs
  static constexpr bool BATCH = !OCC2 && DQK + DV <= 320;  // (beyond that the batches do not fit 512 registers)
  static constexpr int TILE = 64;  // other-side rows per LDS tile (two 32-row sub-tiles)
  static constexpr int RB1 = DQK * 2, RB2 = DV * 2, CPR1 = DQK / 8, CPR2 = DV / 8;
  static constexpr int Y1_BYTES = TILE * RB1, Y2_BYTES = TILE * RB2, STAGE_BYTES = Y1_BYTES + Y2_BYTES;
  // per stage: bias*log2(e) - lse*log2(e) and delta of the tile's rows (key side: they belong to the registers' rows;
  // on the query side they belong to the lane's own row and stay in registers)
  static constexpr int ROW_BYTES = KV_SIDE ? 2 * TILE * 4 : 0;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES + 2 * ROW_BYTES + 2 * BIAS_BYTES;
  static_assert(NORM == NORM_SOFTMAX || NORM == NORM_SIGMOID || NORM == NORM_NONE || NORM == BWD_NORM_NONE_RELU ||
                    NORM == NORM_ABSSUM || NORM == NORM_ABS_OF_SUM,
                "backward: softmax, sigmoid, the abs-sum family, and no normalization with or without ReLU");
  static constexpr bool ABS = NORM == NORM_ABSSUM || NORM == NORM_ABS_OF_SUM;
  static constexpr bool ROWS = NORM == NORM_SOFTMAX || ABS;  // per-row quantities from the forward statistic and delta
  // no normalization (without ReLU) is the abs-sum form with the row factors fixed at 1 and 0: P = S', dS' = dP,
  // per-head decay included
  static constexpr bool LIN = ABS || NORM == NORM_NONE;
  static_assert(LDS_BYTES <= (OCC2 ? 80 : 160) * 1024, "the workgroups of a CU must fit LDS");
  static_assert((TILE * CPR1 / 64) % WAVES == 0 && (TILE * CPR2 / 64) % WAVES == 0, "every wave copies the same number of blocks");
};

__device__ __forceinline__ bf16x8 read_tr_frag(uint32_t addr_lo, uint32_t addr_hi) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)addr_lo);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)addr_hi);
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

__device__ __forceinline__ bf16x8 pack8(const float (&x)[16], int t) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (__bf16)x[8 * t + e];
  return r;
}

template <class C>
__global__ __launch_bounds__(C::THREADS, C::OCC2 ? 2 : 1) void attn_bwd_kernel(const BwdParams p, const DecayTable dt) {
  __shared__ __attribute__((aligned(1024))) char smem[C::LDS_BYTES];
  const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_char*)smem);
  const uint32_t rows0 = lds0 + 2 * C::STAGE_BYTES;
  const uint32_t bias0 = rows0 + 2 * C::ROW_BYTES;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane & 31, half = lane >> 5;
  const int off = p.L_k - p.L_q;
  const int L_own = C::KV_SIDE ? p.L_k : p.L_q, L_oth = C::KV_SIDE ? p.L_q : p.L_k;

  // ---- which rows this workgroup owns ----------------------------------------------
  const int n_heads = C::KV_SIDE ? p.H_kv : p.H_q;
  const int n_own_tiles = (L_own + C::OWN - 1) / C::OWN;
  // Workgroups are dealt to the 8 XCDs round-robin, and each XCD has its own L2.  All workgroups of one (batch,
  // k/v head) group -- its own tiles, times the q heads of the group on the query side -- go to one XCD and run
  // there at the same time, `together` groups side by side: they stream the same rows of the other side a few
  // tiles apart, so a tile that one of them pulled into L2 serves the others.  Within a set of groups the
  // workgroups with most work come first (causal).  The grid is padded to whole sets; the surplus exits here.
  const int n_groups = p.B * p.H_kv;
  const int per_group = C::KV_SIDE ? n_own_tiles : n_own_tiles * p.g;
  const int tg = p.together[C::KV_SIDE ? 1 : 0];
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int set = slot / (tg * per_group), within = slot % (tg * per_group);
  const int item = within / tg, group = (set * tg + within % tg) * 8 + xcd;
  if (group >= n_groups) return;
  const int b = group / p.H_kv, hk = group % p.H_kv;
  int ot = C::KV_SIDE ? item : n_own_tiles - 1 - item / p.g;
  const int ho = C::KV_SIDE ? hk : hk * p.g + item % p.g;  // ho: k/v head (key side) or q head (query side)
  const int own0 = ot * C::OWN, ow0 = own0 + wave * 32;  // first own row of the workgroup / of this wave
  const int own = ow0 + ln;                              // this lane's own row (column of S, dP, G^T)
  const int own_c = own < L_own ? own : L_own - 1;

  // ---- own operands: B fragments, straight from global memory ------------------------
  const __bf16* x1 = C::KV_SIDE ? p.K + b * p.ks[0] + hk * p.ks[1] + (int64_t)own_c * p.ks[2]
                                : p.Q + b * p.qs[0] + ho * p.qs[1] + (int64_t)own_c * p.qs[2];
  const __bf16* x2 = C::KV_SIDE ? p.V + b * p.vs[0] + hk * p.vs[1] + (int64_t)own_c * p.vs[2]
                                : p.dO + (((int64_t)b * p.H_q + ho) * p.L_q + own_c) * C::DV;
  bf16x8 xb1[C::T1], xb2[C::T2];
#pragma unroll
  for (int t = 0; t < C::T1; ++t) xb1[t] = *reinterpret_cast<const bf16x8*>(x1 + (2 * t + half) * 8);
#pragma unroll
  for (int t = 0; t < C::T2; ++t) xb2[t] = *reinterpret_cast<const bf16x8*>(x2 + (2 * t + half) * 8);
  // query side: the row quantities belong to the lane's own row
  // (first: (bias - lse) * log2(e) for softmax, 1 / max(|statistic|, 1) for the abs-sum family; second: delta)
  float nl_own = C::LIN ? 1.f : -INFINITY, dl_own = 0.f;
  if constexpr (!C::KV_SIDE && C::ROWS) {
    if (own < p.L_q) {
      const int64_t r = ((int64_t)b * p.H_q + ho) * p.L_q + own;
      const float st = p.lse[r];
      if constexpr (C::ABS) nl_own = fast_rcp(fmaxf(fabsf(st), 1.f));
      else nl_own = st == -INFINITY ? -INFINITY : p.b2 - st * 1.4426950408889634f;
      dl_own = p.delta[r];
    }
  }
  float lg = 0.f;  // log2 of the decay rate of the q head at hand (0: no decay); key side: set per tile
  if constexpr (!C::KV_SIDE && C::LIN) lg = p.has_decay ? dt.log2_gamma[ho] : 0.f;

  // ---- the walk over the other side --------------------------------------------------
  // key side: the query tiles from the first one that sees key own0, for each q head of
  // the group; query side: the key tiles up to the last one that row own0 + 127 sees.
  int t_first = 0, t_end = (L_oth + C::TILE - 1) / C::TILE;
  if constexpr (C::CAUSAL) {
    if constexpr (C::KV_SIDE) {
      const int i_first = own0 - off;  // first query that sees key own0
      t_first = i_first > 0 ? i_first / C::TILE : 0;
      if (t_first > t_end) t_first = t_end;
      const int i_last = own0 + C::OWN - 1 - off + p.window - 1;  // last query whose window holds a key here
      const int e = i_last < 0 ? 0 : i_last / C::TILE + 1;
      if (e < t_end) t_end = e;
      if (t_end < t_first) t_end = t_first;
    } else {
      const int j_last = own0 + C::OWN - 1 + off;  // last key any row here may see
      const int e = j_last < 0 ? 0 : j_last / C::TILE + 1;
      if (e < t_end) t_end = e;
      const int j_first = own0 + off - p.window + 1;  // first key inside the window of row own0
      t_first = j_first > 0 ? j_first / C::TILE : 0;
      if (t_first > t_end) t_first = t_end;
    }
  }
  const int nt = t_end - t_first;
  const int total = C::KV_SIDE ? nt * p.g : nt;

  // LDS-DMA maps: block nb of a tile = 64 chunks of 16 bytes, linear in LDS; position ->
  // (row, physical chunk), the logical chunk is the physical one XOR the row's swizzle.
  auto issue_tile = [&](int n, int stage) {
    const int hq = C::KV_SIDE ? hk * p.g + n / nt : ho;
    const int r0 = (t_first + (C::KV_SIDE ? n % nt : n)) * C::TILE;
    const __bf16* y1 = C::KV_SIDE ? p.Q + b * p.qs[0] + hq * p.qs[1] : p.K + b * p.ks[0] + hk * p.ks[1];
    const __bf16* y2 = C::KV_SIDE ? p.dO + ((int64_t)b * p.H_q + hq) * p.L_q * C::DV : p.V + b * p.vs[0] + hk * p.vs[1];
    const int64_t s1 = C::KV_SIDE ? p.qs[2] : p.ks[2], s2 = C::KV_SIDE ? (int64_t)C::DV : p.vs[2];
    const uint32_t base = lds0 + stage * C::STAGE_BYTES;
#pragma unroll
    for (int i = 0; i < C::TILE * C::CPR1 / 64 / C::WAVES; ++i) {
      const int nb = wave + i * C::WAVES, pos = nb * 64 + lane;
      const int r = pos / C::CPR1, pc = pos % C::CPR1;
      int row = r0 + r;
      row = row < L_oth ? row : L_oth - 1;
      const uint32_t goff = (uint32_t)(((int64_t)row * s1 + ((pc ^ bswz<C::CPR1>(r)) * 8)) * 2);
      dma16(y1, goff, base + nb * 1024);
    }
#pragma unroll
    for (int i = 0; i < C::TILE * C::CPR2 / 64 / C::WAVES; ++i) {
      const int nb = wave + i * C::WAVES, pos = nb * 64 + lane;
      const int r = pos / C::CPR2, pc = pos % C::CPR2;
      int row = r0 + r;
      row = row < L_oth ? row : L_oth - 1;
      const uint32_t goff = (uint32_t)(((int64_t)row * s2 + ((pc ^ bswz<C::CPR2>(r)) * 8)) * 2);
      dma16(y2, goff, base + C::Y1_BYTES + nb * 1024);
    }
    if constexpr (C::BIAS) {
      // The block of the bias tensor that this tile meets, rows = queries.  Query side: 128 rows x 128 bytes
      // (8 chunks), chunk slot c ^ ((row >> 1) & 7); key side: 64 rows x 256 bytes (16 chunks), slot
      // c ^ ((row & 3) << 2) (read back transposed, 4 rows x 64 bytes at a time).  Chunks that start beyond the
      // last key are redirected to the row's last chunk (rows are padded to 8 elements by contract).
      const __bf16* bb = p.bias + b * p.bs[0] + hq * p.bs[1];
      constexpr int CPRB = C::KV_SIDE ? 16 : 8;
      const int q0 = C::KV_SIDE ? r0 : own0, k0 = C::KV_SIDE ? own0 : r0;
      const int last = ((p.L_k - 1) >> 3) << 3;
#pragma unroll
      for (int i = 0; i < 16 / C::WAVES; ++i) {
        const int nb = wave + i * C::WAVES, pos = nb * 64 + lane;
        const int r = pos / CPRB, pc = pos % CPRB;
        const int c = C::KV_SIDE ? pc ^ ((r & 3) << 2) : pc ^ ((r >> 1) & 7);
        int row = q0 + r, col = k0 + 8 * c;
        row = row < p.L_q ? row : p.L_q - 1;
        col = col < p.L_k ? col : last;
        dma16(bb, (uint32_t)(((int64_t)row * p.bs[2] + col) * 2), bias0 + stage * C::BIAS_BYTES + nb * 1024);
      }
    }
  };
  // key side: the tile's row quantities, wave 0 -> (bias - lse) * log2(e), wave 1 -> delta.  The
  // values are requested when the tile's copy starts and only touched (converted, written to LDS)
  // after the work on the tile before it: nothing waits for memory in between.
  auto load_rowq = [&](int n) -> float {
    float v = 0.f;
    if constexpr (C::KV_SIDE && C::ROWS) {
      if (wave < 2 && lane < C::TILE) {
        const int hq = hk * p.g + n / nt;
        const int i = (t_first + n % nt) * C::TILE + lane;
        const int64_t r = ((int64_t)b * p.H_q + hq) * p.L_q + i;
        const float* src = wave == 0 ? p.lse : p.delta;
        v = wave == 0 ? (C::ABS ? 0.f : -INFINITY) : 0.f;
        if (i < p.L_q) v = src[r];
      }
    }
    return v;
  };
  auto store_rowq = [&](float v, int stage) {
    if constexpr (C::KV_SIDE && C::ROWS) {
      if (wave < 2 && lane < C::TILE) {
        if (wave == 0) v = C::ABS ? fast_rcp(fmaxf(fabsf(v), 1.f)) : v == -INFINITY ? -INFINITY : p.b2 - v * 1.4426950408889634f;
        *reinterpret_cast<__attribute__((address_space(3))) float*>(
            (lds_char*)(uintptr_t)(rows0 + stage * C::ROW_BYTES + wave * C::TILE * 4 + lane * 4)) = v;
      }
    }
  };

  f32x16 g[C::DB], g2[C::HAS2 ? C::DB2 : 1];
#pragma unroll
  for (int d = 0; d < C::DB; ++d) g[d] = zero16();
#pragma unroll
  for (int d = 0; d < C::DB2; ++d) g2[d] = zero16();

  // Per-lane LDS addresses of the fragments in stage 0, sub-tile 0, step 0; stage, sub-tile and
  // 16-row step add compile-time constants (the swizzle only depends on the row modulo 16).
  //   ar1[t], ar2[t]: row fragment of contraction step t, row lane % 32 (A operand of S / dP);
  //   atl[k], ath[k]: the two transposing reads of 32-column block k, rows 4*half + i/4 (+8).
  constexpr int RBT = C::RB1;  // row bytes of the Y1 tile, read transposed for dQ^T / dK^T
  const int f1 = bswz<C::CPR1>(ln), f2 = bswz<C::CPR2>(ln);
  const int li = lane & 15, blk = (lane >> 4) & 1;
  const int trow = 4 * half + (li >> 2), tcl = 2 * blk + ((li & 3) >> 1);
  const int flo = bswz<RBT / 16>(trow), fhi = bswz<RBT / 16>(trow + 8);
  const uint32_t rb1 = lds0 + ln * C::RB1, rb2 = lds0 + C::Y1_BYTES + ln * C::RB2;
  const uint32_t tbl = lds0 + (li & 1) * 8 + trow * RBT, tbh = tbl + 8 * RBT;
  auto a_r1 = [&](int t) { return rb1 + (((2 * t + half) ^ f1) << 4); };
  auto a_r2 = [&](int t) { return rb2 + (((2 * t + half) ^ f2) << 4); };
  auto a_tl = [&](int k) { return tbl + (((4 * k + tcl) ^ flo) << 4); };
  auto a_th = [&](int k) { return tbh + (((4 * k + tcl) ^ fhi) << 4); };
  uint32_t ar1[C::T1], ar2[C::T2], atl[C::DB], ath[C::DB];
  uint32_t atl2[C::HAS2 ? C::DB2 : 1], ath2[C::HAS2 ? C::DB2 : 1];  // fused kernel: the same for the Y2 tile
  if constexpr (C::HAS2) {
    const int glo = bswz<C::CPR2>(trow), ghi = bswz<C::CPR2>(trow + 8);
    const uint32_t t2 = lds0 + C::Y1_BYTES + (li & 1) * 8 + trow * C::RB2;
#pragma unroll
    for (int k = 0; k < C::DB2; ++k) {
      atl2[k] = t2 + (((4 * k + tcl) ^ glo) << 4);
      ath2[k] = t2 + 8 * C::RB2 + (((4 * k + tcl) ^ ghi) << 4);
    }
  }
  {
#pragma unroll
    for (int t = 0; t < C::T1; ++t) ar1[t] = a_r1(t);
#pragma unroll
    for (int t = 0; t < C::T2; ++t) ar2[t] = a_r2(t);
#pragma unroll
    for (int k = 0; k < C::DB; ++k) {
      atl[k] = a_tl(k);
      ath[k] = a_th(k);
    }
  }

  // One 32-row sub-tile of the other side (STAGE, SUB: compile-time LDS position; o0: its first row).
  auto subtile = [&](auto stagec, auto subc, int o0) {
    constexpr int STAGE = decltype(stagec)::value, SUB = decltype(subc)::value;
    // anything visible to this wave's rows?  everything?
    bool any = o0 < L_oth, full = o0 + 31 < L_oth;
    if constexpr (C::CAUSAL) {
      const int wd = p.window;
      if constexpr (C::KV_SIDE) {  // own = keys j, other = queries i: visible iff i + off - window < j <= i + off
        any = any && ow0 <= o0 + 31 + off && o0 + off - wd < ow0 + 31;
        full = full && ow0 + 31 <= o0 + off && o0 + 31 + off - wd < ow0;
      } else {                     // own = queries i, other = keys j
        any = any && o0 <= ow0 + 31 + off && ow0 + off - wd < o0 + 31;
        full = full && o0 + 31 <= ow0 + off && ow0 + 31 + off - wd < o0;
      }
    }
    if (!any) return;
    constexpr uint32_t kRow1 = STAGE * C::STAGE_BYTES + SUB * 32 * C::RB1, kRow2 = STAGE * C::STAGE_BYTES + SUB * 32 * C::RB2;
    // key side: the row quantities of the 16 rows this lane sees, requested ahead of the MFMAs that
    // hide their latency (register r is other-side row o0 + 8*(r/4) + 4*half + (r%4))
    constexpr uint32_t kRq = 2 * C::STAGE_BYTES + STAGE * C::ROW_BYTES + SUB * 32 * 4;
    constexpr bool ROWQ = C::ROWS && C::KV_SIDE;
    f32x4 nl4[4], dl4[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      nl4[q] = f32x4{nl_own, nl_own, nl_own, nl_own};
      dl4[q] = f32x4{dl_own, dl_own, dl_own, dl_own};
      if constexpr (ROWQ) nl4[q] = lds_read16(lds0 + kRq + (8 * q + 4 * half) * 4);
    }
    if constexpr (ROWQ) sched_fence();
    f32x16 s = zero16(), dp = zero16();
    // the fragments of the accumulation step: tr[t][k], k < DB from Y1, the rest (key side) from Y2
    constexpr uint32_t kT = STAGE * C::STAGE_BYTES + SUB * 32 * RBT, kT2 = STAGE * C::STAGE_BYTES + SUB * 32 * C::RB2;
    auto read_acc = [&](int t, int k) {
      if constexpr (C::HAS2) {
        if (k >= C::DB) return read_tr_frag(atl2[k - C::DB] + kT2 + t * 16 * C::RB2, ath2[k - C::DB] + kT2 + t * 16 * C::RB2);
      }
      return read_tr_frag(atl[k < C::DB ? k : 0] + kT + t * 16 * RBT, ath[k < C::DB ? k : 0] + kT + t * 16 * RBT);
    };
    bf16x8 tr[2][C::BATCH ? C::DB + C::DB2 : 1];
    if constexpr (C::BATCH) {
      // One wave per SIMD: nothing else hides the LDS latency, so all fragments of a step are
      // requested before its first MFMA, and those of the accumulation step before the elementwise
      // step (the fences keep the compiler from sinking the reads back to their uses).
      bf16x8 a1[C::T1], a2[C::T2];
#pragma unroll
      for (int t = 0; t < C::T1; ++t) a1[t] = read_k_frag(ar1[t] + kRow1);
#pragma unroll
      for (int t = 0; t < C::T2; ++t) a2[t] = read_k_frag(ar2[t] + kRow2);
      sched_fence();
#pragma unroll
      for (int t = 0; t < C::T1; ++t) s = mfma(a1[t], xb1[t], s);
#pragma unroll
      for (int t = 0; t < C::T2; ++t) dp = mfma(a2[t], xb2[t], dp);
      sched_fence();
#pragma unroll
      for (int k = 0; k < C::DB + C::DB2; ++k) tr[0][k] = read_acc(0, k);
      sched_fence();
    } else {
#pragma unroll
      for (int t = 0; t < C::T1; ++t) s = mfma(read_k_frag(ar1[t] + kRow1), xb1[t], s);
#pragma unroll
      for (int t = 0; t < C::T2; ++t) dp = mfma(read_k_frag(ar2[t] + kRow2), xb2[t], dp);
    }
    float x[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = __builtin_fmaf(s[r], p.c2, C::NORM == NORM_SOFTMAX ? nl4[r / 4][r % 4] : p.b2);
    if constexpr (C::BIAS) {
      // register r = 4 q4 + e is (query, key) = (own row, key 8 q4 + 4 half + e of the sub-tile) on the query side,
      // (query 8 q4 + 4 half + e of the sub-tile, own key) on the key side
      const uint32_t bt = bias0 + STAGE * C::BIAS_BYTES;
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        uint32_t lo, hi;
        if constexpr (C::KV_SIDE) {
          const int row = 32 * SUB + 8 * q4 + 4 * half + ((lane & 15) >> 2);   // the row this lane addresses
          const int cl = 4 * wave + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);  // chunk of its 4 columns
          const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)(
              bt + row * 256 + ((cl ^ ((row & 3) << 2)) << 4) + (lane & 1) * 8));
          const u32x2 w2 = __builtin_bit_cast(u32x2, v);
          lo = w2[0];
          hi = w2[1];
        } else {
          const int row = 32 * wave + ln;
          const u32x2 w2 = *reinterpret_cast<__attribute__((address_space(3))) const u32x2*>(
              (lds_char*)(uintptr_t)(bt + row * 128 + (((4 * SUB + q4) ^ ((row >> 1) & 7)) << 4) + 8 * half));
          lo = w2[0];
          hi = w2[1];
        }
        x[4 * q4 + 0] += __builtin_bit_cast(float, lo << 16) * p.bunit;
        x[4 * q4 + 1] += __builtin_bit_cast(float, lo & 0xffff0000u) * p.bunit;
        x[4 * q4 + 2] += __builtin_bit_cast(float, hi << 16) * p.bunit;
        x[4 * q4 + 3] += __builtin_bit_cast(float, hi & 0xffff0000u) * p.bunit;
      }
    }
    // abs-sum family: distance to the diagonal of register 0's entry, for the decay factor
    const float dist0 = (float)(C::KV_SIDE ? o0 + off - own + 4 * half : own + off - o0 - 4 * half);
    if (!full) {  // a hidden entry gets the exponent that makes its weight exactly 0
      sched_fence();  // (keeps this a branch: most sub-tiles skip it)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int oth = o0 + key_offset(r) + 4 * half;
        bool vis = oth < L_oth;
        if constexpr (C::CAUSAL)
          vis = vis && (C::KV_SIDE ? own <= oth + off && oth + off - p.window < own : oth <= own + off && own + off - p.window < oth);
        x[r] = vis ? x[r] : -INFINITY;
      }
      sched_fence();
    }
    float w[16], w2[C::HAS2 ? 16 : 1];  // the weight (dV) or the score gradient (dQ, dK); fused: both
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      if constexpr (ROWQ)
        if (r % 4 == 0) dl4[r / 4] = lds_read16(lds0 + kRq + C::TILE * 4 + (8 * (r / 4) + 4 * half) * 4);
      float pv;
      if constexpr (C::NORM == NORM_SOFTMAX) {
        pv = fast_exp2(x[r]);
        if constexpr (C::HAS2) w2[r] = pv;
        pv = pv * (dp[r] - dl4[r / 4][r % 4]);
      } else if constexpr (C::NORM == NORM_SIGMOID) {
        pv = fast_rcp(1.f + fast_exp2(-x[r]));
        if constexpr (C::HAS2) w2[r] = pv;
        pv = dp[r] * pv * (1.f - pv);
      } else if constexpr (C::LIN) {  // a hidden entry has x = -inf: weight and gradient 0
        const bool vis = x[r] != -INFINITY;
        const float dist = dist0 + (C::KV_SIDE ? 1.f : -1.f) * (float)key_offset(r);
        const float dec = fast_exp2(lg * fmaxf(dist, 0.f));  // (visible entries have dist >= 0; <= 1 keeps 0 * dec finite)
        const float sp = (vis ? x[r] : 0.f) * dec;          // S'
        const float inv = nl4[r / 4][r % 4], dl = dl4[r / 4][r % 4];
        if constexpr (C::HAS2) w2[r] = sp * inv;
        // g * delta: delta with its sign flipped where S' < 0 (abs-sum), or delta already signed by the row sum
        const float corr = C::NORM == NORM_ABSSUM
                               ? __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, dl) ^ (__builtin_bit_cast(uint32_t, sp) & 0x80000000u))
                               : dl;
        pv = vis ? (dp[r] - corr) * inv * dec : 0.f;
      } else if constexpr (C::NORM == BWD_NORM_NONE_RELU) {  // P = max(x, 0); a hidden entry has x = -inf
        if constexpr (C::HAS2) w2[r] = fmaxf(x[r], 0.f);
        pv = x[r] > 0.f ? dp[r] : 0.f;
      }
      w[r] = pv;
    }
    if constexpr (C::BIAS && !C::KV_SIDE) {
      // the bias enters S' with slope 1: its gradient is dS' itself, 4 x 4 consecutive keys of the lane's own row
      if (p.dbias != nullptr && own < p.L_q) {
        __bf16* drow = p.dbias + (((int64_t)b * p.H_q + ho) * p.L_q + own) * p.dbias_ld + o0 + 4 * half;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          if (o0 + 8 * q4 + 4 * half < p.L_k) {  // (a group across the last key writes into the row's padding)
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (__bf16)w[4 * q4 + e];
            *reinterpret_cast<bf16x4*>(drow + 8 * q4) = v;
          }
      }
    }
    // G^T += Y^T W: per 16-row step t, the DB blocks of Y1^T (dQ^T, dK^T), then (key side) the DB2 blocks of Y2^T
    if constexpr (C::BATCH) {
      sched_fence();
#pragma unroll
      for (int k = 0; k < C::DB + C::DB2; ++k) tr[1][k] = read_acc(1, k);
      sched_fence();
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const bf16x8 wb = pack8(w, t);
#pragma unroll
      for (int k = 0; k < C::DB; ++k) g[k] = mfma(C::BATCH ? tr[t][C::BATCH ? k : 0] : read_acc(t, k), wb, g[k]);
      if constexpr (C::HAS2) {
        const bf16x8 pb = pack8(w2, t);
#pragma unroll
        for (int k = 0; k < C::DB2; ++k)
          g2[k] = mfma(C::BATCH ? tr[t][C::BATCH ? C::DB + k : 0] : read_acc(t, C::DB + k), pb, g2[k]);
      }
    }
  };
  // Tile n: wait for it, start the copy of tile n + 1 into the other stage, work on it.
  auto tile = [&](auto stagec, int n) {
    constexpr int STAGE = decltype(stagec)::value;
    // tile n has landed, and every wave is done with the stage that tile n + 1 goes to
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
    float rowq_next = 0.f;
    if (n + 1 < total) {
      issue_tile(n + 1, STAGE ^ 1);
      rowq_next = load_rowq(n + 1);
    }
    const int r0 = (t_first + (C::KV_SIDE ? n % nt : n)) * C::TILE;
    if constexpr (C::KV_SIDE && C::LIN) lg = p.has_decay ? dt.log2_gamma[hk * p.g + n / nt] : 0.f;
    subtile(stagec, std::integral_constant<int, 0>{}, r0);
    subtile(stagec, std::integral_constant<int, 1>{}, r0 + 32);
    if (n + 1 < total) store_rowq(rowq_next, STAGE ^ 1);
  };

  if (total > 0) {
    issue_tile(0, 0);
    store_rowq(load_rowq(0), 0);
  }
  // Everything loaded so far is consumed here once.  Otherwise the compiler, which must assume at
  // the loop's entry that those loads may still be in flight, waits for vmcnt to drain in front of
  // the MFMAs inside the loop -- and vmcnt also counts the tile copies, so every tile would wait for
  // the copy of the next one instead of running beside it.
#pragma unroll
  for (int t = 0; t < C::T1; ++t) asm volatile("" ::"v"(xb1[t]));
#pragma unroll
  for (int t = 0; t < C::T2; ++t) asm volatile("" ::"v"(xb2[t]));
  asm volatile("" ::"v"(nl_own), "v"(dl_own));
  for (int n = 0; n < total; n += 2) {
    tile(std::integral_constant<int, 0>{}, n);
    if (n + 1 < total) tile(std::integral_constant<int, 1>{}, n + 1);
  }

  // ---- results: register r of block db is column own, row d = 32 db + 8 (r/4) + 4 half + r%4 ----
  if (own < L_own) {
    constexpr int D = C::DQK;
    float* o = (C::KV_SIDE ? p.dK + ((int64_t)b * p.H_kv + hk) * p.L_k * D : p.dQ + ((int64_t)b * p.H_q + ho) * p.L_q * D) +
               (int64_t)own * D;
    const float f = p.scale;
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
      for (int q = 0; q < 4; ++q)
        *reinterpret_cast<f32x4*>(o + 32 * db + 8 * q + 4 * half) =
            f32x4{g[db][4 * q] * f, g[db][4 * q + 1] * f, g[db][4 * q + 2] * f, g[db][4 * q + 3] * f};
    if constexpr (C::HAS2) {
      float* o2 = p.dV + (((int64_t)b * p.H_kv + hk) * p.L_k + own) * C::DV;
#pragma unroll
      for (int db = 0; db < C::DB2; ++db)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *reinterpret_cast<f32x4*>(o2 + 32 * db + 8 * q + 4 * half) =
              f32x4{g2[db][4 * q], g2[db][4 * q + 1], g2[db][4 * q + 2], g2[db][4 * q + 3]};
    }
  }
}

}  // namespace ae
