// Fused parallel-pattern attention forward kernel for gfx950 (CDNA4).
//
// One workgroup owns BLOCK_M = 32*QB*WAVES query rows of one (batch, q-head); each
// wavefront owns QB blocks of 32 of them and walks the visible key/value tiles of
// BLOCK_N = 32*NKB keys.  Per tile (paper Section 4.1: parallel pattern with
// the online row-norm interface):
//   relevance scoring   S^T = K_tile Q^T          (bf16 MFMA 32x32x16, fp32 acc)
//   modification        scale / bias / decay / relu / mask, in registers
//   online row-norm     per-row running state (max+sum, or abs-sum), registers
//   aggregation         O^T += V_tile^T P^T       (bf16 MFMA, fp32 acc)
//
// Why the transposed products: in the 32x32 accumulator layout a lane owns ONE
// column and 16 rows.  With S^T (rows = keys, columns = queries) every value a
// lane holds belongs to a single query, so the row reductions of the
// normalization are in-lane plus one exchange between lane l and lane l^32, the
// per-row rescale of O is a per-lane scalar, and the accumulator registers of
// S^T are, with no data movement, the B operand of the second MFMA: the order
// in which keys are contracted is free, so V is read from LDS in the key order
// that the accumulator layout dictates (ds_read_b64_tr_b16 does the transpose).
//
// The key loop is software-pipelined inside each wavefront so that matrix and
// vector work of DIFFERENT tiles sit in the same basic block:
//   phase A(j):  S(j+1) = K(j+1) Q^T   (MFMA)  ||  weights P(j) from S(j)   (VALU)
//   phase B(j):  O += V(j)^T P(j)      (MFMA)  ||  mask / row max of S(j+1) (VALU)
// K therefore runs one tile ahead of V through the double-buffered LDS.
//
// K/V tiles go from global memory straight into LDS (global_load_lds_dwordx4:
// no staging registers, no ds_write): a wave instruction fills 1 KB of LDS
// linearly, lane l supplying bytes 16*l.., while the global address is free per
// lane.  The tiles are therefore stored unpadded and the bank spreading is done
// by an XOR swizzle of the 16-byte chunk index, applied on the global-address
// side when loading and on the LDS-address side when reading fragments.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

// Optional phase timing (build with -DAE_PROFILE): per-wave cycle totals between
// the marked points are written to the buffer passed in Params::prof.
#ifndef AE_MFMA_PRIO
#define AE_MFMA_PRIO 2
#endif
#ifdef AE_PROFILE
#define AE_TICK(k)                                            \
  do {                                                        \
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");        \
    const uint64_t now_ = __builtin_readcyclecounter();       \
    prof_acc[k] += now_ - prof_last;                          \
    prof_last = now_;                                         \
  } while (0)
#else
#define AE_TICK(k) do { } while (0)
#endif

namespace ae {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
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
  int map_mode; // experiment: workgroup -> tile mapping
  unsigned long long* prof;  // AE_PROFILE builds: [grid][waves][8] cycle totals, else unused
};

struct DecayTable {
  float log2_gamma[kMaxDecayHeads];
};

template <int DQK_, int DV_, int NORM_, int MOD_, bool CAUSAL_, int WAVES_, int NKB_, int QB_, int STAGES_, bool PIPE_>
struct Cfg {
  static constexpr int DQK = DQK_, DV = DV_, NORM = NORM_, MOD = MOD_, WAVES = WAVES_, NKB = NKB_, QB = QB_;
  static constexpr bool CAUSAL = CAUSAL_;
  static constexpr int BLOCK_N = 32 * NKB;
  static constexpr int BLOCK_M = 32 * QB * WAVES;
  static constexpr int THREADS = 64 * WAVES;
  // LDS tiles are row-major and unpadded; CPR = 16-byte chunks per row.
  static constexpr int RB_K = DQK * 2, RB_V = DV * 2;
  static constexpr int CPR_K = DQK / 8, CPR_V = DV / 8;
  static constexpr int K_BYTES = BLOCK_N * RB_K;
  static constexpr int V_BYTES = BLOCK_N * RB_V;
  // K/V tiles are fetched AHEAD tiles before use into rings of STAGES buffers.
  static constexpr int STAGES = STAGES_, AHEAD = STAGES - 1;
  // PIPE: phase A of a step scores the NEXT tile while the weights of the current
  // one are computed (needs a second set of score registers).  Without it every
  // step scores, normalises and aggregates one tile in sequence and relies on
  // the second wave of the SIMD for overlap.
  static constexpr bool PIPE = PIPE_;
  static constexpr int LDS_BYTES = STAGES * (K_BYTES + V_BYTES);
  static constexpr int NB_K = K_BYTES / 1024, NB_V = V_BYTES / 1024;  // 1 KB blocks per tile
  static constexpr int KI = (NB_K + WAVES - 1) / WAVES, VI = (NB_V + WAVES - 1) / WAVES;
  static constexpr int LOADS_PER_STEP = KI + VI;  // wave-level DMA instructions per tile pair
  static_assert(AHEAD * LOADS_PER_STEP <= 63, "vmcnt cannot count that many loads in flight");
  static_assert(K_BYTES % 1024 == 0 && V_BYTES % 1024 == 0, "tiles must be whole 1 KB blocks");
  static_assert(CPR_K == 8 || CPR_K == 16 || CPR_K == 24, "K swizzle is defined for these row sizes");
  static_assert(CPR_V == 8 || CPR_V == 16 || CPR_V == 32, "V swizzle is defined for these row sizes");
  static_assert(DQK % 16 == 0 && DV % 32 == 0, "head dims must fit the MFMA tile");
  static_assert(LDS_BYTES <= 160 * 1024, "tile does not fit LDS");
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
// max(a, b, c) in one instruction.  Written as asm because fmaxf() on values the
// compiler cannot prove canonical costs an extra v_max per operand in IEEE mode.
__device__ __forceinline__ float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

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
// The running softmax reference only moves when a tile's row max exceeds it by
// more than this many powers of two (weights then stay below 2^kLazyLog2).
constexpr float kLazyLog2 = 8.0f;

// ---- chunk swizzles -------------------------------------------------------------
// K fragments are read with 128-bit loads, 16 lanes at a time, one row each and
// the same logical chunk: the chunk index is XORed with a function of the row
// that takes 16 values over 16 consecutive rows (rows of 128 or 384 bytes
// alternate between the two halves of the 256-byte bank window, which supplies
// one of the four bits).
template <int CPR>
__device__ __forceinline__ int kswz(int row) {
  return CPR % 16 == 0 ? (row & 15) : ((row >> 1) & 7);
}
// V fragments are read with 64-bit transposing loads, 32 lanes covering 4
// consecutive rows x 64 bytes: groups of 4 chunks are XORed with the row index.
template <int CPR>
__device__ __forceinline__ int vswz(int row) {
  return CPR >= 16 ? (row & 3) : ((row >> 1) & 1);
}

// ---- global -> LDS, no registers in between --------------------------------------
// Element offsets (from the tile's first row) of the chunks this lane fetches
// for each of the wave's 1 KB blocks; loop invariant.
template <int WAVES, int ROWS, int CPR, bool IS_V, int N>
__device__ __forceinline__ void dma_offsets(int wave, int64_t row_stride, int (&goff)[N], int (&grow)[N]) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    constexpr int NB = ROWS * CPR / 64;
    const int p = ((wave + i * WAVES) % NB) * 64 + lane;  // chunk position in the LDS tile
    const int row = p / CPR, pc = p % CPR;
    const int c = IS_V ? (pc ^ (4 * vswz<CPR>(row))) : (pc ^ kswz<CPR>(row));
    grow[i] = row;
    goff[i] = row * (int)row_stride + c * 8;
  }
}

// Starts the copy of tile rows [j0, j0 + ROWS) into the LDS tile at `lds`.
// Rows past the end of the sequence re-read the last valid row: their scores
// are masked, and finite values keep 0 * V finite.  Every wave issues the same
// number of loads per tile (a wave with no block left repeats one: same bytes
// to the same place), so the number of loads in flight is the same everywhere
// and s_waitcnt vmcnt(n) can retire tiles in order.
//
// The instruction is issued as inline asm on purpose: for the builtin form the
// compiler tracks the LDS write and, unable to tell which buffer an LDS read
// touches, puts s_waitcnt vmcnt(0) in front of the fragment reads -- which
// serialises every step on the full latency of the copies just started.  Here
// the waits are explicit instead (wait_dma_and_sync).
__device__ __forceinline__ void dma16(const void* base_uniform, uint32_t byte_off, uint32_t lds_addr_uniform) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
      : "memory", "m0");
}

template <int WAVES, int ROWS, int CPR, int N>
__device__ __forceinline__ void dma_tile(const __bf16* base, int64_t row_stride, int j0, int L_k, uint32_t lds, int wave,
                                         const int (&goff)[N], const int (&grow)[N]) {
  constexpr int NB = ROWS * CPR / 64;
  const __bf16* tile = base + (int64_t)j0 * row_stride;  // wave-uniform
  const bool ragged = j0 + ROWS > L_k;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const int bi = (wave + i * WAVES) % NB;
    int off = goff[i];
    if (ragged) off -= max(0, j0 + grow[i] - (L_k - 1)) * (int)row_stride;
    dma16(tile, (uint32_t)off * 2u, lds + bi * 1024);
  }
}

// Waits until at most `N` of this wave's DMA loads are still in flight, then
// meets the other waves: what they waited for is visible too.  A bare s_barrier
// is used on purpose: __syncthreads() also drains every load in flight
// (vmcnt(0)), which would undo the prefetch depth.  LDS reads of the step have
// returned by then (each was awaited by the MFMA that consumed it), so a buffer
// is only overwritten after every wave is done reading it.
template <int N>
__device__ __forceinline__ void wait_dma_and_sync() {
#ifdef AE_EXP_NOBARRIER
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
#else
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
#endif
}

// Per-wave running state of the online row normalization.
template <class C>
struct RowState {
  float m;  // softmax: lazy running reference max (log2 domain)
  float l;  // softmax: running sum of weights; abs-sum family: running sum (this lane's 16*NKB keys)
  f32x16 o[C::DV / 32];
};

// Nothing may be moved across this point by the instruction scheduler.  The
// phases below are written as explicit groups "one MFMA + the LDS read for a
// later MFMA + a slice of vector work", fenced from each other, so that the
// matrix pipe always has vector work from another tile to overlap with and the
// number of fragments in flight (registers) stays bounded.
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

// A lane holds 16*NKB scores of one query per tile: element e = 16*kb + r is key
// j0 + 32*kb + 8*(r/4) + 4*half + (r%4).  Work on them is cut into pairs
// (elements 2q, 2q+1 -> one packed bf16x2 word).
__device__ __forceinline__ constexpr int key_offset(int e) { return 32 * (e / 16) + 8 * ((e % 16) / 4) + (e % 4); }

// Per-tile, per-lane constants of the modification.
struct TileCtx {
  int jlim;     // element e is visible  <=>  key_offset(e) <= jlim   (masked tiles only)
  float dbase;  // decay: log2(gamma) * (i + off - j0 - 4*half)
};

template <class C, bool MASKED>
__device__ __forceinline__ TileCtx tile_ctx(const Params& p, int i, int j0, int off, float g2) {
  const int half = (threadIdx.x & 63) >> 5;
  TileCtx c;
  c.jlim = MASKED ? min(C::CAUSAL ? i + off : p.L_k - 1, p.L_k - 1) - j0 - 4 * half : 0;
  c.dbase = C::MOD == MOD_DECAY ? g2 * (float)(i + off - j0 - 4 * half) : 0.f;
  return c;
}

// ---- modification + first half of the row norm, one pair of a scored tile -----
// Afterwards the two elements hold, per norm:
//   softmax  the raw score, -inf where masked (mx accumulates the lane's max)
//   sigmoid  2^-(scale*s + bias) in log2 units, +inf where masked
//   others   the fully modified score x, 0 where masked
template <class C, bool MASKED>
__device__ __forceinline__ void post_pair(const Params& p, int q, f32x16 (&s)[C::NKB], const TileCtx& tc, float g2,
                                          float& mx) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int e = 2 * q + u;
    float x = s[e / 16][e % 16];
    const bool hidden = MASKED && (key_offset(e) > tc.jlim);
    if constexpr (C::NORM == NORM_SOFTMAX) {
      if (hidden) x = -INFINITY;
    } else if constexpr (C::NORM == NORM_SIGMOID) {
      x = fast_exp2(__builtin_fmaf(x, -p.c, -p.b2));
      if (hidden) x = INFINITY;
    } else {
      if constexpr (C::MOD == MOD_DECAY) {
        // gamma^(i + off - j) = 2^(log2(gamma) * (i + off - j))
        x = x * p.c * fast_exp2(__builtin_fmaf(-g2, (float)key_offset(e), tc.dbase));
      } else {
        x = __builtin_fmaf(x, p.c, p.b2);
        if constexpr (C::MOD == MOD_RELU) x = fmaxf(x, 0.f);
      }
      if (hidden) x = 0.f;
    }
    s[e / 16][e % 16] = x;
  }
  if constexpr (C::NORM == NORM_SOFTMAX) {
    const int e = 2 * q;
    mx = max3(mx, s[e / 16][e % 16], s[(e + 1) / 16][(e + 1) % 16]);
  }
}

// Softmax: combines the two half rows and decides whether the lazy reference
// maximum has to move.
template <class C>
__device__ __forceinline__ void post_done(const Params& p, const RowState<C>& st, float mx, bool& moved, float& xm) {
  if constexpr (C::NORM == NORM_SOFTMAX) {
    mx = max_halves(mx);
    xm = __builtin_fmaf(mx, p.c, p.b2);  // c > 0
    moved = xm > st.m + kLazyLog2;
  }
}

// Moves the softmax reference maximum where post_done asked for it and rescales
// the running sum and the output accumulators (rare after the first tiles).
template <class C>
__device__ __forceinline__ void lazy_rescale(RowState<C>& st, bool moved, float xm) {
  if constexpr (C::NORM == NORM_SOFTMAX) {
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
      const float m_new = moved ? xm : st.m;
      const float alpha = moved ? fast_exp2(st.m - m_new) : 1.f;
      st.m = m_new;
      st.l *= alpha;
#pragma unroll
      for (int db = 0; db < C::DV / 32; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
    }
  }
}

// ---- second half of the row norm, one pair: weight -> packed bf16x2 ------------
template <class C>
__device__ __forceinline__ uint32_t finish_pair(const Params& p, int q, const f32x16 (&s)[C::NKB], float k0,
                                                float& acc) {
  const int e = 2 * q;
  float x0 = s[e / 16][e % 16], x1 = s[(e + 1) / 16][(e + 1) % 16];
  if constexpr (C::NORM == NORM_SOFTMAX) {
    x0 = fast_exp2(__builtin_fmaf(x0, p.c, k0));
    x1 = fast_exp2(__builtin_fmaf(x1, p.c, k0));
  } else if constexpr (C::NORM == NORM_SIGMOID) {
    x0 = fast_rcp(1.f + x0);
    x1 = fast_rcp(1.f + x1);
  } else if constexpr (C::NORM == NORM_ABSSUM) {
    acc += fabsf(x0) + fabsf(x1);
  }
  bf16x2 pr;
  pr[0] = (__bf16)x0;
  pr[1] = (__bf16)x1;
  if constexpr (C::NORM == NORM_SOFTMAX || C::NORM == NORM_ABS_OF_SUM) {
    // row sum over the rounded weights, two per v_dot2c_f32_bf16
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    acc = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, acc, false);
  }
  return __builtin_bit_cast(uint32_t, pr);
}

// koff[t]: this lane's byte offset, inside a K tile, of its 16-byte piece of
// contraction step t for key row (lane % 32) -- swizzle included.
template <class C>
__device__ __forceinline__ void k_frag_offsets(int (&koff)[C::DQK / 16]) {
  const int lane = threadIdx.x & 63;
  const int ql = lane & 31, half = lane >> 5;
#pragma unroll
  for (int t = 0; t < C::DQK / 16; ++t) koff[t] = ql * C::RB_K + (((2 * t + half) ^ kswz<C::CPR_K>(ql)) * 16);
}

// Transposing LDS read: within each 16-lane block, lane i supplies the address
// of row (i/4), columns 4*(i%4)..+3 and receives column i of the 4 rows.
// Blocks 0/1 of the wave cover d 0..15 / 16..31 for key half 0, blocks 2/3 the
// same for key half 1.  voff[db]: this lane's byte offset inside a V tile for
// the 32-wide block db of output columns, key rows 4*half + (i/4) -- swizzle
// included (the swizzle only depends on the row modulo 4, a per-lane constant).
template <class C>
__device__ __forceinline__ void v_frag_offsets(int (&voff)[C::DV / 32]) {
  const int lane = threadIdx.x & 63;
  const int half = lane >> 5, li = lane & 15;
  const int row = 4 * half + (li >> 2);
  const int cl = 2 * ((lane >> 4) & 1) + ((li & 3) >> 1);  // chunk within the 64-byte group
#pragma unroll
  for (int db = 0; db < C::DV / 32; ++db)
    voff[db] = row * C::RB_V + ((4 * (db ^ vswz<C::CPR_V>(row)) + cl) * 16) + (li & 1) * 8;
}

__device__ __forceinline__ bf16x8 read_v_frag(const char* a0, int row8_bytes) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(a0 + row8_bytes));
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

#ifndef AE_FRAG_AHEAD
#define AE_FRAG_AHEAD 4
#endif
constexpr int kFragAhead = AE_FRAG_AHEAD;  // LDS fragment reads kept in flight ahead of their MFMA

// ---- phase A: S_nxt = K_tile Q^T  ||  weights of the previous tile --------------
//   DO_QK   score the tile at `ksm` into s_nxt (relevance scoring)
//   DO_FIN  turn s_cur into the packed weights pf (second half of the row norm)
// Every K fragment read from LDS feeds the MFMAs of all QB query blocks.
template <class C, bool DO_QK, bool DO_FIN>
__device__ __forceinline__ void phase_a(const Params& p, const char* ksm, const int (&koff)[C::DQK / 16],
                                        const bf16x8 (&qf)[C::QB][C::DQK / 16], f32x16 (&s_nxt)[C::QB][C::NKB],
                                        const f32x16 (&s_cur)[C::QB][C::NKB], RowState<C> (&st)[C::QB],
                                        bf16x8 (&pf)[C::QB][2 * C::NKB]) {
  constexpr int QB = C::QB, T = C::DQK / 16;
  constexpr int NF = DO_QK ? C::NKB * T : 0;            // fragments
  constexpr int NM = NF * QB;                           // MFMAs
  constexpr int NPAIR = DO_FIN ? 8 * C::NKB * QB : 0;   // vector work items
  // Pairs done before the first MFMA: they cover the latency of the first
  // fragment reads, which cannot be issued before the tile is published.
  constexpr int FRONT = !DO_QK ? NPAIR : (NPAIR * 4 > NM * 3 ? NPAIR / 4 : 0);
  constexpr int PF = kFragAhead < NF ? kFragAhead : NF;

  bf16x8 ring[PF > 0 ? PF : 1];
#pragma unroll
  for (int g = 0; g < PF; ++g)
    ring[g] = *reinterpret_cast<const bf16x8*>(ksm + (g / T) * 32 * C::RB_K + koff[g % T]);

  float k0[QB], acc[QB];
  u32x4 pk[QB][DO_FIN ? 2 * C::NKB : 1];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    acc[qb] = 0.f;
    k0[qb] = 0.f;
    if constexpr (DO_FIN && C::NORM == NORM_SOFTMAX) k0[qb] = p.b2 - ((st[qb].m == -INFINITY) ? 0.f : st[qb].m);
  }
  auto do_pair = [&](int pi) {
    const int qb = pi / (8 * C::NKB), q = pi % (8 * C::NKB);
    pk[qb][q / 4][q % 4] = finish_pair<C>(p, q, s_cur[qb], k0[qb], acc[qb]);
  };
#pragma unroll
  for (int pi = 0; pi < FRONT; ++pi) do_pair(pi);
  sched_fence();

#pragma unroll
  for (int mi = 0; mi < NM; ++mi) {
    const int g = mi / QB, qb = mi % QB;
    const int kb = g / T, t = g % T;
    if (t == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s_nxt[qb][kb][r] = 0.f;
    }
    s_nxt[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[g % PF], qf[qb][t], s_nxt[qb][kb], 0, 0, 0);
    if (qb == QB - 1 && g + PF < NF)  // refill the slot just consumed
      ring[g % PF] = *reinterpret_cast<const bf16x8*>(ksm + ((g + PF) / T) * 32 * C::RB_K + koff[(g + PF) % T]);
#pragma unroll
    for (int pi = FRONT; pi < NPAIR; ++pi)
      if ((pi - FRONT) * NM / (NPAIR - FRONT) == mi) do_pair(pi);
    sched_fence();
  }
  if constexpr (DO_FIN) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
      for (int t = 0; t < 2 * C::NKB; ++t) pf[qb][t] = __builtin_bit_cast(bf16x8, pk[qb][t]);
      if constexpr (C::NORM != NORM_SIGMOID && C::NORM != NORM_NONE) st[qb].l += acc[qb];
    }
  }
}

// ---- phase B: O^T += V_tile^T P^T  ||  modification / row max of the next tile --
//   DO_PV    aggregate the tile at `vsm` with the weights pf
//   DO_POST  mask / modify / reduce the freshly scored s_nxt (tile starting at j0)
// Every V fragment read from LDS feeds the MFMAs of all QB query blocks.
template <class C, bool DO_PV, bool DO_POST, bool MASKED>
__device__ __forceinline__ void phase_b(const Params& p, const char* vsm, const int (&voff)[C::DV / 32],
                                        const bf16x8 (&pf)[C::QB][2 * C::NKB], RowState<C> (&st)[C::QB],
                                        f32x16 (&s_nxt)[C::QB][C::NKB], int i0, int j0, int off, float g2,
                                        bool (&moved)[C::QB], float (&xm)[C::QB]) {
  constexpr int QB = C::QB, DB = C::DV / 32;
  constexpr int NF = DO_PV ? DB * 2 * C::NKB : 0;
  constexpr int NM = NF * QB;
  constexpr int NPAIR = DO_POST ? 8 * C::NKB * QB : 0;
  constexpr int FRONT = !DO_PV ? NPAIR : (NPAIR * 4 > NM * 3 ? NPAIR / 4 : 0);
  constexpr int PF = kFragAhead < NF ? kFragAhead : NF;

  bf16x8 ring[PF > 0 ? PF : 1];
#pragma unroll
  for (int g = 0; g < PF; ++g) ring[g] = read_v_frag(vsm + 16 * (g / DB) * C::RB_V + voff[g % DB], 8 * C::RB_V);

  TileCtx tc[QB];
  float mx[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    mx[qb] = -INFINITY;
    if constexpr (DO_POST) tc[qb] = tile_ctx<C, MASKED>(p, i0 + 32 * qb, j0, off, g2);
  }
  auto do_pair = [&](int pi) {
    const int qb = pi / (8 * C::NKB), q = pi % (8 * C::NKB);
    post_pair<C, MASKED>(p, q, s_nxt[qb], tc[qb], g2, mx[qb]);
  };
#pragma unroll
  for (int pi = 0; pi < FRONT; ++pi) do_pair(pi);
  sched_fence();

#pragma unroll
  for (int mi = 0; mi < NM; ++mi) {
    const int g = mi / QB, qb = mi % QB;
    const int t = g / DB, db = g % DB;  // key-step major: weights pf[.][t] are consumed in order
    st[qb].o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[g % PF], pf[qb][t], st[qb].o[db], 0, 0, 0);
    if (qb == QB - 1 && g + PF < NF)  // refill the slot just consumed
      ring[g % PF] = read_v_frag(vsm + 16 * ((g + PF) / DB) * C::RB_V + voff[(g + PF) % DB], 8 * C::RB_V);
#pragma unroll
    for (int pi = FRONT; pi < NPAIR; ++pi)
      if ((pi - FRONT) * NM / (NPAIR - FRONT) == mi) do_pair(pi);
    sched_fence();
  }
  if constexpr (DO_POST) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) post_done<C>(p, st[qb], mx[qb], moved[qb], xm[qb]);
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
  int slot = w >> 3;
  int group = (slot / per_group) * 8 + (w & 7);
  int t = slot % per_group;
  if (p.map_mode == 1) {
    group = w / per_group;
    t = w % per_group;
  } else if (p.map_mode >= 2) {
    const int I = p.map_mode;
    const int blk = slot / (I * per_group), r = slot % (I * per_group);
    group = (blk * I + (r % I)) * 8 + (w & 7);
    t = r / I;
  }
  if (group >= p.n_groups) return;
  const int b = group / p.H_kv, hkv = group % p.H_kv;
  const int hq = hkv * p.g + (t % p.g);
  const int qt_lin = t / p.g;
  const int qtile = C::CAUSAL ? (p.n_qtiles - 1 - qt_lin) : qt_lin;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: keeps per-wave branches uniform
  const int ql = lane & 31, half = lane >> 5;
  const int off = p.L_k - p.L_q;
  const int i_wg = qtile * C::BLOCK_M;
  const int iw0 = i_wg + wave * 32 * C::QB;
  const int i0 = iw0 + ql;  // this lane's query row in q-block 0; q-block qb adds 32*qb

  const __bf16* qbase = p.Q + b * p.qs[0] + hq * p.qs[1];
  const __bf16* kbase = p.K + b * p.ks[0] + hkv * p.ks[1];
  const __bf16* vbase = p.V + b * p.vs[0] + hkv * p.vs[1];
  float* obase = p.O + b * p.os[0] + hq * p.os[1];

  // ---- Q fragments (B operand of S^T = K Q^T), resident for the whole kernel -
  bf16x8 qf[C::QB][C::DQK / 16];
  RowState<C> st[C::QB];
#pragma unroll
  for (int qb = 0; qb < C::QB; ++qb) {
    const int i = i0 + 32 * qb;
#pragma unroll
    for (int tt = 0; tt < C::DQK / 16; ++tt) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (i < p.L_q) v = *reinterpret_cast<const u32x4*>(qbase + (int64_t)i * p.qs[2] + tt * 16 + half * 8);
      if (p.neg_q) v ^= (u32x4){0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
      qf[qb][tt] = __builtin_bit_cast(bf16x8, v);
    }
    st[qb].m = -INFINITY;
    st[qb].l = 0.f;
#pragma unroll
    for (int db = 0; db < C::DV / 32; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) st[qb].o[db][r] = 0.f;
  }

  float g2 = 0.f;
  if constexpr (C::MOD == MOD_DECAY) g2 = dt.log2_gamma[hq];

  // key tiles the workgroup walks, and the prefix of them this wave can see
  int kmax = p.L_k, kmax_w = p.L_k;
  if (C::CAUSAL) {
    kmax = max(0, min(p.L_k, i_wg + C::BLOCK_M + off));
    kmax_w = max(0, min(p.L_k, iw0 + 32 * C::QB + off));
  }
  const int n_tiles = (kmax + C::BLOCK_N - 1) / C::BLOCK_N;
  const int n_vis = (kmax_w + C::BLOCK_N - 1) / C::BLOCK_N;
  // wave-uniform: does tile jt cross the causal diagonal or the end of the keys?
  auto needs_mask = [&](int jt) {
    const int j0 = jt * C::BLOCK_N;
    return (j0 + C::BLOCK_N > p.L_k) || (C::CAUSAL && (j0 + C::BLOCK_N - 1 > iw0 + off));
  };

  // LDS: STAGES K buffers, then STAGES V buffers; tile j lives in buffer j % STAGES.
  constexpr int S = C::STAGES, P = C::AHEAD;
  char* const ksm0 = smem;
  char* const vsm0 = smem + S * C::K_BYTES;
  // LDS byte address of the first buffer, as the copy engine wants it (M0)
  const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) char*)smem);
  int koff[C::DQK / 16], voff[C::DV / 32];
  k_frag_offsets<C>(koff);
  v_frag_offsets<C>(voff);
  int kgoff[C::KI], kgrow[C::KI], vgoff[C::VI], vgrow[C::VI];
  dma_offsets<C::WAVES, C::BLOCK_N, C::CPR_K, false>(wave, p.ks[2], kgoff, kgrow);
  dma_offsets<C::WAVES, C::BLOCK_N, C::CPR_V, true>(wave, p.vs[2], vgoff, vgrow);
  // Tile indices past the last tile are clamped: the copy is redundant but keeps
  // the count of loads in flight uniform (see dma_tile).
#ifdef AE_EXP_TILE0
  const int last_tile = 0;
#else
  const int last_tile = max(n_tiles - 1, 0);
#endif
  auto load_k = [&](int jt, int buf) {
    dma_tile<C::WAVES, C::BLOCK_N, C::CPR_K>(kbase, p.ks[2], min(jt, last_tile) * C::BLOCK_N, p.L_k,
                                             lds0 + buf * C::K_BYTES, wave, kgoff, kgrow);
  };
  auto load_v = [&](int jt, int buf) {
    dma_tile<C::WAVES, C::BLOCK_N, C::CPR_V>(vbase, p.vs[2], min(jt, last_tile) * C::BLOCK_N, p.L_k,
                                             lds0 + (S * C::K_BYTES) + buf * C::V_BYTES, wave, vgoff, vgrow);
  };

  // scores of the even / odd tile in flight (PIPE); otherwise only s_a is used
  f32x16 s_a[C::QB][C::NKB], s_b[C::PIPE ? C::QB : 1][C::PIPE ? C::NKB : 1];
  bool moved[C::QB];
  float xm[C::QB];
  auto rescale_all = [&]() {
#pragma unroll
    for (int qb = 0; qb < C::QB; ++qb) lazy_rescale<C>(st[qb], moved[qb], xm[qb]);
  };

  // ---- prologue: start K(0), then the first AHEAD (K, V) pairs; score tile 0 ---
  if (n_tiles > 0) {
    dma_tile<C::WAVES, C::BLOCK_N, C::CPR_K>(kbase, p.ks[2], 0, p.L_k, lds0, wave, kgoff, kgrow);
#pragma unroll
    for (int a = 0; a < P; ++a) {
      load_k(a + 1, (a + 1) % S);
      load_v(a, a % S);
    }
    wait_dma_and_sync<P * C::LOADS_PER_STEP>();  // K(0) has landed everywhere
    if (n_vis > 0) {
      bf16x8 pf[C::QB][2 * C::NKB];
      phase_a<C, true, false>(p, ksm0, koff, qf, s_a, s_a, st, pf);
      if (needs_mask(0))
        phase_b<C, false, true, true>(p, vsm0, voff, pf, st, s_a, i0, 0, off, g2, moved, xm);
      else
        phase_b<C, false, true, false>(p, vsm0, voff, pf, st, s_a, i0, 0, off, g2, moved, xm);
      rescale_all();
    }
    wait_dma_and_sync<(P - 1) * C::LOADS_PER_STEP>();  // K(1) and V(0) have landed
  }

#ifdef AE_PROFILE
  uint64_t prof_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  uint64_t prof_last = __builtin_readcyclecounter();
#endif
  // One pipelined step (SLOT = jt % STAGES).  On entry LDS holds K(jt+1) and
  // V(jt) and s_cur holds S(jt).  K(jt+1+AHEAD) and V(jt+AHEAD) are requested
  // into the buffers of K(jt) and V(jt-1), which nobody reads any more.
  auto step = [&](int jt, auto slot_tag, f32x16 (&s_cur)[C::QB][C::NKB], f32x16 (&s_nxt)[C::QB][C::NKB]) {
    constexpr int SLOT = decltype(slot_tag)::value;
    load_k(jt + 1 + P, SLOT);
    load_v(jt + P, (SLOT + P) % S);
    const char* k_next = ksm0 + ((SLOT + 1) % S) * C::K_BYTES;
    const char* v_cur = vsm0 + SLOT * C::V_BYTES;
    if constexpr (C::PIPE) {
      if (jt + 1 < n_vis) {
        bf16x8 pf[C::QB][2 * C::NKB];
        // phase A: score tile jt+1 while turning tile jt's scores into weights
        phase_a<C, true, true>(p, k_next, koff, qf, s_nxt, s_cur, st, pf);
        // phase B: aggregate tile jt while masking / reducing tile jt+1's scores
        if (needs_mask(jt + 1))
          phase_b<C, true, true, true>(p, v_cur, voff, pf, st, s_nxt, i0, (jt + 1) * C::BLOCK_N, off, g2, moved, xm);
        else
          phase_b<C, true, true, false>(p, v_cur, voff, pf, st, s_nxt, i0, (jt + 1) * C::BLOCK_N, off, g2, moved, xm);
        rescale_all();
      } else if (jt < n_vis) {
        // this wave's last visible tile: nothing further to score
        bf16x8 pf[C::QB][2 * C::NKB];
        phase_a<C, false, true>(p, k_next, koff, qf, s_nxt, s_cur, st, pf);
        phase_b<C, true, false, false>(p, v_cur, voff, pf, st, s_nxt, i0, 0, off, g2, moved, xm);
      }
    } else {
      // one set of score registers: weights and aggregation of tile jt, then the
      // scores of tile jt+1 into the same registers
      AE_TICK(0);
      if (jt < n_vis) {
        bf16x8 pf[C::QB][2 * C::NKB];
        phase_a<C, false, true>(p, k_next, koff, qf, s_cur, s_cur, st, pf);
        AE_TICK(1);
        // The two waves of a SIMD are arbitrated oldest-first: without help the
        // older one wins every cycle, its vector phases delay the younger one's
        // MFMAs and it then idles at the barrier.  Matrix phases therefore run
        // at raised priority, vector phases at the default.
        __builtin_amdgcn_s_setprio(AE_MFMA_PRIO);
        phase_b<C, true, false, false>(p, v_cur, voff, pf, st, s_cur, i0, 0, off, g2, moved, xm);
        AE_TICK(2);
        if (jt + 1 < n_vis) {
          phase_a<C, true, false>(p, k_next, koff, qf, s_cur, s_cur, st, pf);
          __builtin_amdgcn_s_setprio(0);
          AE_TICK(3);
          if (needs_mask(jt + 1))
            phase_b<C, false, true, true>(p, v_cur, voff, pf, st, s_cur, i0, (jt + 1) * C::BLOCK_N, off, g2, moved, xm);
          else
            phase_b<C, false, true, false>(p, v_cur, voff, pf, st, s_cur, i0, (jt + 1) * C::BLOCK_N, off, g2, moved, xm);
          rescale_all();
          AE_TICK(4);
        }
        __builtin_amdgcn_s_setprio(0);
      }
    }
    wait_dma_and_sync<(P - 1) * C::LOADS_PER_STEP>();  // K(jt+2) and V(jt+1) have landed
    AE_TICK(5);
  };

  // ---- main loop, unrolled by STAGES so that buffer choices are compile-time ---
  static_assert(S == 2 || S == 4, "the loop below is written for two or four stages");
  auto step_at = [&](int jt, auto slot_tag) {
    if constexpr (!C::PIPE)
      step(jt, slot_tag, s_a, s_a);
    else if constexpr (decltype(slot_tag)::value % 2 == 0)
      step(jt, slot_tag, s_a, s_b);
    else
      step(jt, slot_tag, s_b, s_a);
  };
  for (int jt = 0; jt < n_tiles; jt += S) {
    step_at(jt, std::integral_constant<int, 0>{});
    if (jt + 1 < n_tiles) step_at(jt + 1, std::integral_constant<int, 1>{});
    if constexpr (S == 4) {
      if (jt + 2 < n_tiles) step_at(jt + 2, std::integral_constant<int, 2>{});
      if (jt + 3 < n_tiles) step_at(jt + 3, std::integral_constant<int, 3>{});
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // redundant tail copies must land before LDS is released

#ifdef AE_PROFILE
  if (p.prof && lane == 0)
    for (int k = 0; k < 8; ++k) p.prof[((size_t)blockIdx.x * C::WAVES + wave) * 8 + k] = prof_acc[k];
#endif
  // ---- online_epilogue + store ------------------------------------------------
#pragma unroll
  for (int qb = 0; qb < C::QB; ++qb) {
    float inv = 1.f;
    if constexpr (C::NORM == NORM_SOFTMAX) {
      const float l = sum_halves(st[qb].l);
      inv = l > 0.f ? 1.f / l : 0.f;
    } else if constexpr (C::NORM == NORM_ABSSUM) {
      inv = 1.f / fmaxf(sum_halves(st[qb].l), 1.f);
    } else if constexpr (C::NORM == NORM_ABS_OF_SUM) {
      inv = 1.f / fmaxf(fabsf(sum_halves(st[qb].l)), 1.f);
    }
    const int i = i0 + 32 * qb;
    if (i < p.L_q) {
      float* orow = obase + (int64_t)i * p.os[2];
#pragma unroll
      for (int db = 0; db < C::DV / 32; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = st[qb].o[db][4 * r4 + e] * inv;
          *reinterpret_cast<f32x4*>(orow + db * 32 + r4 * 8 + half * 4) = v;
        }
    }
  }
}

}  // namespace ae
