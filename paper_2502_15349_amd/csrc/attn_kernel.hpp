// Fused parallel-pattern attention forward kernel for gfx950 (CDNA4).
//
// One workgroup owns BLOCK_M = 32*WAVES query rows of one (batch, q-head); each
// wavefront owns 32 of them and walks the visible keys in sub-tiles of 32 keys,
// two sub-tiles per 64-key LDS tile.  Per sub-tile (paper Section 4.1: parallel
// pattern with the online row-norm interface):
//   relevance scoring   S^T = K_sub Q^T           (bf16 MFMA 32x32x16, fp32 acc)
//   modification        scale / bias / decay / relu / mask, in registers
//   online row-norm     per-row running state (max+sum, or abs-sum), registers
//   aggregation         O^T += V_sub^T P^T        (bf16 MFMA, fp32 acc)
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
// Key loop.  The tiles every wave of the workgroup sees in full (no causal
// diagonal, no ragged end) are walked by a branch-free loop in which the two
// waves of a SIMD alternate between a vector phase and a matrix phase, one
// always a phase behind the other (see Steady below).  The remaining tiles
// (diagonal, ragged tail) go through a general loop with wave-uniform branches
// for "nothing visible" and "needs the mask".
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
  int g;           // H_q / H_kv
  int n_qtiles;    // ceil(L_q / BLOCK_M)
  int n_groups;    // B * H_kv
  int interleave;  // (batch, kv head) groups walked together on one XCD
  int64_t qs[3], ks[3], vs[3], os[3];  // element strides {batch, head, row}
  float c;         // |scale| * log2(e)  (softmax, sigmoid)  or |scale| (others)
  float b2;        // bias * log2(e)     (softmax, sigmoid)  or bias (others)
  int neg_q;       // scale < 0: the sign is moved onto Q (exact for bf16)
};

struct DecayTable {
  float log2_gamma[kMaxDecayHeads];
};

template <int DQK_, int DV_, int NORM_, int MOD_, bool CAUSAL_, int WAVES_>
struct Cfg {
  static constexpr int DQK = DQK_, DV = DV_, NORM = NORM_, MOD = MOD_, WAVES = WAVES_;
  static constexpr bool CAUSAL = CAUSAL_;
  static constexpr int SUB_N = 32;    // keys per compute sub-tile
  static constexpr int BLOCK_N = 64;  // keys per LDS tile (two sub-tiles)
  static constexpr int BLOCK_M = 32 * WAVES;
  static constexpr int THREADS = 64 * WAVES;
  // LDS tiles are row-major and unpadded; CPR = 16-byte chunks per row.
  static constexpr int RB_K = DQK * 2, RB_V = DV * 2;
  static constexpr int CPR_K = DQK / 8, CPR_V = DV / 8;
  static constexpr int K_BYTES = BLOCK_N * RB_K;
  static constexpr int V_BYTES = BLOCK_N * RB_V;
  // While tile j is being worked on, tiles j and j+1 are readable (scoring and
  // the fragment ring run ahead of aggregation) and tile j+2 is arriving.
  static constexpr int STAGES = 3;
  static constexpr int LDS_BYTES = STAGES * (K_BYTES + V_BYTES);
  static constexpr int NB_K = K_BYTES / 1024, NB_V = V_BYTES / 1024;  // 1 KB blocks per tile
  static constexpr int KI = (NB_K + WAVES - 1) / WAVES, VI = (NB_V + WAVES - 1) / WAVES;
  static constexpr int T = DQK / 16;  // contraction steps of the scoring MFMA
  static constexpr int DB = DV / 32;  // 32-wide blocks of output columns
  static constexpr int PF = 4;  // LDS fragment reads kept in flight ahead of their MFMA
  static_assert(WAVES % 2 == 0, "waves pair up per SIMD");
  static_assert(DQK % 16 == 0 && DV % 32 == 0, "head dims must fit the MFMA tile");
  static_assert(K_BYTES % 1024 == 0 && V_BYTES % 1024 == 0, "tiles must be whole 1 KB blocks");
  static_assert(CPR_K == 8 || CPR_K == 16 || CPR_K == 24, "K swizzle is defined for these row sizes");
  static_assert(CPR_V == 8 || CPR_V == 16 || CPR_V == 32, "V swizzle is defined for these row sizes");
  static_assert(LDS_BYTES <= 160 * 1024, "tiles do not fit LDS");
};

// Calls f(std::integral_constant<int, B>) ... f(std::integral_constant<int, E-1>):
// a loop whose index is a compile-time constant inside the body.
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
// max(a, b, c): one v_max3_f32.  The device code is built with NaNs assumed
// absent, otherwise every operand the compiler cannot prove canonical costs an
// extra v_max in IEEE mode.  (Not written as inline asm: the scores come straight
// out of an MFMA, and the wait states between an MFMA and the first read of its
// result are only inserted in front of instructions the compiler knows.)
__device__ __forceinline__ float max3(float a, float b, float c) { return __builtin_fmaxf(__builtin_fmaxf(a, b), c); }

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
// The running softmax reference only moves when a sub-tile's row max exceeds it
// by more than this many powers of two (weights then stay below 2^kLazyLog2).
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
// Byte offsets (from the tile's first row) of the 16-byte chunks this lane
// fetches for each of the wave's 1 KB blocks, and the tile row they sit in;
// loop invariant.  A wave with no block left repeats one (same bytes to the
// same place), so every wave issues the same number of loads per tile.
template <int WAVES, int ROWS, int CPR, bool IS_V, int N>
__device__ __forceinline__ void dma_offsets(int wave, int64_t row_stride, uint32_t (&goff)[N], int (&grow)[N]) {
  constexpr int NB = ROWS * CPR / 64;
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const int p = ((wave + i * WAVES) % NB) * 64 + lane;  // chunk position in the LDS tile
    const int row = p / CPR, pc = p % CPR;
    const int c = IS_V ? (pc ^ (4 * vswz<CPR>(row))) : (pc ^ kswz<CPR>(row));
    grow[i] = row;
    goff[i] = (uint32_t)(row * (int)row_stride + c * 8) * 2u;
  }
}

// One LDS-DMA instruction: 64 lanes x 16 bytes from base + byte_off (per lane)
// to LDS bytes [lds_addr, lds_addr + 1024).
//
// Issued as inline asm on purpose: for the builtin form the compiler tracks the
// LDS write and, unable to tell which buffer an LDS read touches, puts
// s_waitcnt vmcnt(0) in front of the fragment reads -- which serialises every
// step on the full latency of the copies just started.  Here the waits are
// explicit instead (wait_dma_and_sync).
__device__ __forceinline__ void dma16(const void* base_uniform, uint32_t byte_off, uint32_t lds_addr_uniform) {
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
      : "memory", "m0");
}

// Starts the copy of tile rows [j0, j0 + ROWS) into the LDS tile at `lds`.
// FULL: the caller knows all rows exist.  Otherwise rows past the end of the
// sequence re-read the last valid row: their scores are masked, and finite
// values keep 0 * V finite.
template <int WAVES, int ROWS, int CPR, bool FULL, int N>
__device__ __forceinline__ void dma_tile(const __bf16* base, int64_t row_stride, int j0, int L_k, uint32_t lds, int wave,
                                         const uint32_t (&goff)[N], const int (&grow)[N]) {
  constexpr int NB = ROWS * CPR / 64;
  const __bf16* tile = base + (int64_t)j0 * row_stride;  // wave-uniform
  if (FULL || j0 + ROWS <= L_k) {
#pragma unroll
    for (int i = 0; i < N; ++i) dma16(tile, goff[i], lds + ((wave + i * WAVES) % NB) * 1024);
  } else {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const uint32_t back = (uint32_t)max(0, j0 + grow[i] - (L_k - 1)) * (uint32_t)row_stride * 2u;
      dma16(tile, goff[i] - back, lds + ((wave + i * WAVES) % NB) * 1024);
    }
  }
}

// Waits until none of this wave's DMA loads is in flight, then meets the other
// waves: what they waited for is visible too.  A bare s_barrier is enough: the
// LDS reads of a tile have returned before the barrier that precedes the copy
// into its buffer (each was awaited by the MFMA that consumed it, and reads
// still in flight at a barrier belong to tiles that stay resident), so a buffer
// is only overwritten after every wave is done reading it.
__device__ __forceinline__ void wait_dma_and_sync() { asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory"); }

// Workgroup barrier between phases of the steady-state loop.
__device__ __forceinline__ void phase_barrier() { asm volatile("s_barrier" ::: "memory"); }

// The value is computed before this point and not recomputed after it: an
// empty volatile asm keeps the optimiser from sinking the arithmetic of a vector
// phase past the barrier, next to its first use in the following matrix phase.
template <class V>
__device__ __forceinline__ void pin(V& v) {
  asm volatile("" : "+v"(v));
}

// Nothing may be moved across this point by the instruction scheduler.
__device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

// Per-wave running state of the online row normalization.
template <class C>
struct RowState {
  float m;  // softmax: lazy running reference max (log2 domain)
  float l;  // softmax: running sum of weights; abs-sum family: running sum (this lane's keys only)
  f32x16 o[C::DB];
};

// A lane holds 16 scores of one query per sub-tile: register r is key
// j0 + 8*(r/4) + 4*half + (r%4).  Work on them is cut into 8 pairs (registers
// 2q, 2q+1 -> one packed bf16x2 word); pairs 0..3 form the B operand of the
// first aggregation step (keys 0..15 of the sub-tile), pairs 4..7 of the second.
__device__ __forceinline__ constexpr int key_offset(int r) { return 8 * (r / 4) + (r % 4); }

// Per-sub-tile, per-lane constants of the modification.
struct TileCtx {
  int jlim;     // register r is visible  <=>  key_offset(r) <= jlim   (masked sub-tiles only)
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

// ---- modification + first half of the row norm, one pair of a scored sub-tile --
// Afterwards the two registers hold, per norm:
//   softmax  the raw score, -inf where masked (mx accumulates the lane's max)
//   sigmoid  2^-(scale*s + bias) in log2 units, +inf where masked
//   others   the fully modified score x, 0 where masked
template <class C, bool MASKED>
__device__ __forceinline__ void post_pair(const Params& p, int q, f32x16& s, const TileCtx& tc, float g2, float& mx) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int r = 2 * q + u;
    float x = s[r];
    const bool hidden = MASKED && (key_offset(r) > tc.jlim);
    if constexpr (C::NORM == NORM_SOFTMAX) {
      if (hidden) x = -INFINITY;
    } else if constexpr (C::NORM == NORM_SIGMOID) {
      x = fast_exp2(__builtin_fmaf(x, -p.c, -p.b2));
      if (hidden) x = INFINITY;
    } else {
      if constexpr (C::MOD == MOD_DECAY) {
        // gamma^(i + off - j) = 2^(log2(gamma) * (i + off - j))
        x = x * p.c * fast_exp2(__builtin_fmaf(-g2, (float)key_offset(r), tc.dbase));
      } else {
        x = __builtin_fmaf(x, p.c, p.b2);
        if constexpr (C::MOD == MOD_RELU) x = fmaxf(x, 0.f);
      }
      if (hidden) x = 0.f;
    }
    s[r] = x;
  }
  if constexpr (C::NORM == NORM_SOFTMAX) mx = max3(mx, s[2 * q], s[2 * q + 1]);
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
// the running sum and the output accumulators (rare after the first sub-tiles).
template <class C>
__device__ __forceinline__ void lazy_rescale(RowState<C>& st, bool moved, float xm) {
  if constexpr (C::NORM == NORM_SOFTMAX) {
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
      const float m_new = moved ? xm : st.m;
      const float alpha = moved ? fast_exp2(st.m - m_new) : 1.f;
      st.m = m_new;
      st.l *= alpha;
#pragma unroll
      for (int db = 0; db < C::DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
    }
  }
}

// ---- second half of the row norm, one pair: weight -> packed bf16x2 ------------
template <class C>
__device__ __forceinline__ uint32_t finish_pair(const Params& p, int q, const f32x16& s, float k0, float& acc) {
  float x0 = s[2 * q], x1 = s[2 * q + 1];
  if constexpr (C::NORM == NORM_SOFTMAX) {
    x0 = fast_exp2(__builtin_fmaf(x0, p.c, k0));
    x1 = fast_exp2(__builtin_fmaf(x1, p.c, k0));
  } else if constexpr (C::NORM == NORM_SIGMOID) {
    x0 = fast_rcp(1.f + x0);
    x1 = fast_rcp(1.f + x1);
  } else if constexpr (C::NORM == NORM_ABSSUM) {
    acc += fabsf(x0) + fabsf(x1);
  } else if constexpr (C::NORM == NORM_ABS_OF_SUM) {
    acc += x0 + x1;  // signed terms cancel: the normaliser needs the unrounded sum
  }
  bf16x2 pr;
  pr[0] = (__bf16)x0;
  pr[1] = (__bf16)x1;
  if constexpr (C::NORM == NORM_SOFTMAX) {
    // row sum over the rounded weights, two per v_dot2c_f32_bf16
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    acc = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, acc, false);
  }
  return __builtin_bit_cast(uint32_t, pr);
}

// Softmax exponent offset for the current reference maximum.
template <class C>
__device__ __forceinline__ float finish_k0(const Params& p, const RowState<C>& st) {
  if constexpr (C::NORM == NORM_SOFTMAX) return p.b2 - ((st.m == -INFINITY) ? 0.f : st.m);
  return 0.f;
}
template <class C>
__device__ __forceinline__ void finish_done(RowState<C>& st, float acc) {
  if constexpr (C::NORM != NORM_SIGMOID && C::NORM != NORM_NONE) st.l += acc;
}

// kaddr[t]: this lane's LDS byte address, inside the current K buffer, of its
// 16-byte piece of contraction step t for key row (lane % 32) -- swizzle
// included.  Rows 32..63 of the tile are at +32*RB_K (the swizzle repeats).
template <class C>
__device__ __forceinline__ void k_frag_offsets(uint32_t base, uint32_t (&kaddr)[C::T]) {
  const int lane = threadIdx.x & 63;
  const int half = lane >> 5, ql = lane & 31;
#pragma unroll
  for (int t = 0; t < C::T; ++t) kaddr[t] = base + ql * C::RB_K + (((2 * t + half) ^ kswz<C::CPR_K>(ql)) * 16);
}

// Transposing LDS read: within each 16-lane block, lane i supplies the address
// of row (i/4), columns 4*(i%4)..+3 and receives column i of the 4 rows.
// Blocks 0/1 of the wave cover d 0..15 / 16..31 for key half 0, blocks 2/3 the
// same for key half 1.  vaddr[db]: this lane's LDS byte address inside the
// current V buffer for the 32-wide block db of output columns, key rows
// 4*half + (i/4) -- swizzle included (it only depends on the row modulo 4, a
// per-lane constant).
template <class C>
__device__ __forceinline__ void v_frag_offsets(uint32_t base, uint32_t (&vaddr)[C::DB]) {
  const int lane = threadIdx.x & 63;
  const int half = lane >> 5, li = lane & 15;
  const int row = 4 * half + (li >> 2);
  const int cl = 2 * ((lane >> 4) & 1) + ((li & 3) >> 1);  // chunk within the 64-byte group
#pragma unroll
  for (int db = 0; db < C::DB; ++db)
    vaddr[db] = base + row * C::RB_V + ((4 * (db ^ vswz<C::CPR_V>(row)) + cl) * 16) + (li & 1) * 8;
}

typedef __attribute__((address_space(3))) char lds_char;
__device__ __forceinline__ bf16x8 read_k_frag(uint32_t addr) {
  return *reinterpret_cast<__attribute__((address_space(3))) const bf16x8*>((lds_char*)(uintptr_t)addr);
}
__device__ __forceinline__ bf16x8 read_v_frag(uint32_t addr, int row8_bytes) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)addr);
  const s16x4 hi =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)(addr + row8_bytes));
  const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, both);
}

// A operand of the aggregation MFMA for sub-tile `sub` (0/1) of the V tile,
// 16-key step t (0/1) and output-column block db.
template <class C>
__device__ __forceinline__ bf16x8 load_v_frag(const uint32_t (&vaddr)[C::DB], int sub, int t, int db) {
  return read_v_frag(vaddr[db] + (32 * sub + 16 * t) * C::RB_V, 8 * C::RB_V);
}


__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}

// ================================================================================
// General sub-step pieces (prologue, diagonal and ragged tiles): each block of
// MFMAs primes its own fragment ring.
// ================================================================================

// s = K_sub Q^T for the sub-tile whose first row is at LDS offset krow_off of the
// buffer kaddr points into.
template <class C>
__device__ __forceinline__ void score_block(const uint32_t (&kaddr)[C::T], int krow_off, const bf16x8 (&qf)[C::T],
                                            f32x16& s) {
  constexpr int PF = C::PF;
  bf16x8 ring[PF];
#pragma unroll
  for (int g = 0; g < PF; ++g) ring[g] = read_k_frag(kaddr[g] + krow_off);
  sched_fence();
  s = zero16();
#pragma unroll
  for (int g = 0; g < C::T; ++g) {
    s = mfma(ring[g % PF], qf[g], s);
    if (g + PF < C::T) ring[g % PF] = read_k_frag(kaddr[g + PF] + krow_off);
    sched_fence();
  }
}

// O^T += V_sub^T P^T for sub-tile vsub of the V buffer vaddr points into.
template <class C>
__device__ __forceinline__ void aggregate_block(const uint32_t (&vaddr)[C::DB], int vsub, const u32x4 (&pk)[2],
                                                RowState<C>& st) {
  constexpr int PF = C::PF, DB = C::DB, NM = 2 * DB;
  bf16x8 ring[PF];
#pragma unroll
  for (int g = 0; g < PF; ++g) ring[g] = load_v_frag<C>(vaddr, vsub, g / DB, g % DB);
  sched_fence();
#pragma unroll
  for (int g = 0; g < NM; ++g) {
    const int t = g / DB, db = g % DB;
    st.o[db] = mfma(ring[g % PF], __builtin_bit_cast(bf16x8, pk[t]), st.o[db]);
    if (g + PF < NM) ring[g % PF] = load_v_frag<C>(vaddr, vsub, (g + PF) / DB, (g + PF) % DB);
    sched_fence();
  }
}

// Modified scores of a sub-tile -> packed weights, row sum folded into the state.
template <class C>
__device__ __forceinline__ void weights_all(const Params& p, const f32x16& s, RowState<C>& st, u32x4 (&pk)[2]) {
  const float k0 = finish_k0<C>(p, st);
  float acc = 0.f;
#pragma unroll
  for (int q = 0; q < 8; ++q) pk[q / 4][q % 4] = finish_pair<C>(p, q, s, k0, acc);
  finish_done<C>(st, acc);
}

// Modification (+ mask) and row max of the freshly scored sub-tile starting at key j0.
template <class C, bool MASKED>
__device__ __forceinline__ void modify_all(const Params& p, f32x16& s, RowState<C>& st, int i, int j0, int off, float g2) {
  const TileCtx tc = tile_ctx<C, MASKED>(p, i, j0, off, g2);
  float mx = -INFINITY, xm = 0.f;
  bool moved = false;
#pragma unroll
  for (int q = 0; q < 8; ++q) post_pair<C, MASKED>(p, q, s, tc, g2, mx);
  post_done<C>(p, st, mx, moved, xm);
  lazy_rescale<C>(st, moved, xm);
}

// ================================================================================
// Steady-state iteration: one 64-key tile = two sub-steps, branch free.
// ================================================================================
//
// A sub-step is a vector phase (modification and row max of the scores at hand,
// weights, row sum) followed by a matrix phase (aggregation of that sub-tile,
// scoring of the next one), each closed by a workgroup barrier.  The upper half
// of the waves -- the second wave of every SIMD -- runs exactly one phase behind
// the lower half (it passes one extra barrier on entry, the lower half one on
// exit).  So at any time each SIMD has one wave in its vector phase and one in
// its matrix phase: vector instructions and MFMAs of two waves that run the same
// phase at the same time would simply queue behind each other.
//
// The MFMAs of an iteration are numbered 0 .. N-1 in issue order; numbers >= N
// wrap into the next iteration.  Their A operands pass through one small ring of
// registers that is kept full across phases and iterations: the LDS read for
// MFMA n + PF is issued right behind MFMA n, so no matrix phase starts by
// waiting for LDS.
template <class C>
struct Sched {
  static constexpr int T = C::T, DB = C::DB, NPV = 2 * C::DB, NS = NPV + T, N = 2 * NS, PF = C::PF;
  static_assert(T >= PF && NPV >= PF, "the ring must not span more than two blocks of MFMAs");
  static constexpr bool is_score(int r) { return r >= NPV; }  // position r inside a sub-step: aggregate, then score
  // first MFMA that reads the NEXT K buffer (sub-step 1 scores rows 0..31 of it)
  static constexpr int kFirstNextK = NS + NPV;
};

template <class C>
struct Steady {
  using S = Sched<C>;
  const Params& p;
  const bf16x8 (&qf)[C::T];
  RowState<C>& st;
  u32x4 (&pk)[2];
  bf16x8 (&ring)[S::PF];
  uint32_t (&kaddr)[C::T];
  uint32_t (&vaddr)[C::DB];
  uint32_t dk, dv;  // byte distance to the next K / V buffer of the ring of LDS stages
  int i, off;
  float g2;

  // Issues the LDS read that feeds MFMA n.  Reads are issued in MFMA order, so
  // the fragment addresses are advanced to the next buffer exactly where the
  // first read of that buffer is due.
  template <int n>
  __device__ __forceinline__ void fetch() {
    constexpr int m = n % S::N, sub = m / S::NS, r = m % S::NS;
    if constexpr (n == S::kFirstNextK) {
#pragma unroll
      for (int t = 0; t < C::T; ++t) kaddr[t] += dk;
    }
    if constexpr (n == S::N) {  // the wrapped reads are V fragments of the next tile
#pragma unroll
      for (int db = 0; db < C::DB; ++db) vaddr[db] += dv;
    }
    if constexpr (S::is_score(r))
      ring[n % S::PF] = read_k_frag(kaddr[r - S::NPV] + (sub == 0 ? 32 * C::RB_K : 0));
    else
      ring[n % S::PF] = load_v_frag<C>(vaddr, sub, r / C::DB, r % C::DB);
  }

  // Vector phase of sub-step SUB: the scores in s (sub-tile starting at key j0,
  // every key visible) become packed weights in pk; the row state follows.
  template <int SUB>
  __device__ __forceinline__ void vector_phase(f32x16& s, int j0) {
    const TileCtx tc = tile_ctx<C, false>(p, i, j0, off, g2);
    float mx = -INFINITY, xm = 0.f, acc = 0.f;
    bool moved = false;
#pragma unroll
    for (int q = 0; q < 8; ++q) post_pair<C, false>(p, q, s, tc, g2, mx);
    post_done<C>(p, st, mx, moved, xm);
    lazy_rescale<C>(st, moved, xm);
    const float k0 = finish_k0<C>(p, st);
#pragma unroll
    for (int q = 0; q < 8; ++q) pk[q / 4][q % 4] = finish_pair<C>(p, q, s, k0, acc);
    finish_done<C>(st, acc);
    pin(pk[0]);
    pin(pk[1]);
    sched_fence();
  }

  // Matrix phase of sub-step SUB (0/1): O += V_sub^T P^T with the weights in pk,
  // then s = scores of the next sub-tile.
  // `aside` is called once, behind the second MFMA (a slot for a few independent instructions).
  template <int SUB, class F>
  __device__ __forceinline__ void matrix_phase(f32x16& s, F&& aside) {
    static_for<0, S::NS>([&](auto rc) {
      constexpr int r = decltype(rc)::value, n = SUB * S::NS + r;
      if constexpr (S::is_score(r)) {
        constexpr int g = r - S::NPV;
        if constexpr (g == 0) s = zero16();
        s = mfma(ring[n % S::PF], qf[g], s);
      } else {
        constexpr int t = r / C::DB, db = r % C::DB;
        st.o[db] = mfma(ring[n % S::PF], __builtin_bit_cast(bf16x8, pk[t]), st.o[db]);
      }
      fetch<n + S::PF>();
      if constexpr (r == 1) aside();
      sched_fence();
    });
  }
};

template <class C>
__global__ __launch_bounds__(C::THREADS) void attn_fwd_kernel(const Params p, const DecayTable dt) {
  __shared__ __attribute__((aligned(1024))) char smem[C::LDS_BYTES];

  // ---- workgroup -> (batch, kv head, q head, q tile) ------------------------
  // Workgroups are handed to the 8 XCDs round-robin by id.  All q tiles and all
  // q heads of one (batch, kv head) group are mapped to ONE XCD so that the
  // group's K/V is served by that XCD's L2.  Several groups are walked together
  // (interleaved slot by slot): workgroups of one group stream the same K/V
  // tiles at the same time, and with a single group per XCD all 32 CUs would
  // queue on the few L2 channels that hold the current tile.  Within a group the
  // causal tiles with the most key tiles are issued first.
  const int w = blockIdx.x;
  const int per_group = p.n_qtiles * p.g;
  const int I = p.interleave;
  const int slot = w >> 3;
  const int blk = slot / (I * per_group), r_in = slot % (I * per_group);
  const int group = (blk * I + (r_in % I)) * 8 + (w & 7);
  if (group >= p.n_groups) return;
  const int t_in = r_in / I;
  const int b = group / p.H_kv, hkv = group % p.H_kv;
  const int hq = hkv * p.g + (t_in % p.g);
  const int qt_lin = t_in / p.g;
  const int qtile = C::CAUSAL ? (p.n_qtiles - 1 - qt_lin) : qt_lin;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // scalar: keeps per-wave branches uniform
  const int ql = lane & 31, half = lane >> 5;
  const int off = p.L_k - p.L_q;
  const int i_wg = qtile * C::BLOCK_M;
  const int iw0 = i_wg + wave * 32;
  const int i = iw0 + ql;  // this lane's query row

  const __bf16* qbase = p.Q + b * p.qs[0] + hq * p.qs[1];
  const __bf16* kbase = p.K + b * p.ks[0] + hkv * p.ks[1];
  const __bf16* vbase = p.V + b * p.vs[0] + hkv * p.vs[1];
  float* obase = p.O + b * p.os[0] + hq * p.os[1];

  // ---- Q fragments (B operand of S^T = K Q^T), resident for the whole kernel -
  bf16x8 qf[C::T];
#pragma unroll
  for (int tt = 0; tt < C::T; ++tt) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (i < p.L_q) v = *reinterpret_cast<const u32x4*>(qbase + (int64_t)i * p.qs[2] + tt * 16 + half * 8);
    if (p.neg_q) v ^= (u32x4){0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
    qf[tt] = __builtin_bit_cast(bf16x8, v);
  }
  RowState<C> st;
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int db = 0; db < C::DB; ++db) st.o[db] = zero16();

  float g2 = 0.f;
  if constexpr (C::MOD == MOD_DECAY) g2 = dt.log2_gamma[hq];

  // keys the workgroup walks, and the prefix of them this wave can see
  int kmax = p.L_k, kmax_w = p.L_k;
  if (C::CAUSAL) {
    kmax = max(0, min(p.L_k, i_wg + C::BLOCK_M + off));
    kmax_w = max(0, min(p.L_k, iw0 + 32 + off));
  }
  const int n_tiles = (kmax + C::BLOCK_N - 1) / C::BLOCK_N;  // LDS tiles (workgroup)
  const int n_vis = (kmax_w + C::SUB_N - 1) / C::SUB_N;      // visible sub-tiles (wave)
  // Tiles [0, n_steady) take the branch-free loop.  Iteration jt scores sub-tiles
  // up to 2*jt + 2, which the workgroup's first query row must see in full, and
  // starts the copy of tile jt + 2, which must be a whole tile.
  int n_steady;
  {
    const int lim = C::CAUSAL ? min(p.L_k - 1, i_wg + off) : p.L_k - 1;  // last key visible to every row
    n_steady = lim >= 95 ? (lim - 31) / 64 : 0;
    n_steady = max(0, min(n_steady, p.L_k / 64 - 2));
  }
  // wave-uniform: does sub-tile u cross the causal diagonal or the end of the keys?
  auto needs_mask = [&](int u) {
    const int j0 = u * C::SUB_N;
    return (j0 + C::SUB_N > p.L_k) || (C::CAUSAL && (j0 + C::SUB_N - 1 > iw0 + off));
  };

  // LDS: STAGES K buffers, then STAGES V buffers; tile j lives in buffer j % STAGES.
  const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_char*)smem);
  const uint32_t vlds0 = lds0 + C::STAGES * C::K_BYTES;
  uint32_t kaddr[C::T], vaddr[C::DB];  // fragment addresses inside the K / V buffer in use
  k_frag_offsets<C>(lds0, kaddr);
  v_frag_offsets<C>(vlds0, vaddr);
  uint32_t kgoff[C::KI], vgoff[C::VI];
  int kgrow[C::KI], vgrow[C::VI];
  dma_offsets<C::WAVES, C::BLOCK_N, C::CPR_K, false>(wave, p.ks[2], kgoff, kgrow);
  dma_offsets<C::WAVES, C::BLOCK_N, C::CPR_V, true>(wave, p.vs[2], vgoff, vgrow);
  // Tile indices past the last tile are clamped: the copy is redundant but keeps
  // every wave's stream of loads identical.
  const int last_tile = max(n_tiles - 1, 0);
  auto load_kv = [&](int jt, int buf, auto full) {
    constexpr bool FULL = decltype(full)::value;
    const int j0 = (FULL ? jt : min(jt, last_tile)) * C::BLOCK_N;
    dma_tile<C::WAVES, C::BLOCK_N, C::CPR_K, FULL>(kbase, p.ks[2], j0, p.L_k, lds0 + buf * C::K_BYTES, wave, kgoff, kgrow);
    dma_tile<C::WAVES, C::BLOCK_N, C::CPR_V, FULL>(vbase, p.vs[2], j0, p.L_k, vlds0 + buf * C::V_BYTES, wave, vgoff, vgrow);
  };
  auto next_buf = [](int bidx) { return bidx + 1 == C::STAGES ? 0 : bidx + 1; };

  f32x16 s_a;       // scores of the sub-tile to aggregate next
  u32x4 pk[2];      // packed weights of the sub-tile being aggregated

  // ---- prologue: tiles 0 and 1 -> LDS; score and modify sub-tile 0 ---------------
  if (n_tiles > 0) {
    load_kv(0, 0, std::false_type{});
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    load_kv(1, 1, std::false_type{});
    if (n_vis > 0) {
      score_block<C>(kaddr, 0, qf, s_a);
      if (n_steady == 0) {  // the steady-state loop modifies the scores it is handed itself
        if (needs_mask(0))
          modify_all<C, true>(p, s_a, st, i, 0, off, g2);
        else
          modify_all<C, false>(p, s_a, st, i, 0, off, g2);
      }
    }
    wait_dma_and_sync();
  }

  // On entry to iteration jt LDS holds tiles jt and jt+1; kaddr / vaddr point into
  // the buffers of tile jt (index buf); s_a holds sub-tile 2*jt, modified.
  int buf = 0;
  int jt = 0;

  // ---- steady state ----------------------------------------------------------------
  // Per iteration and wave: vector(2jt) | matrix<0> | vector(2jt+1) | matrix<1>, a
  // barrier after each.  The copy of tile jt+2 goes into the buffer of tile jt-1,
  // which the trailing half of the waves reads until the barrier that ends the
  // leading half's vector(2jt); it is issued in three slices -- in matrix<0>,
  // vector(2jt+1) and matrix<1> -- because the CU's vector memory path takes
  // 64 bytes per clock and an instruction that finds its queue full blocks the
  // wave that issues it.  Each wave awaits its slices at the end of matrix<0> of
  // the next iteration, one barrier before the first wave reads the tile.
  if (n_steady > 0) {
    bf16x8 ring[C::PF];
    Steady<C> sd{p, qf, st, pk, ring, kaddr, vaddr, 0u, 0u, i, off, g2};
    static_for<0, C::PF>([&](auto nc) { sd.template fetch<decltype(nc)::value>(); });
    const bool trailing = wave >= C::WAVES / 2;  // second wave of its SIMD
    // slice PART (0..2) of the copy of the whole tile at (ktile, vtile) into LDS stage `stage`
    constexpr int kSlices = 3;
    auto copy_slice = [&](auto part, const __bf16* ktile, const __bf16* vtile, int stage) {
      constexpr int PART = decltype(part)::value;
      static_for<0, C::KI + C::VI>([&](auto ic) {
        constexpr int n = decltype(ic)::value;
        if constexpr (n % kSlices == PART) {
          if constexpr (n < C::KI)
            dma16(ktile, kgoff[n], lds0 + stage * C::K_BYTES + ((wave + n * C::WAVES) % C::NB_K) * 1024);
          else
            dma16(vtile, vgoff[n - C::KI], vlds0 + stage * C::V_BYTES + ((wave + (n - C::KI) * C::WAVES) % C::NB_V) * 1024);
        }
      });
    };
    constexpr int kSlice0 = (C::KI + C::VI + kSlices - 1) / kSlices;  // instructions in slice 0
    if (trailing) phase_barrier();
    for (; jt < n_steady; ++jt) {
      const int nb = next_buf(buf), stage = next_buf(nb);
      sd.dk = (uint32_t)((nb - buf) * C::K_BYTES);
      sd.dv = (uint32_t)((nb - buf) * C::V_BYTES);
      const __bf16* ktile = kbase + (int64_t)(jt + 2) * C::BLOCK_N * p.ks[2];  // a whole tile (see n_steady)
      const __bf16* vtile = vbase + (int64_t)(jt + 2) * C::BLOCK_N * p.vs[2];
      sd.template vector_phase<0>(s_a, 2 * jt * C::SUB_N);
      phase_barrier();
      sd.template matrix_phase<0>(s_a, [&] { copy_slice(std::integral_constant<int, 0>{}, ktile, vtile, stage); });
      // all but the slice just issued: this wave's share of tile jt+1 has landed
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kSlice0) : "memory");
      phase_barrier();
      copy_slice(std::integral_constant<int, 1>{}, ktile, vtile, stage);
      sd.template vector_phase<1>(s_a, (2 * jt + 1) * C::SUB_N);
      phase_barrier();
      sd.template matrix_phase<1>(s_a, [&] { copy_slice(std::integral_constant<int, 2>{}, ktile, vtile, stage); });
      phase_barrier();
      buf = nb;
    }
    if (!trailing) phase_barrier();  // both halves are at the same point again
    wait_dma_and_sync();             // every wave's share of tile jt+1 has landed
    // s_a: scores of sub-tile 2*jt, which every row of the workgroup sees in full
    modify_all<C, false>(p, s_a, st, i, 2 * jt * C::SUB_N, off, g2);
  }

  // ---- general loop: diagonal and ragged tiles -----------------------------------------
  // Sub-step u: sub-tile u is turned into weights and aggregated (sub-tile vsub of
  // the current V buffer); then sub-tile u+1 is scored from K rows [krow_off, +32)
  // of the buffer kaddr points into, and modified.
  auto sub_step = [&](int u, int krow_off, int vsub) {
    if (u >= n_vis) return;
    weights_all<C>(p, s_a, st, pk);
    sched_fence();
    aggregate_block<C>(vaddr, vsub, pk, st);
    if (u + 1 < n_vis) {
      score_block<C>(kaddr, krow_off, qf, s_a);
      if (needs_mask(u + 1))
        modify_all<C, true>(p, s_a, st, i, (u + 1) * C::SUB_N, off, g2);
      else
        modify_all<C, false>(p, s_a, st, i, (u + 1) * C::SUB_N, off, g2);
    }
  };
  for (; jt < n_tiles; ++jt) {
    const int nb = next_buf(buf);
    load_kv(jt + 2, next_buf(nb), std::false_type{});
    sub_step(2 * jt, 32 * C::RB_K, 0);  // scores rows 32..63 of K(jt)
    {
      const uint32_t dk = (uint32_t)((nb - buf) * C::K_BYTES);
#pragma unroll
      for (int t = 0; t < C::T; ++t) kaddr[t] += dk;
    }
    sub_step(2 * jt + 1, 0, 1);  // scores rows 0..31 of K(jt+1)
    {
      const uint32_t dv = (uint32_t)((nb - buf) * C::V_BYTES);
#pragma unroll
      for (int db = 0; db < C::DB; ++db) vaddr[db] += dv;
    }
    buf = nb;
    wait_dma_and_sync();
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // redundant tail copies must land before LDS is released

  // ---- online_epilogue + store ------------------------------------------------
  float inv = 1.f;
  if constexpr (C::NORM == NORM_SOFTMAX) {
    const float l = sum_halves(st.l);
    inv = l > 0.f ? 1.f / l : 0.f;
  } else if constexpr (C::NORM == NORM_ABSSUM) {
    inv = 1.f / fmaxf(sum_halves(st.l), 1.f);
  } else if constexpr (C::NORM == NORM_ABS_OF_SUM) {
    inv = 1.f / fmaxf(fabsf(sum_halves(st.l)), 1.f);
  }
  if (i < p.L_q) {
    float* orow = obase + (int64_t)i * p.os[2];
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = st.o[db][4 * r4 + e] * inv;
        *reinterpret_cast<f32x4*>(orow + db * 32 + r4 * 8 + half * 4) = v;
      }
  }
}

}  // namespace ae
