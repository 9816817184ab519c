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
// Key loop.  Per sub-tile a wave runs a vector phase (modification, row max,
// weights, row sum) and a matrix phase (aggregation of that sub-tile, scoring of
// the next one); the two waves of a SIMD alternate, one always a phase behind
// the other (see KeyLoop below).  A wave whose rows see no further keys (causal
// diagonal) keeps passing the barriers and skips the work; masking is a small
// wave-uniform branch around the sub-tiles that cross the diagonal, the end of
// the keys or the lower edge of a sliding window.  The iterations in which none
// of that can happen run a short form without those tests (see the kernel).
//
// The query rows (on the way in) and the output rows (on the way out) pass
// through LDS, so that every global memory instruction moves 1 KB of whole
// cache lines although a lane's MFMA fragments are 16-byte pieces of one row.
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
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

enum : int { NORM_SOFTMAX = 0, NORM_SIGMOID = 1, NORM_ABSSUM = 2, NORM_ABS_OF_SUM = 3, NORM_NONE = 4 };
enum : int { MOD_PLAIN = 0, MOD_DECAY = 1, MOD_RELU = 2, MOD_BIAS_T = 3 };  // PLAIN carries a runtime bias (0 for "none"); BIAS_T: an additive bias tensor

constexpr int kMaxDecayHeads = 256;

struct Params {
  const __bf16* Q;
  const __bf16* K;
  const __bf16* V;
  void* O;  // fp32, or bf16 if out_bf16
  float* stats;  // optional [B, H_q, L_q]: final row statistic of the normalization (null: not written)
  const __bf16* bias;  // MOD_BIAS_T: additive bias per (query, key), element strides bs[] = {batch, head, row}
  int64_t bs[3];
  int B, H_q, H_kv, L_q, L_k;
  int g;           // H_q / H_kv
  int n_qtiles;    // ceil(L_q / BLOCK_M)
  int n_groups;    // B * H_kv
  int interleave;  // (batch, kv head) groups walked together on one XCD
  int64_t qs[3], ks[3], vs[3], os[3];  // element strides {batch, head, row}
  float c;         // |scale| * log2(e)  (softmax, sigmoid)  or |scale| (others)
  float b2;        // bias * log2(e)     (softmax, sigmoid)  or bias (others)
  int neg_q;       // scale < 0: the sign is moved onto Q (exact for bf16)
  int out_bf16;    // O holds bf16 instead of fp32
  int window;      // sliding-window kernels: key j is also hidden if j <= i + (L_k - L_q) - window
  // Split keys (n_splits > 1): the launch holds n_splits copies of the base_grid items; copy c
  // walks key tiles [c * split_tiles, (c + 1) * split_tiles) only and writes its normalised
  // partial rows (fp32, [split, B, H_q, L_q, D_v]) and their log-sum-exp ([split, B, H_q, L_q])
  // to the workspace instead of O / stats; attn_merge_kernel combines them.
  int n_splits, split_tiles, base_grid;
  float* ws_o;
  float* ws_lse;
  // Recurrent pattern, chunks as batch entries (MOD_DECAY with NORM_NONE only; null: off): batch entry
  // b >= state_b0 of head h starts from the carried state in front of its chunk, a bf16 matrix [D_v][D_qk] at
  // state + (b - state_b0) * state_bs + h * state_hs:  O[i] = c * gamma^(i+1) * q_i H  +  the walk over the keys.
  const __bf16* state;
  int64_t state_bs, state_hs;
  int state_b0;
};

struct DecayTable {
  float log2_gamma[kMaxDecayHeads];
};

// MASK_: 0 none, 1 causal, 2 causal with a sliding window (Params::window keys per query)
// FOLD_ (softmax and sigmoid without a bias tensor): the exponent comes out of the scoring MFMA ready to use.
// Q is multiplied by |scale| * log2(e) when loaded and rounded to bf16 again (the paper's own form: its
// modification scales q, Section 4.1), and the constant term of the exponent -- minus the running reference
// maximum of the row (softmax), the bias (sigmoid) -- is the INITIAL VALUE of the MFMA accumulator, a register
// set that only changes when the reference moves.  That removes the multiply-add in front of every exponential,
// and for softmax the row maximum as well: the reference only has to move when a weight would overflow, which
// the row sum (needed anyway) shows.  The host picks FOLD where the second rounding of q is harmless
// (|scale| sqrt(D_qk) <= 2: scores of unit-variance inputs with a standard deviation of at most 2).
template <int DQK_, int DV_, int NORM_, int MOD_, int MASK_, int WAVES_, int FOLD_ = 0>
struct Cfg {
  static constexpr int DQK = DQK_, DV = DV_, NORM = NORM_, MOD = MOD_, WAVES = WAVES_;
  static constexpr bool FOLD = FOLD_ != 0;
  static_assert(!FOLD || ((NORM_ == NORM_SOFTMAX || NORM_ == NORM_SIGMOID) && MOD_ == MOD_PLAIN), "FOLD: softmax or sigmoid, no bias tensor");
  static constexpr int MASK = MASK_;
  static constexpr bool CAUSAL = MASK_ != 0, WINDOW = MASK_ == 2;
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
  // At the end the same LDS stages the output: per wave 32 rows x OC columns of fp32.
  static constexpr int OC = DV < 128 ? DV : 128;
  // A stage holds a K tile followed by a V tile.  At the start the query rows pass
  // through the LDS behind stage 0 (32 rows per wave, laid out like a K sub-tile).
  static constexpr int STAGE_BYTES = K_BYTES + V_BYTES, Q_BYTES = WAVES * 32 * RB_K;
  static constexpr int TILE_BYTES = STAGES * STAGE_BYTES, OUT_BYTES = WAVES * 32 * OC * 4;
  static constexpr int cmax(int a, int b) { return a > b ? a : b; }
  // (bias tensor: two buffers of 2 KB per wave behind the stages, see KeyLoop::copy_bias)
  static constexpr int BIAS_BYTES = MOD_ == MOD_BIAS_T ? WAVES * 4096 : 0;
  // D_qk = 256: the query rows of a workgroup (128 KB) do not fit behind stage 0; the fragments are loaded
  // straight from memory there (a slower start of the workgroup, once per 256 rows)
  static constexpr bool kQDirect = STAGE_BYTES + Q_BYTES > 160 * 1024;
  static constexpr int LDS_BYTES = cmax(TILE_BYTES + BIAS_BYTES, cmax(OUT_BYTES, kQDirect ? 0 : STAGE_BYTES + Q_BYTES));
  static constexpr int NB_K = K_BYTES / 1024, NB_V = V_BYTES / 1024;  // 1 KB blocks per tile
  static constexpr int KI = (NB_K + WAVES - 1) / WAVES, VI = (NB_V + WAVES - 1) / WAVES;
  static constexpr int T = DQK / 16;  // contraction steps of the scoring MFMA
  static constexpr int DB = DV / 32;  // 32-wide blocks of output columns
  static constexpr int VA = DB < 4 ? DB : 4;  // V fragment base addresses kept per lane
  // LDS fragment reads kept in flight ahead of their MFMA: a ring of PF register quads.  It must divide the MFMAs of
  // an iteration, 4 (DB + T), and fit either block of a sub-step.  Four cover an LDS latency of 128 clocks at one
  // MFMA per 32; under the load of eight wavefronts and the tile copies the latency is longer, and eight measured
  // 1-3 % faster where the registers are there (128/128 and 192/128; the sliding-window kernels have none to spare).
#ifndef AE_TUNE_PF
#define AE_TUNE_PF 8
#endif
  static constexpr int PF = (4 * (DV / 32 + DQK / 16)) % AE_TUNE_PF == 0 && AE_TUNE_PF <= DQK / 16 && AE_TUNE_PF <= 2 * (DV / 32) &&
                                    DQK + DV <= 320 && MASK_ != 2 && MOD_ != MOD_BIAS_T
                                ? AE_TUNE_PF : 4;
  // A copy instruction that finds the CU's vector memory queue full blocks the wave
  // that issues it, and with it everything behind it in program order.  Where the
  // matrix phase is the longer one the copies are issued in the vector phases (the
  // K tile in the first, the V tile in the second of an iteration), so that the
  // wave issuing MFMAs is never held up; where the vector phase is the longer one
  // (few MFMAs per sub-tile), in three slices spread over matrix and vector phases.
  static constexpr bool kCopyInVector = T + 2 * DB >= 12;
  static_assert(WAVES % 2 == 0, "waves pair up per SIMD");
  static_assert(DQK % 16 == 0 && DV % 32 == 0, "head dims must fit the MFMA tile");
  static_assert(K_BYTES % 1024 == 0 && V_BYTES % 1024 == 0, "tiles must be whole 1 KB blocks");
  static_assert(CPR_K == 8 || CPR_K == 16 || CPR_K == 24 || CPR_K == 32, "K swizzle is defined for these row sizes");
  static_assert(CPR_V == 8 || CPR_V == 16 || CPR_V == 32, "V swizzle is defined for these row sizes");
  static_assert(LDS_BYTES <= 160 * 1024, "tiles do not fit LDS");
  // FOLD sigmoid at 64/64: the scoring accumulator's initial value (the bias, the same in all 16 registers) is built
  // where it is used instead of being held in registers: 138 -> 116 registers, which lets a second workgroup onto
  // the compute unit (C3: 33.8 -> 36.5 % of peak on the same box)
  static constexpr bool kSplatInit = DQK_ == 64 && DV_ == 64;
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
// A tile of ROWS rows x CPR chunks is copied as NB blocks of 1 KB (64 chunks), one
// wave instruction each; wave w copies blocks w, w + WAVES, ...  (a wave with no
// block left repeats one -- same bytes to the same place -- so every wave issues
// the same number of loads per tile).  Per block a lane needs the byte offset of
// its chunk from the tile's first row.  Where the blocks of a wave are a whole
// number of swizzle periods apart, one offset serves them all and the distance
// is added to the wave-uniform base pointer instead.
template <int WAVES, int ROWS, int CPR, bool IS_V>
struct DmaMap {
  static constexpr int NB = ROWS * CPR / 64, N = (NB + WAVES - 1) / WAVES;
  static constexpr int kPeriod = IS_V ? 4 : 16;        // rows after which the swizzle repeats
  static constexpr int kRowStep = WAVES * 64 / CPR;    // rows between two blocks of a wave
  static constexpr bool kShared = NB % WAVES == 0 && (WAVES * 64) % CPR == 0 && kRowStep % kPeriod == 0;
  static constexpr int NOFF = kShared ? 1 : N;

  // tile row of this lane's chunk in block i of the wave
  static __device__ __forceinline__ int row(int wave, int i) {
    return ((((wave + i * WAVES) % NB) * 64) + (int)(threadIdx.x & 63)) / CPR;
  }
  static __device__ __forceinline__ void offsets(int wave, int64_t row_stride, uint32_t (&goff)[NOFF]) {
#pragma unroll
    for (int i = 0; i < NOFF; ++i) {
      const int p = ((wave + i * WAVES) % NB) * 64 + (int)(threadIdx.x & 63);  // chunk position in the LDS tile
      const int r = p / CPR, pc = p % CPR;
      const int c = IS_V ? (pc ^ (4 * vswz<CPR>(r))) : (pc ^ kswz<CPR>(r));
      goff[i] = (uint32_t)(r * (int)row_stride + c * 8) * 2u;
    }
  }
};

// One LDS-DMA instruction: 64 lanes x 16 bytes from base + byte_off (per lane)
// to LDS bytes [lds_addr, lds_addr + 1024).
//
// Issued as inline asm on purpose: for the builtin form the compiler tracks the
// LDS write and, unable to tell which buffer an LDS read touches, puts
// s_waitcnt vmcnt(0) in front of the fragment reads -- which serialises every
// step on the full latency of the copies just started.  Here the waits are
// explicit instead (wait_dma_and_sync).
// (The base pointer is passed through readfirstlane: under scalar register pressure the
// compiler may have moved its arithmetic to the vector unit, and the instruction needs it
// in scalar registers; for a value that already is scalar this is a plain copy.)
__device__ __forceinline__ const void* uniform_ptr(const void* ptr) {
  const uint64_t a = (uint64_t)(uintptr_t)ptr;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  return (const void*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ void dma16(const void* base_uniform, uint32_t byte_off, uint32_t lds_addr_uniform) {
  base_uniform = uniform_ptr(base_uniform);
  lds_addr_uniform = __builtin_amdgcn_readfirstlane(lds_addr_uniform);  // (the same for the LDS address)
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
      : "memory", "m0");
}

// The same with the LDS address given as a wave-uniform base plus a compile-time
// constant, added on the way into M0.
template <int LDS_IMM>
__device__ __forceinline__ void dma16_at(const void* base_uniform, uint32_t byte_off, uint32_t lds_base_uniform) {
  base_uniform = uniform_ptr(base_uniform);
  lds_base_uniform = __builtin_amdgcn_readfirstlane(lds_base_uniform);
  asm volatile(
      "s_add_i32 m0, %0, %3\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_base_uniform), "v"(byte_off), "s"(base_uniform), "n"(LDS_IMM)
      : "memory", "m0", "scc");
}

// Waits until none of this wave's DMA loads is in flight, then meets the other
// waves: what they waited for is visible too.
__device__ __forceinline__ void wait_dma_and_sync() { asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory"); }

// Workgroup barrier between phases of the key loop.  A bare s_barrier is enough:
// the LDS reads of a tile have returned before the barrier that precedes the copy
// into its buffer (each was awaited by the MFMA that consumed it, and reads still
// in flight at a barrier belong to tiles that stay resident), so a buffer is only
// overwritten after every wave is done reading it.
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
  float thr;  // FOLD softmax: the lane's 16-key partial row sum above which the reference must move (-1: no reference yet)
  f32x16 o[C::DB];
};

// A lane holds 16 scores of one query per sub-tile: register r is key
// j0 + 8*(r/4) + 4*half + (r%4).  Work on them is cut into 8 pairs (registers
// 2q, 2q+1 -> one packed bf16x2 word); pairs 0..3 form the B operand of the
// first aggregation step (keys 0..15 of the sub-tile), pairs 4..7 of the second.
__device__ __forceinline__ constexpr int key_offset(int r) { return 8 * (r / 4) + (r % 4); }

// ---- masking ------------------------------------------------------------------------
// Hidden scores (beyond the causal diagonal or the end of the keys) are replaced
// before the modification by the value that makes their weight exactly 0 where
// such a value exists (softmax: -inf; sigmoid: the infinity that the modification
// turns into 2^+inf), otherwise the modified score is zeroed afterwards.
template <class C>
__device__ __forceinline__ void mask_raw(f32x16& s, int jlim, float hidden) {
  if constexpr (C::NORM == NORM_SOFTMAX || C::NORM == NORM_SIGMOID) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (key_offset(r) > jlim) s[r] = hidden;
  }
}
// The same for the lower edge of a sliding window: register r is hidden if key_offset(r) < jlo.
template <class C>
__device__ __forceinline__ void mask_raw_below(f32x16& s, int jlo, float hidden) {
  if constexpr (C::NORM == NORM_SOFTMAX || C::NORM == NORM_SIGMOID) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (key_offset(r) < jlo) s[r] = hidden;
  }
}
template <class C>
__device__ __forceinline__ void mask_modified_below(f32x16& s, int jlo) {
  if constexpr (C::NORM != NORM_SOFTMAX && C::NORM != NORM_SIGMOID) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (key_offset(r) < jlo) s[r] = 0.f;
  }
}
template <class C>
__device__ __forceinline__ void mask_modified(f32x16& s, int jlim) {
  if constexpr (C::NORM != NORM_SOFTMAX && C::NORM != NORM_SIGMOID) {
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (key_offset(r) > jlim) s[r] = 0.f;
  }
}

// ---- modification + first half of the row norm, one pair of a scored sub-tile --
// Afterwards the two registers hold, per norm:
//   softmax  the raw score (mx accumulates the lane's max)
//   sigmoid  2^-(scale*s + bias) in log2 units
//   others   the fully modified score x
template <class C>
__device__ __forceinline__ void post_pair(const Params& p, int q, f32x16& s, float dbase, float g2, float& mx,
                                          uint32_t bias_pair = 0) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int r = 2 * q + u;
    float x = s[r];
    if constexpr (C::MOD == MOD_BIAS_T) {
      // the pair's two bf16 bias values, widened
      const float bv = __builtin_bit_cast(float, u == 0 ? bias_pair << 16 : bias_pair & 0xffff0000u);
      // sigmoid: p.c = scale * log2(e), p.b2 = log2(e).  Softmax keeps the modified score in natural units here
      // (p.c = scale; the row max is taken over it) and moves to powers of two in the exponent's FMA (p.b2 =
      // log2(e)), which saves the multiplication of every bias value.  Others: p.c = scale.
      if constexpr (C::NORM == NORM_SIGMOID) x = fast_exp2(-__builtin_fmaf(x, p.c, bv * p.b2));
      else x = __builtin_fmaf(x, p.c, bv);
    } else if constexpr (C::NORM == NORM_SOFTMAX) {
    } else if constexpr (C::NORM == NORM_SIGMOID) {
      x = fast_exp2(__builtin_fmaf(x, -p.c, -p.b2));
    } else if constexpr (C::MOD == MOD_DECAY) {
      // gamma^(i + off - j) = 2^(log2(gamma) * (i + off - j))
      x = x * p.c * fast_exp2(__builtin_fmaf(-g2, (float)key_offset(r), dbase));
    } else {
      x = __builtin_fmaf(x, p.c, p.b2);
      if constexpr (C::MOD == MOD_RELU) x = fmaxf(x, 0.f);
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
    xm = C::MOD == MOD_BIAS_T ? mx * p.b2 : __builtin_fmaf(mx, p.c, p.b2);  // c > 0
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
  if constexpr (C::NORM == NORM_SOFTMAX && C::MOD == MOD_BIAS_T) {
    x0 = fast_exp2(__builtin_fmaf(x0, p.b2, k0));
    x1 = fast_exp2(__builtin_fmaf(x1, p.b2, k0));
    acc += x0 + x1;
  } else if constexpr (C::NORM == NORM_SOFTMAX) {
    x0 = fast_exp2(__builtin_fmaf(x0, p.c, k0));
    x1 = fast_exp2(__builtin_fmaf(x1, p.c, k0));
    // Row sum in fp32 with plain adds: v_dot2c_f32_bf16 on the packed weights would
    // halve the instruction count but runs on the matrix pipe, in the MFMAs' way.
    acc += x0 + x1;
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
  return __builtin_bit_cast(uint32_t, pr);
}

// Softmax exponent offset for the current reference maximum.
template <class C>
__device__ __forceinline__ float finish_k0(const Params& p, const RowState<C>& st) {
  if constexpr (C::NORM == NORM_SOFTMAX) return (C::MOD == MOD_BIAS_T ? 0.f : p.b2) - ((st.m == -INFINITY) ? 0.f : st.m);
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
// per-lane constant).  The swizzle permutes blocks within groups of 4, so block
// db >= 4 is block db - 4 plus 256 bytes and only VA = min(DB, 4) addresses are kept.
template <class C>
__device__ __forceinline__ void v_frag_offsets(uint32_t base, uint32_t (&vaddr)[C::VA]) {
  const int lane = threadIdx.x & 63;
  const int half = lane >> 5, li = lane & 15;
  const int row = 4 * half + (li >> 2);
  const int cl = 2 * ((lane >> 4) & 1) + ((li & 3) >> 1);  // chunk within the 64-byte group
#pragma unroll
  for (int db = 0; db < C::VA; ++db)
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

__device__ __forceinline__ void lds_write16(uint32_t addr, f32x4 v) {
  *reinterpret_cast<__attribute__((address_space(3))) f32x4*>((lds_char*)(uintptr_t)addr) = v;
}
__device__ __forceinline__ f32x4 lds_read16(uint32_t addr) {
  return *reinterpret_cast<__attribute__((address_space(3))) const f32x4*>((lds_char*)(uintptr_t)addr);
}

// A operand of the aggregation MFMA for sub-tile `sub` (0/1) of the V tile,
// 16-key step t (0/1) and output-column block db.
template <class C>
__device__ __forceinline__ bf16x8 load_v_frag(const uint32_t (&vaddr)[C::VA], int sub, int t, int db) {
  return read_v_frag(vaddr[db % C::VA] + (db / C::VA) * 256 + (32 * sub + 16 * t) * C::RB_V, 8 * C::RB_V);
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

// s = K_sub Q^T for the sub-tile whose first row is at LDS offset krow_off of the
// buffer kaddr points into (prologue: scores of the very first sub-tile).
template <class C>
__device__ __forceinline__ void score_block(const uint32_t (&kaddr)[C::T], int krow_off, const bf16x8 (&qf)[C::T],
                                            f32x16& s, const f32x16& init) {
  constexpr int PF = C::PF;
  bf16x8 ring[PF];
#pragma unroll
  for (int g = 0; g < PF; ++g) ring[g] = read_k_frag(kaddr[g] + krow_off);
  sched_fence();
  s = init;
#pragma unroll
  for (int g = 0; g < C::T; ++g) {
    s = mfma(ring[g % PF], qf[g], s);
    if (g + PF < C::T) ring[g % PF] = read_k_frag(kaddr[g + PF] + krow_off);
    sched_fence();
  }
}

// ================================================================================
// Key loop body: one 64-key tile = two sub-steps.
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
// waiting for LDS.  (A wave only ever skips phases at the end of its key range,
// so the ring never has to be resynchronised.)
template <class C>
struct Sched {
  static constexpr int T = C::T, DB = C::DB, NPV = 2 * C::DB, NS = NPV + T, N = 2 * NS, PF = C::PF;
  static_assert(T >= PF && NPV >= PF, "the ring must not span more than two blocks of MFMAs");
  static_assert(N % PF == 0, "ring slots are assigned by MFMA number modulo PF, across iterations too");
  static constexpr bool is_score(int r) { return r >= NPV; }  // position r inside a sub-step: aggregate, then score
  // first MFMA that reads the NEXT K buffer (sub-step 1 scores rows 0..31 of it)
  static constexpr int kFirstNextK = NS + NPV;
};

template <class C>
struct KeyLoop {
  using S = Sched<C>;
  const Params& p;
  const bf16x8 (&qf)[C::T];
  RowState<C>& st;
  u32x4 (&pk)[2];
  f32x16& cinit;  // FOLD: initial value of the scoring accumulator (see Cfg)
  bf16x8 (&ring)[S::PF];
  uint32_t (&kaddr)[C::T];
  uint32_t (&vaddr)[C::VA];
  uint32_t dk, dv;  // byte distance to the next K / V buffer of the ring of LDS stages
  int i, off;       // this lane's query row; L_k - L_q
  int iw0;          // first query row of the wave
  float g2;         // decay: log2(gamma) of this head
  // Decay, factorised per sub-tile where that cannot overflow (gamma in [1/16, 1]):
  // gamma^(i + off - j) = 2^(g2 * (i + off - j0 - 4*half)) * a8^(r/4) * b[r%4] for
  // register r, with the wave-uniform constants a8 = gamma^-8, b[k] = gamma^-k.
  bool fact;
  float a8, b1, b2, b3;
  // Bias tensor.  A lane needs 16 values of its own query row per sub-tile, but loads shaped like that
  // touch 32 rows per instruction and the CU's memory pipe takes ~60 clk for each.  Instead the wave
  // copies its 32 rows x 32 keys into 2 KB of LDS of its own with two LDS-DMA instructions (16 rows x
  // 64 bytes each, like a K/V copy: no registers, no compiler-tracked load), one vector phase ahead
  // and into one of two buffers, and each lane reads back 4 x 8 bytes of its own row.  LDS slot of
  // the 16-byte chunk c of row r: c ^ ((r >> 2) & 3), applied to the global address when copying
  // (16 lanes read 16 different slots).  Chunks that start beyond the last key are redirected to the
  // row's last chunk (their values belong to hidden keys); rows are padded to 8 elements by contract.
  // The copy is awaited with an exact count: `bias_newer` = the tile-copy instructions issued behind
  // it, which may stay in flight.
  const __bf16* bwave = nullptr;  // bias of this (batch, q head)
  uint32_t bgoff[2] = {0, 0};     // byte offset of row iw0 + 16t + lane/4 (clamped), t = 0, 1
  uint32_t bscr = 0;              // LDS address of the wave's 2 x 2 KB
  int bias_j0 = -1;               // sub-tile whose copy was requested last
  int bias_newer = 0;
  u32x2 bcur[4] = {};             // the sub-tile at hand, per lane

  __device__ __forceinline__ void copy_bias(int j0) const {
    const int lane = threadIdx.x & 63;
    const uint32_t dst = bscr + ((j0 / C::SUB_N) & 1) * 2048;
    const int last = ((p.L_k - 1) >> 3) << 3;  // first key of the row's last chunk
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int r = 16 * t + (lane >> 2);
      int col = j0 + 8 * ((lane & 3) ^ ((r >> 2) & 3));
      col = col < p.L_k ? col : last;
      dma16(bwave, bgoff[t] + 2u * (uint32_t)col, dst + t * 1024);
    }
  }
  static __device__ __forceinline__ void wait_vm(int newer) {
    switch (newer) {
      case 1: asm volatile("s_waitcnt vmcnt(1)" ::: "memory"); break;
      case 2: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
      case 3: asm volatile("s_waitcnt vmcnt(3)" ::: "memory"); break;
      case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
      case 5: asm volatile("s_waitcnt vmcnt(5)" ::: "memory"); break;
      case 6: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
      default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;  // 0, or more than listed: wait for all
    }
  }
  // The sub-tile's bias values to the lanes.  If its copy was not requested ahead (the first sub-tile of
  // a walk, or a wave that sat out the phase before) it is made and fully awaited here.
  __device__ __forceinline__ void take_bias(int j0) {
    if (bias_j0 == j0) {
      wait_vm(bias_newer);
    } else {
      copy_bias(j0);
      wait_vm(0);
    }
    const int lane = threadIdx.x & 63, half = lane >> 5, ql = lane & 31;
    const uint32_t src = bscr + ((j0 / C::SUB_N) & 1) * 2048 + ql * 64 + 8 * half;
#pragma unroll
    for (int a = 0; a < 4; ++a)
      bcur[a] = *reinterpret_cast<__attribute__((address_space(3))) const u32x2*>((lds_char*)(uintptr_t)(src + ((a ^ ((ql >> 2) & 3)) << 4)));
  }
  // Requests the sub-tile after j0 for the next vector phase; `newer`: the tile-copy instructions that
  // this wave issues between here and that phase.
  __device__ __forceinline__ void request_bias(int j0, int newer) {
    if (j0 + C::SUB_N < p.L_k) {
      copy_bias(j0 + C::SUB_N);
      bias_j0 = j0 + C::SUB_N;
      bias_newer = newer;
    }
  }

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
      for (int db = 0; db < C::VA; ++db) vaddr[db] += dv;
    }
    if constexpr (S::is_score(r))
      ring[n % S::PF] = read_k_frag(kaddr[r - S::NPV] + (sub == 0 ? 32 * C::RB_K : 0));
    else
      ring[n % S::PF] = load_v_frag<C>(vaddr, sub, r / C::DB, r % C::DB);
  }

  // FOLD kernels: the scores arrive as exponents (log2 units, constant term included; hidden ones as -inf).
  //
  // Softmax: y = c s - m with m the row's reference.  Weights 2^y, row sum, and that is all -- as long as no
  // weight can overflow, which the lane's partial row sum shows: while it stays below kSumLimit every weight
  // did.  Otherwise (rare: the reference is set from the row's first visible keys, and scores above it by
  // more than 20 powers of two are not what attention inputs look like; or the row has no reference yet) the
  // row maximum is formed after all, the reference moves, sum and output are rescaled and the weights redone.
  // Any reference gives the same result up to rounding: weights, sum and output scale together.
  //
  // Sigmoid: y = log2 of w = e^x.  1 / (1 + 1 / w) = w - w^2 + w^3 - ...: where every w of the sub-tile is
  // at most 1/16 the weight is taken as w - w^2, one multiply-add behind the exponential instead of an
  // addition and a reciprocal (relative error w^2 <= 2^-8, one unit of the bf16 weight's last place, and
  // only at the largest weights); else the exact form.  Under the usual bias of -ln(keys) almost every
  // sub-tile qualifies.
  static constexpr float kSumLimit = 1048576.f;  // 2^20
  static constexpr float kSmallExp = -4.f;
  __device__ __forceinline__ void folded_weights(f32x16& s, float& acc) {
    if constexpr (C::NORM == NORM_SOFTMAX) {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float x0 = fast_exp2(s[2 * q]), x1 = fast_exp2(s[2 * q + 1]);
        acc += x0 + x1;
        bf16x2 pr;
        pr[0] = (__bf16)x0;
        pr[1] = (__bf16)x1;
        pk[q / 4][q % 4] = __builtin_bit_cast(uint32_t, pr);
      }
      if (__builtin_amdgcn_ballot_w64(acc > st.thr) != 0) {
        float mx = -INFINITY;
#pragma unroll
        for (int q = 0; q < 8; ++q) mx = max3(mx, s[2 * q], s[2 * q + 1]);
        mx = max_halves(mx);  // of the exponents, i.e. relative to the current reference (0 where there is none)
        const bool unset = st.m == -INFINITY;
        const bool move = unset ? mx > -INFINITY : mx > kLazyLog2;
        const float d = move ? mx : 0.f;
        if (__builtin_amdgcn_ballot_w64(move && !unset) != 0) {  // rows without a reference have nothing to rescale
          const float alpha = (move && !unset) ? fast_exp2(-d) : 1.f;
          st.l *= alpha;
#pragma unroll
          for (int db = 0; db < C::DB; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) st.o[db][r] *= alpha;
        }
        if (move) st.m = unset ? mx : st.m + mx;
        const bool still_unset = st.m == -INFINITY;
        st.thr = still_unset ? -1.f : kSumLimit;
        const float nm = still_unset ? 0.f : -st.m;
#pragma unroll
        for (int r = 0; r < 16; ++r) cinit[r] = nm;
        acc = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const float x0 = fast_exp2(s[2 * q] - d), x1 = fast_exp2(s[2 * q + 1] - d);
          acc += x0 + x1;
          bf16x2 pr;
          pr[0] = (__bf16)x0;
          pr[1] = (__bf16)x1;
          pk[q / 4][q % 4] = __builtin_bit_cast(uint32_t, pr);
        }
      }
    } else {
      // largest exponent of the lane's 16 (a tree: three levels instead of a chain of eight)
      const float t0 = max3(s[0], s[1], s[2]), t1 = max3(s[3], s[4], s[5]), t2 = max3(s[6], s[7], s[8]);
      const float t3 = max3(s[9], s[10], s[11]), t4 = max3(s[12], s[13], s[14]);
      const float mx = fmaxf(max3(t0, t1, t2), max3(t3, t4, s[15]));
      if (__builtin_amdgcn_ballot_w64(mx > kSmallExp) != 0) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          bf16x2 pr;
          pr[0] = (__bf16)fast_rcp(1.f + fast_exp2(-s[2 * q]));
          pr[1] = (__bf16)fast_rcp(1.f + fast_exp2(-s[2 * q + 1]));
          pk[q / 4][q % 4] = __builtin_bit_cast(uint32_t, pr);
        }
      } else {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const float w0 = fast_exp2(s[2 * q]), w1 = fast_exp2(s[2 * q + 1]);
          bf16x2 pr;
          pr[0] = (__bf16)__builtin_fmaf(-w0, w0, w0);
          pr[1] = (__bf16)__builtin_fmaf(-w1, w1, w1);
          pk[q / 4][q % 4] = __builtin_bit_cast(uint32_t, pr);
        }
      }
    }
  }

  // Vector phase: the raw scores in s (sub-tile u, starting at key j0 = 32u) become
  // packed weights in pk; the row state follows.
  // FAST: the caller knows that no key of the sub-tile is hidden from any row of the wave.
  template <bool FAST>
  __device__ __forceinline__ void vector_phase(f32x16& s, int j0) {
    const int half = (threadIdx.x & 63) >> 5;
    // wave-uniform: does the sub-tile cross the causal diagonal or the end of the keys?
    const bool masked = !FAST && ((j0 + C::SUB_N > p.L_k) || (C::CAUSAL && (j0 + C::SUB_N - 1 > iw0 + off)));
    // register r is visible  <=>  key_offset(r) <= jlim
    const int jlim = min(C::CAUSAL ? i + off : p.L_k - 1, p.L_k - 1) - j0 - 4 * half;
    // sliding window: the sub-tile reaches below the window of the wave's last row; visible <=> key_offset(r) >= jlo
    const bool masked_lo = !FAST && C::WINDOW && (j0 < iw0 + 31 + off - p.window + 1);
    const int jlo = i + off - p.window + 1 - j0 - 4 * half;
    const float dbase = C::MOD == MOD_DECAY ? g2 * (float)(i + off - j0 - 4 * half) : 0.f;
    float mx = -INFINITY, xm = 0.f, acc = 0.f;
    bool moved = false;
    if (masked) mask_raw<C>(s, jlim, -INFINITY);
    if (masked_lo) mask_raw_below<C>(s, jlo, -INFINITY);
    if constexpr (C::FOLD) {
      folded_weights(s, acc);
    } else {
    if (C::MOD == MOD_DECAY && fact) {
      // one exponential per lane and sub-tile instead of one per score
      float ra = p.c * fast_exp2(dbase);
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        s[4 * a + 0] *= ra;
        s[4 * a + 1] *= ra * b1;
        s[4 * a + 2] *= ra * b2;
        s[4 * a + 3] *= ra * b3;
        ra *= a8;
      }
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q) post_pair<C>(p, q, s, dbase, g2, mx, bcur[q / 2][q % 2]);
    }
    if (masked) mask_modified<C>(s, jlim);
    if (masked_lo) mask_modified_below<C>(s, jlo);
    post_done<C>(p, st, mx, moved, xm);
    lazy_rescale<C>(st, moved, xm);
    const float k0 = finish_k0<C>(p, st);
#pragma unroll
    for (int q = 0; q < 8; ++q) pk[q / 4][q % 4] = finish_pair<C>(p, q, s, k0, acc);
    }
    finish_done<C>(st, acc);
    pin(pk[0]);
    pin(pk[1]);
    sched_fence();
  }

  // Matrix phase of sub-step SUB (0/1): O += V_sub^T P^T with the weights in pk,
  // then (if `score`) s = raw scores of the next sub-tile.  `aside` is called once,
  // behind the second MFMA (a slot for a few independent instructions).
  template <int SUB, class F>
  __device__ __forceinline__ void matrix_phase(f32x16& s, bool score, F&& aside) {
    static_for<0, S::NPV>([&](auto rc) {
      constexpr int r = decltype(rc)::value, n = SUB * S::NS + r;
      constexpr int t = r / C::DB, db = r % C::DB;
      st.o[db] = mfma(ring[n % S::PF], __builtin_bit_cast(bf16x8, pk[t]), st.o[db]);
      fetch<n + S::PF>();
      if constexpr (r == 1) aside();
      sched_fence();
    });
    if (score) {
      static_for<S::NPV, S::NS>([&](auto rc) {
        constexpr int r = decltype(rc)::value, n = SUB * S::NS + r, g = r - S::NPV;
        if constexpr (g == 0) {
          if constexpr (C::FOLD && C::kSplatInit) {
            // the constant term (sigmoid: the bias; softmax: minus the row's reference, zero while it has none) as 16
            // moves here, in the matrix phase, whose wave leaves the vector port idle, instead of 16 registers held
            // for the whole kernel (the value is hidden from the optimiser so that it does not hoist the vector back
            // out of the loop)
            float b = C::NORM == NORM_SIGMOID ? p.b2 : (st.m == -INFINITY ? 0.f : -st.m);
            asm volatile("" : "+v"(b));
            f32x16 init;
#pragma unroll
            for (int r = 0; r < 16; ++r) init[r] = b;
            s = mfma(ring[n % S::PF], qf[g], init);
          } else {
            s = mfma(ring[n % S::PF], qf[g], C::FOLD ? cinit : zero16());
          }
        }
        else s = mfma(ring[n % S::PF], qf[g], s);
        fetch<n + S::PF>();
        sched_fence();
      });
      pin(s);
    }
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
  int w = blockIdx.x, split = 0;
  if (p.n_splits > 1) {
    split = w / p.base_grid;
    w -= split * p.base_grid;
  }
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
  // byte address of the head's first output row (O holds 4- or 2-byte elements), its row
  // stride in elements, and the head's row statistics; with split keys the workspace's
  bool o_bf16 = p.out_bf16 != 0;
  int64_t o_row = p.os[2];
  char* obase = static_cast<char*>(p.O) + (b * p.os[0] + hq * p.os[1]) * (o_bf16 ? 2 : 4);
  float* stats = p.stats ? p.stats + ((int64_t)b * p.H_q + hq) * p.L_q : nullptr;
  if (p.n_splits > 1) {
    const int64_t head = ((int64_t)split * p.B + b) * p.H_q + hq;
    o_bf16 = false;
    o_row = C::DV;
    obase = reinterpret_cast<char*>(p.ws_o + head * p.L_q * C::DV);
    stats = p.ws_lse + head * p.L_q;
  }

  RowState<C> st;
  st.m = -INFINITY;
  st.l = 0.f;
  st.thr = -1.f;
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
  if (iw0 >= p.L_q) kmax_w = 0;  // a wave past the last query row only helps with the copies
  int n_tiles = (kmax + C::BLOCK_N - 1) / C::BLOCK_N;  // LDS tiles (workgroup): tiles [jt0, n_tiles) are walked
  int n_vis = (kmax_w + C::SUB_N - 1) / C::SUB_N;      // visible sub-tiles (wave): those below n_vis
  // The walk over the key tiles.  Without a window: tiles 0 .. n_tiles-1 in order.  With a
  // sliding window the workgroup needs tiles jt0 .. n_tiles-1 (jt0: tile of the first key its
  // first row sees) and a wave's own rows start at sub-tile u_first.  The order of the key
  // tiles is free (every reduction here is commutative), and the walk is rotated: first the
  // tiles from jtm on -- no row of the workgroup has its window's lower edge in them, so they
  // are walked exactly like a causal problem that starts at tile jtm -- then tiles jt0 ..
  // jtm-1, which the lower edges pass through, in the general form of the iteration.  This
  // keeps the general form behind the short one in the program, as without a window.
  // A wave with no key of its own in a sub-tile runs the matrix phases with all-zero weights
  // (it would only wait at the barriers otherwise), which keeps its fragment ring, its LDS
  // addresses and its scores in step with the others.
  int jt0 = 0, jtm = 0, u_first = 0;
  if (!C::WINDOW && p.n_splits > 1) {  // this workgroup's share of the key tiles
    jt0 = jtm = split * p.split_tiles;
    n_tiles = min(n_tiles, jt0 + p.split_tiles);
    n_vis = min(n_vis, 2 * n_tiles);
  }
  if (C::WINDOW) {
    jt0 = max(0, i_wg + off - p.window + 1) / C::BLOCK_N;
    jtm = (max(0, i_wg + (C::WAVES - 1) * 32 + off - p.window + 32) + C::BLOCK_N - 1) / C::BLOCK_N;
    jtm = max(jt0, min(jtm, n_tiles));
    u_first = max(0, iw0 + off - p.window + 1) / C::SUB_N;
  }
  const int n_walk = max(n_tiles - jt0, 0), n_lead = n_tiles - jtm;  // positions in the walk; those before the rotation
  auto tile_at = [&](int pos) { return C::WINDOW ? (pos < n_lead ? jtm + pos : jt0 + (pos - n_lead)) : jt0 + pos; };
  // LDS: STAGES stages of a K buffer and a V buffer; tile j lives in stage j % STAGES.
  const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_char*)smem);
  const uint32_t vlds0 = lds0 + C::K_BYTES;
  uint32_t kaddr[C::T], vaddr[C::VA];  // fragment addresses inside the K / V buffer in use
  k_frag_offsets<C>(lds0, kaddr);
  v_frag_offsets<C>(vlds0, vaddr);
  using KMap = DmaMap<C::WAVES, C::BLOCK_N, C::CPR_K, false>;
  using VMap = DmaMap<C::WAVES, C::BLOCK_N, C::CPR_V, true>;
  static_assert(KMap::N == C::KI && VMap::N == C::VI, "copy instruction counts");
  uint32_t kgoff[KMap::NOFF], vgoff[VMap::NOFF];
  KMap::offsets(wave, p.ks[2], kgoff);
  VMap::offsets(wave, p.vs[2], vgoff);
  // A tile index past the last tile is clamped (only the prologue's copy of tile 1
  // of a one-tile walk asks for one).
  const int last_tile = max(n_tiles - 1, 0);
  constexpr int kCopies = C::KI + C::VI;  // copy instructions per wave and tile
  // Copy instructions n of tile jt with n % NSL == PART into LDS stage `stage`
  // (NSL = 1: the whole tile).
  auto copy_slice = [&](auto nsl, auto part, int jt, int stage) {
    constexpr int NSL = decltype(nsl)::value, PART = decltype(part)::value;
    const int j0 = min(jt, last_tile) * C::BLOCK_N;
    const __bf16* ktile = kbase + (int64_t)j0 * p.ks[2];  // wave-uniform
    const __bf16* vtile = vbase + (int64_t)j0 * p.vs[2];
    const bool whole = j0 + C::BLOCK_N <= p.L_k;
    static_for<0, kCopies>([&](auto ic) {
      constexpr int n = decltype(ic)::value;
      if constexpr (NSL > 0 ? n % (NSL > 0 ? NSL : 1) == PART : ((n < C::KI) == (PART == 0))) {
        constexpr bool isk = n < C::KI;
        constexpr int m = isk ? n : n - C::KI, NB = isk ? C::NB_K : C::NB_V;
        const uint32_t dst = (isk ? lds0 : vlds0) + stage * C::STAGE_BYTES + ((wave + m * C::WAVES) % NB) * 1024;
        using Map = std::conditional_t<isk, KMap, VMap>;
        const int64_t pitch = isk ? p.ks[2] : p.vs[2];  // elements per row
        const __bf16* tile = isk ? ktile : vtile;
        uint32_t goff;
        if constexpr (isk) goff = kgoff[Map::kShared ? 0 : m];
        else goff = vgoff[Map::kShared ? 0 : m];
        if (whole) {
          if constexpr (Map::kShared) tile += (int64_t)(m * Map::kRowStep) * pitch;  // wave-uniform
        } else {
          // Rows past the end of the sequence re-read the last valid row: their
          // scores are masked, and finite values keep 0 * V finite.  The lane
          // offset is an unsigned 32-bit quantity added to the base pointer: the
          // base stays at the tile's first row so that stepping back never wraps.
          if constexpr (Map::kShared) goff += (uint32_t)(m * Map::kRowStep) * (uint32_t)pitch * 2u;
          goff -= (uint32_t)max(0, j0 + Map::row(wave, m) - (p.L_k - 1)) * (uint32_t)pitch * 2u;
        }
        dma16(tile, goff, dst);
      }
    });
  };
  using One = std::integral_constant<int, 1>;
  using Zero = std::integral_constant<int, 0>;
  auto next_buf = [](int bidx) { return bidx + 1 == C::STAGES ? 0 : bidx + 1; };

  // The same copy for a tile known to lie wholly inside the sequence, with the
  // tile's first rows and the LDS stage's bases (this wave's first block) kept in
  // running wave-uniform variables: per instruction a pointer step (shared
  // offsets only), the LDS address and the copy itself.
  static_assert(KMap::NB % C::WAVES == 0 && VMap::NB % C::WAVES == 0, "every wave copies the same number of distinct blocks");
  const int64_t ktile_step = (int64_t)C::BLOCK_N * p.ks[2], vtile_step = (int64_t)C::BLOCK_N * p.vs[2];
  const int64_t kblk_step = (int64_t)KMap::kRowStep * p.ks[2], vblk_step = (int64_t)VMap::kRowStep * p.vs[2];
  const __bf16 *kcp = kbase, *vcp = vbase;  // first rows of the next tile the short form copies (set before its loop)
  const uint32_t kdst0 = lds0 + wave * 1024, vdst0 = vlds0 + wave * 1024;
  auto copy_whole = [&](auto nsl, auto part, int stage) {
    constexpr int NSL = decltype(nsl)::value, PART = decltype(part)::value;
    const uint32_t kdst = kdst0 + stage * C::STAGE_BYTES, vdst = vdst0 + stage * C::STAGE_BYTES;
    static_for<0, kCopies>([&](auto ic) {
      constexpr int n = decltype(ic)::value;
      if constexpr (NSL > 0 ? n % (NSL > 0 ? NSL : 1) == PART : ((n < C::KI) == (PART == 0))) {
        constexpr bool isk = n < C::KI;
        constexpr int m = isk ? n : n - C::KI;
        using Map = std::conditional_t<isk, KMap, VMap>;
        const __bf16* tile = isk ? kcp : vcp;
        if constexpr (Map::kShared) tile += m * (isk ? kblk_step : vblk_step);
        uint32_t goff;
        if constexpr (isk) goff = kgoff[Map::kShared ? 0 : m];
        else goff = vgoff[Map::kShared ? 0 : m];
        dma16_at<m * C::WAVES * 1024>(tile, goff, isk ? kdst : vdst);
      }
    });
  };

  f32x16 s_a;   // scores of the sub-tile to aggregate next
  u32x4 pk[2];  // packed weights of the sub-tile being aggregated
  // initial value of the scoring accumulator: zero; FOLD softmax: minus the row's reference (zero until it has
  // one); FOLD sigmoid: the bias in log2 units
  f32x16 cinit;
#pragma unroll
  for (int r = 0; r < 16; ++r) cinit[r] = (C::FOLD && C::NORM == NORM_SIGMOID) ? p.b2 : 0.f;

  // ---- prologue: Q fragments; tiles 0 and 1 -> LDS; raw scores of sub-tile 0 -------
  // The Q fragments (B operand of S^T = K Q^T, resident for the whole kernel) hold,
  // per lane, 16-byte pieces of one query row: loaded straight from memory, every
  // instruction would touch 32 rows.  The wave's 32 rows are copied to LDS like a K
  // sub-tile instead (1 KB of consecutive bytes per instruction, same swizzle)
  // and read back as fragments.  They land behind stage 0, next to tile 0, which is
  // copied at the same time; tile 1 follows once every wave has its fragments.
  bf16x8 qf[C::T];
  // recurrent pattern, chunks as batch entries: this chunk starts from a carried state (see Params::state)
  constexpr bool kState = C::MOD == MOD_DECAY && C::NORM == NORM_NONE && !C::WINDOW && C::DQK == C::DV && C::DV <= 128;
  bf16x8 hf[kState ? C::DB : 1][kState ? C::T : 1];
  const bool has_state = kState && p.state != nullptr && b >= p.state_b0;  // uniform over the workgroup
  if (n_walk > 0) {
    using QMap = DmaMap<1, 32, C::CPR_K, false>;
    const uint32_t qlds = lds0 + C::STAGE_BYTES + wave * (32 * C::RB_K);
    // rows past the end of the queries repeat the last one (their output is not stored)
    const int qrow0 = min(iw0, max(p.L_q - 32, 0));
    const __bf16* qtile = qbase + (int64_t)qrow0 * p.qs[2];
    if constexpr (!C::kQDirect) {
      static_for<0, QMap::N>([&](auto mc) {
        constexpr int m = decltype(mc)::value;
        const int pos = m * 64 + lane, r = pos / C::CPR_K, pc = pos % C::CPR_K;
        const int row = min(iw0 + r, p.L_q - 1) - qrow0;
        const uint32_t goff = (uint32_t)(row * (int)p.qs[2] + (pc ^ kswz<C::CPR_K>(r)) * 8) * 2u;
        dma16_at<m * 1024>(qtile, goff, qlds);
      });
    }
    copy_slice(One{}, Zero{}, tile_at(0), 0);
    if constexpr (kState) {
      // The state is stored transposed ([D_v][D_qk]), so a lane's A fragment (output column lane % 32 of block
      // db, 8 consecutive d) is 16 bytes of one row.  Plain loads, issued here so that they share the memory
      // latency of the queries and the first tile (the wait below covers all three).
      if (has_state) {
        const __bf16* hrow = p.state + (int64_t)(b - p.state_b0) * p.state_bs + (int64_t)hq * p.state_hs +
                             (int64_t)ql * C::DQK + 8 * half;
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
          for (int tt = 0; tt < C::T; ++tt) hf[db][tt] = *reinterpret_cast<const bf16x8*>(hrow + db * 32 * C::DQK + tt * 16);
      }
    }
    wait_dma_and_sync();  // one memory latency for the queries and the first tile
    uint32_t qaddr[C::T];
    k_frag_offsets<C>(qlds, qaddr);
    const __bf16* qrow = qbase + (int64_t)min(i, p.L_q - 1) * p.qs[2] + 8 * half;  // kQDirect: this lane's row
#pragma unroll
    for (int tt = 0; tt < C::T; ++tt) {
      u32x4 v;
      if constexpr (C::kQDirect) v = *reinterpret_cast<const u32x4*>(qrow + 16 * tt);
      else v = __builtin_bit_cast(u32x4, read_k_frag(qaddr[tt]));
      if (p.neg_q) v ^= (u32x4){0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
      bf16x8 qv = __builtin_bit_cast(bf16x8, v);
      if constexpr (C::FOLD) {
#pragma unroll
        for (int e = 0; e < 8; ++e) qv[e] = (__bf16)((float)qv[e] * p.c);
      }
      qf[tt] = qv;
    }
    if constexpr (kState) {
      // Read-out of the carried state: O^T starts at H^T Q^T instead of zero; the Q fragments serve as B operand
      // as they stand.  Done before the copy of tile 1 is issued: the wait the compiler puts in front of the
      // fragments' first use then finds nothing else in flight.
      if (has_state) {
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
          for (int tt = 0; tt < C::T; ++tt) st.o[db] = mfma(hf[db][tt], qf[tt], st.o[db]);
        const float f = p.c * fast_exp2(g2 * (float)(i + 1));
#pragma unroll
        for (int db = 0; db < C::DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) st.o[db][r] *= f;
      }
    }
    // every wave has read its rows before tile 1 overwrites them
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    copy_slice(One{}, Zero{}, n_walk > 1 ? tile_at(1) : tile_at(0), 1);
    if (C::WINDOW || n_vis > 2 * jt0) score_block<C>(kaddr, 0, qf, s_a, cinit);
  }

  // ---- key loop ------------------------------------------------------------------------
  // On entry to iteration jt LDS holds tile jt, and tile jt+1 is complete or about
  // to be (see below); kaddr / vaddr point into the buffers of tile jt (stage index
  // buf); s_a holds the raw scores of sub-tile 2*jt.
  // Per iteration and wave: vector(2jt) | matrix<0> | vector(2jt+1) | matrix<1>, a
  // barrier after each.  The copy of tile jt+2 goes into the stage of tile jt-1.
  // The trailing half of the waves reads V(jt-1) until the barrier that ends the
  // leading half's vector(2jt), and K(jt-1) only until a phase earlier; so the K
  // tile may be copied from vector(2jt) on and the V tile from matrix<0> on.  The
  // copy is cut into slices issued in different phases (the CU's vector memory
  // path takes 64 bytes per clock; see Cfg::kCopyInVector for where).  Each wave
  // awaits its slices at the end of matrix<0> of the next iteration, one barrier
  // before the first wave reads the tile.
  //
  // A wave issues at most one instruction every four to five clocks, whatever its
  // kind, so the length of a vector phase is its instruction count: the first
  // n_main iterations of a wave -- every key visible to every row, the following
  // sub-tile needed, the tile to copy whole -- run a form of the iteration with no
  // visibility tests, no masking and the short copy; the rest (the diagonal and
  // the end of the keys) run the general form.  Both pass the same barriers; the
  // last two iterations have no tile left to copy and wait for all copies instead.
  if (n_walk > 0) {
    bf16x8 ring[C::PF];
    KeyLoop<C> kl{p, qf, st, pk, cinit, ring, kaddr, vaddr, 0u, 0u, i, off, iw0, g2, false, 1.f, 1.f, 1.f, 1.f};
    if constexpr (C::MOD == MOD_BIAS_T) {
      kl.bwave = p.bias + b * p.bs[0] + hq * p.bs[1];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int r = iw0 + 16 * t + (lane >> 2);
        kl.bgoff[t] = (uint32_t)((int64_t)(r < p.L_q ? r : p.L_q - 1) * p.bs[2] * 2);
      }
      kl.bscr = lds0 + C::TILE_BYTES + wave * 4096;  // behind the K/V stages
    }
    if constexpr (C::MOD == MOD_DECAY) {
      kl.fact = g2 <= 0.f && g2 >= -4.f;  // per head, hence uniform over the workgroup
      kl.a8 = fast_exp2(-8.f * g2);
      kl.b1 = fast_exp2(-g2);
      kl.b2 = fast_exp2(-2.f * g2);
      kl.b3 = fast_exp2(-3.f * g2);
    }
    if (C::WINDOW || n_vis > 2 * jt0) static_for<0, C::PF>([&](auto nc) { kl.template fetch<decltype(nc)::value>(); });
    const bool trailing = wave >= C::WAVES / 2;  // second wave of its SIMD
    int buf = 0;

    // The vector phase of a sub-tile, or all-zero weights for one in front of the wave's window.
    auto vector_or_zero = [&](auto fastc, bool real, int j0) {
      if (real) {
        kl.template vector_phase<decltype(fastc)::value>(s_a, j0);
      } else {
        pk[0] = pk[1] = (u32x4){0u, 0u, 0u, 0u};
        pin(pk[0]);
        pin(pk[1]);
      }
    };
    // One step of the walk: position pos, tile jt = tile_at(pos).
    auto iteration = [&](auto fastc, int pos) {
      constexpr bool FAST = decltype(fastc)::value;
      const int nb = next_buf(buf), stage = next_buf(nb);
      kl.dk = kl.dv = (uint32_t)((nb - buf) * C::STAGE_BYTES);
      const int jt = FAST ? pos + jtm : tile_at(pos);
      const int u = 2 * jt;
      // sub-tiles the wave runs its phases for / has weights of its own in / scores ahead
      const bool vis0 = FAST || C::WINDOW || u < n_vis, vis1 = FAST || C::WINDOW || u + 1 < n_vis;
      const bool real0 = FAST || !C::WINDOW || (u >= u_first && u < n_vis);
      const bool real1 = FAST || !C::WINDOW || (u + 1 >= u_first && u + 1 < n_vis);
      const bool sc0 = FAST || C::WINDOW || u + 1 < n_vis;
      const bool sc1 = FAST || (C::WINDOW ? pos + 1 < n_walk : u + 2 < n_vis);
      const bool more = FAST || pos + 2 < n_walk;  // there is a tile two positions on to copy
      auto copy = [&](auto nsl, auto part) {
        if constexpr (FAST) copy_whole(nsl, part, stage);
        else if (more) copy_slice(nsl, part, tile_at(pos + 2), stage);
      };
      // This wave's share of tile jt+1 has landed: all of its copies but the `newest`
      // of tile jt+2 just issued (if there is a tile jt+2).
      auto await_next_tile = [&](auto newest) {
        if (more) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(decltype(newest)::value) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      };
      // Where the copy of tile jt+2 is issued (see Cfg::kCopyInVector).
      // Vector phase of sub-tile j0 with the copy slice that goes in front of it.  With a bias tensor the
      // sub-tile's bias values are taken first and the next ones requested, ahead of the slice: `newer` copy
      // instructions follow the request before the next vector phase and may stay in flight then.
      auto vector_with_copy = [&](bool vis, bool real, int j0, int newer, auto&& copy_fn) {
        if constexpr (C::MOD == MOD_BIAS_T) {
          if (vis && real) {
            kl.take_bias(j0);
            kl.request_bias(j0, more ? newer : 0);
          }
          copy_fn();
        } else {
          copy_fn();
        }
        if (vis) vector_or_zero(fastc, real, j0);
      };
      if constexpr (C::kCopyInVector) {
        using Part = std::integral_constant<int, -1>;  // 0: the K tile, 1: the V tile
        vector_with_copy(vis0, real0, u * C::SUB_N, C::KI, [&] { copy(Part{}, Zero{}); });
        phase_barrier();
        if (vis0) kl.template matrix_phase<0>(s_a, sc0, [] {});
        await_next_tile(std::integral_constant<int, C::KI>{});
        phase_barrier();
        vector_with_copy(vis1, real1, (u + 1) * C::SUB_N, C::VI, [&] { copy(Part{}, One{}); });
        phase_barrier();
        if (vis1) kl.template matrix_phase<1>(s_a, sc1, [] {});
        phase_barrier();
      } else {
        using Two = std::integral_constant<int, 2>;
        using Three = std::integral_constant<int, 3>;
        constexpr int kSlice0 = (kCopies + 2) / 3;  // instructions in slice 0
        vector_with_copy(vis0, real0, u * C::SUB_N, kSlice0, [] {});  // (slice 0 follows in the matrix phase)
        phase_barrier();
        if (vis0)
          kl.template matrix_phase<0>(s_a, sc0, [&] { copy(Three{}, Zero{}); });
        else
          copy(Three{}, Zero{});
        await_next_tile(std::integral_constant<int, kSlice0>{});
        phase_barrier();
        vector_with_copy(vis1, real1, (u + 1) * C::SUB_N, kCopies - kSlice0, [&] { copy(Three{}, One{}); });
        phase_barrier();
        if (vis1)
          kl.template matrix_phase<1>(s_a, sc1, [&] { copy(Three{}, Two{}); });
        else
          copy(Three{}, Two{});
        phase_barrier();
      }
      if constexpr (FAST) {
        kcp += ktile_step;
        vcp += vtile_step;
      }
      buf = nb;
    };

    // Positions pos < n_fast of this wave take the short form (tile jt = jtm + pos): sub-tiles
    // 2jt, 2jt+1 and 2jt+2 are visible, no key of tile jt is hidden from any of its rows
    // (neither by the diagonal, nor by the end of the keys, nor -- from jtm on -- by the lower
    // edge of a window), and the tile two positions on is a whole tile before the rotation.
    int m1 = min((n_vis - 1) / 2, min(p.L_k / C::BLOCK_N, n_tiles) - 2);
    if (C::CAUSAL) m1 = min(m1, (iw0 + off + 1) / C::BLOCK_N);
    const int n_fast = max(m1 - jtm, 0);

    if (trailing) phase_barrier();
    kcp = kbase + (jtm + 2) * ktile_step;  // the first tile the short form copies
    vcp = vbase + (jtm + 2) * vtile_step;
    int pos = 0;
    for (; pos < n_fast; ++pos) iteration(std::true_type{}, pos);
    for (; pos < n_walk; ++pos) iteration(std::false_type{}, pos);
    if (!trailing) phase_barrier();  // both halves are at the same point again
  }
  // No copy is in flight (the last iterations issue none) and every wave is past its
  // last fragment read: the LDS of the tiles is free.
  wait_dma_and_sync();

  // ---- online_epilogue + store ------------------------------------------------
  float inv = 1.f;
  if constexpr (C::NORM == NORM_SOFTMAX || C::NORM == NORM_ABSSUM || C::NORM == NORM_ABS_OF_SUM) {
    const float l = sum_halves(st.l);
    float stat = l;  // abs-sum family: the sum itself
    if constexpr (C::NORM == NORM_SOFTMAX) {
      inv = l > 0.f ? 1.f / l : 0.f;
      // weights are 2^(x*log2e - m): sum_j exp(x_j) = 2^m * l  (FOLD leaves a constant bias out of m: every
      // weight of the row carries it, so only the statistic sees it)
      stat = l > 0.f ? (st.m + (C::FOLD ? p.b2 : 0.f) + __builtin_amdgcn_logf(l)) * 0.6931471805599453f : -INFINITY;
    } else if constexpr (C::NORM == NORM_ABSSUM) {
      inv = 1.f / fmaxf(l, 1.f);
    } else {
      inv = 1.f / fmaxf(fabsf(l), 1.f);
    }
    if (stats != nullptr && half == 0 && i < p.L_q) stats[i] = stat;
  }
  // A lane holds 4-column pieces of one output row, 32 bytes apart from its
  // partner's: stored directly, every instruction would touch 32 rows with 32
  // bytes each.  Instead each wave turns its 32 x OC block around in a private
  // piece of LDS (16-byte chunk c of row r at position c ^ (r % 16): both the
  // column-wise writes and the row-wise reads are free of bank conflicts) and
  // stores whole rows, 1 KB of full cache lines per instruction.
  constexpr int OC = C::OC, CPRO = OC / 4, DBP = OC / 32;
  const uint32_t obuf = lds0 + wave * (32 * OC * 4);
#pragma unroll
  for (int pass = 0; pass < C::DV / OC; ++pass) {
#pragma unroll
    for (int dbl = 0; dbl < DBP; ++dbl)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = st.o[pass * DBP + dbl][4 * r4 + e] * inv;
        const int c = dbl * 8 + r4 * 2 + half;
        lds_write16(obuf + ql * (OC * 4) + ((c ^ (ql & 15)) * 16), v);
      }
#pragma unroll
    for (int k = 0; k < 32 * CPRO / 64; ++k) {
      const int row = k * (64 / CPRO) + lane / CPRO, pc = lane % CPRO;
      const f32x4 v = lds_read16(obuf + row * (OC * 4) + ((pc ^ (row & 15)) * 16));
      if (iw0 + row < p.L_q) {
        const int64_t e = (int64_t)(iw0 + row) * o_row + pass * OC + pc * 4;  // element offset in the head
        if (o_bf16) {
          bf16x4 h;
#pragma unroll
          for (int k4 = 0; k4 < 4; ++k4) h[k4] = (__bf16)v[k4];
          *reinterpret_cast<bf16x4*>(obase + e * 2) = h;
        } else {
          *reinterpret_cast<f32x4*>(obase + e * 4) = v;
        }
      }
    }
  }
}

}  // namespace ae
