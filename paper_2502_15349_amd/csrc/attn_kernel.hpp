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
// Instruction stream.  On this hardware a wave that issues MFMAs back to back
// keeps the SIMD's issue stage to itself: the vector work of the other wave on
// the SIMD does not slip in between, and matrix and vector phases of the two
// waves simply add up.  What does overlap is vector work placed BETWEEN the
// MFMAs of the same wave.  The key loop is therefore software-pipelined over
// sub-tiles (PIPE) so that every MFMA has vector work of a different sub-tile
// next to it:
//   phase A(u):  S(u+1) = K(u+1) Q^T  (MFMA)  ||  first half of the weights P(u)
//   phase B(u):  O += V(u)^T P(u)     (MFMA)  ||  second half of P(u), then
//                                                  mask / row max of S(u+1)
// written as explicit groups "one MFMA + the LDS read for a later MFMA + a slice
// of vector work" fenced from each other.  Without PIPE (head dims whose
// accumulators leave no room for a second score buffer) the four pieces run one
// after the other per sub-tile.
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

// Optional phase timing (build with -DAE_PROFILE): per-wave cycle totals between
// the marked points are written to the buffer passed in Params::prof.
#ifdef AE_PROFILE
#define AE_TICK(k)                                      \
  do {                                                  \
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  \
    const uint64_t now_ = __builtin_readcyclecounter(); \
    prof_acc[k] += now_ - prof_last;                    \
    prof_last = now_;                                   \
  } while (0)
#else
#define AE_TICK(k) \
  do {             \
  } while (0)
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
  const __bf16* V;   // [B, H_kv, L_k, D_v], or with VT kernels the transposed copy [B, H_kv, D_v, ldvt]
  float* O;
  int B, H_q, H_kv, L_q, L_k;
  int g;           // H_q / H_kv
  int n_qtiles;    // ceil(L_q / BLOCK_M)
  int n_groups;    // B * H_kv
  int interleave;  // (batch, kv head) groups walked together on one XCD
  int ldvt;        // VT kernels: keys per row of the transposed V copy (L_k rounded up to 64, zero filled)
  int64_t qs[3], ks[3], vs[3], os[3];  // element strides {batch, head, row}
  float c;         // |scale| * log2(e)  (softmax, sigmoid)  or |scale| (others)
  float b2;        // bias * log2(e)     (softmax, sigmoid)  or bias (others)
  int neg_q;       // scale < 0: the sign is moved onto Q (exact for bf16)
  unsigned long long* prof;  // AE_PROFILE builds: [grid][waves][8] cycle totals, else unused
};

struct DecayTable {
  float log2_gamma[kMaxDecayHeads];
};

template <int DQK_, int DV_, int NORM_, int MOD_, bool CAUSAL_, int WAVES_, bool PIPE_, bool VT_>
struct Cfg {
  static constexpr int DQK = DQK_, DV = DV_, NORM = NORM_, MOD = MOD_, WAVES = WAVES_;
  static constexpr bool CAUSAL = CAUSAL_, PIPE = PIPE_;
  // VT: V arrives pre-transposed ([D_v][keys], written by transpose_v_kernel), so the
  // aggregation reads its A fragments with one 128-bit LDS load instead of two
  // 64-bit transposing loads (LDS instruction issue is the first limit of this
  // kernel).  The key order inside a 16-key step then has to be the natural one,
  // which is arranged by permuting which K row each lane scores (k_frag_offsets).
  static constexpr bool VT = VT_;
  static constexpr int SUB_N = 32;    // keys per compute sub-tile
  static constexpr int BLOCK_N = 64;  // keys per LDS tile (two sub-tiles)
  static constexpr int BLOCK_M = 32 * WAVES;
  static constexpr int THREADS = 64 * WAVES;
  // LDS tiles are row-major and unpadded; CPR = 16-byte chunks per row.
  static constexpr int RB_K = DQK * 2, RB_V = DV * 2;
  static constexpr int CPR_K = DQK / 8, CPR_V = VT ? 8 : DV / 8;  // VT: rows are 64 keys = 128 bytes
  static constexpr int K_BYTES = BLOCK_N * RB_K;
  static constexpr int V_BYTES = BLOCK_N * RB_V;  // same size either way round
  // Scoring runs one sub-tile ahead of aggregation, so while tile j is being
  // aggregated K(j) and K(j+1) are both read and K(j+2) is arriving; V(j) is
  // read while V(j+1) arrives.
  static constexpr int K_STAGES = 3, V_STAGES = 2;
  static constexpr int LDS_BYTES = K_STAGES * K_BYTES + V_STAGES * V_BYTES;
  static constexpr int NB_K = K_BYTES / 1024, NB_V = V_BYTES / 1024;  // 1 KB blocks per tile
  static constexpr int KI = (NB_K + WAVES - 1) / WAVES, VI = (NB_V + WAVES - 1) / WAVES;
  static constexpr int T = DQK / 16;  // contraction steps of the scoring MFMA
  static constexpr int DB = DV / 32;  // 32-wide blocks of output columns
  static constexpr int VA = VT ? 4 : DB;  // per-lane V fragment base addresses
  static_assert(DQK % 16 == 0 && DV % 32 == 0, "head dims must fit the MFMA tile");
  static_assert(K_BYTES % 1024 == 0 && V_BYTES % 1024 == 0, "tiles must be whole 1 KB blocks");
  static_assert(CPR_K == 8 || CPR_K == 16 || CPR_K == 24, "K swizzle is defined for these row sizes");
  static_assert(CPR_V == 8 || CPR_V == 16 || CPR_V == 32, "V swizzle is defined for these row sizes");
  static_assert(LDS_BYTES <= 160 * 1024, "tiles do not fit LDS");
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
// Rows past the end of the sequence re-read the last valid row: their scores
// are masked, and finite values keep 0 * V finite.
template <int WAVES, int ROWS, int CPR, int N>
__device__ __forceinline__ void dma_tile(const __bf16* base, int64_t row_stride, int j0, int L_k, uint32_t lds, int wave,
                                         const uint32_t (&goff)[N], const int (&grow)[N]) {
  constexpr int NB = ROWS * CPR / 64;
  const __bf16* tile = base + (int64_t)j0 * row_stride;  // wave-uniform
  if (j0 + ROWS <= L_k) {
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
// waves: what they waited for is visible too.  A bare s_barrier is enough: LDS
// reads of the step have returned by then (each was awaited by the MFMA that
// consumed it), so a buffer is only overwritten after every wave is done
// reading it.
__device__ __forceinline__ void wait_dma_and_sync() { asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory"); }

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
// (VT kernels: register r is key j0 + 16*(r/8) + 8*half + (r%8), see k_frag_offsets.)
template <bool VT>
__device__ __forceinline__ constexpr int key_offset(int r) {
  return VT ? 16 * (r / 8) + (r % 8) : 8 * (r / 4) + (r % 4);
}

// Per-sub-tile, per-lane constants of the modification.
struct TileCtx {
  int jlim;     // register r is visible  <=>  key_offset(r) <= jlim   (masked sub-tiles only)
  float dbase;  // decay: log2(gamma) * (i + off - j0 - (4 or 8)*half)
};

template <class C, bool MASKED>
__device__ __forceinline__ TileCtx tile_ctx(const Params& p, int i, int j0, int off, float g2) {
  const int half = (threadIdx.x & 63) >> 5;
  TileCtx c;
  constexpr int HS = C::VT ? 8 : 4;  // key offset of the upper half wave
  c.jlim = MASKED ? min(C::CAUSAL ? i + off : p.L_k - 1, p.L_k - 1) - j0 - HS * half : 0;
  c.dbase = C::MOD == MOD_DECAY ? g2 * (float)(i + off - j0 - HS * half) : 0.f;
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
    const bool hidden = MASKED && (key_offset<C::VT>(r) > tc.jlim);
    if constexpr (C::NORM == NORM_SOFTMAX) {
      if (hidden) x = -INFINITY;
    } else if constexpr (C::NORM == NORM_SIGMOID) {
      x = fast_exp2(__builtin_fmaf(x, -p.c, -p.b2));
      if (hidden) x = INFINITY;
    } else {
      if constexpr (C::MOD == MOD_DECAY) {
        // gamma^(i + off - j) = 2^(log2(gamma) * (i + off - j))
        x = x * p.c * fast_exp2(__builtin_fmaf(-g2, (float)key_offset<C::VT>(r), tc.dbase));
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
  const int half = lane >> 5;
  int ql = lane & 31;
  // VT: MFMA row m scores key (m with bits 2 and 3 swapped), so that a lane's
  // accumulator registers 8t..8t+7 are keys 16t + 8*half + 0..7 in order -- the
  // order of a 16-byte piece of a transposed V row.
  if (C::VT) ql = (ql & ~12) | ((ql & 4) << 1) | ((ql & 8) >> 1);
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
__device__ __forceinline__ void v_frag_offsets(uint32_t base, uint32_t (&vaddr)[C::VA]) {
  const int lane = threadIdx.x & 63;
  const int half = lane >> 5, li = lane & 15;
  if constexpr (C::VT) {
    // Transposed tile: row d (128 bytes = 64 keys), chunk 2*ts + half holds keys
    // 16*ts + 8*half .. +7 (ts = 16-key step inside the tile, 0..3).  Chunks are
    // swizzled like K rows of 128 bytes; output-column block db is at +32 rows.
    const int d = lane & 31;
#pragma unroll
    for (int ts = 0; ts < 4; ++ts) vaddr[ts] = base + d * 128 + (((2 * ts + half) ^ kswz<8>(d)) * 16);
  } else {
    const int row = 4 * half + (li >> 2);
    const int cl = 2 * ((lane >> 4) & 1) + ((li & 3) >> 1);  // chunk within the 64-byte group
#pragma unroll
    for (int db = 0; db < C::DB; ++db)
      vaddr[db] = base + row * C::RB_V + ((4 * (db ^ vswz<C::CPR_V>(row)) + cl) * 16) + (li & 1) * 8;
  }
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
__device__ __forceinline__ bf16x8 load_v_frag(const uint32_t (&vaddr)[C::VA], int sub, int t, int db) {
  if constexpr (C::VT)
    return read_k_frag(vaddr[2 * sub + t] + db * 32 * 128);
  else
    return read_v_frag(vaddr[db] + (32 * sub + 16 * t) * C::RB_V, 8 * C::RB_V);
}

constexpr int kFragAhead = 4;  // LDS fragment reads kept in flight ahead of their MFMA

// ---- phase A: S_nxt = K_sub Q^T  ||  weight pairs [FIN_LO, FIN_HI) of s_cur ------
//   DO_QK   score the sub-tile whose first row is at LDS offset `krow_off` of the
//           buffer kaddr points into
template <class C, bool DO_QK, int FIN_LO, int FIN_HI>
__device__ __forceinline__ void phase_a(const Params& p, const uint32_t (&kaddr)[C::T], int krow_off,
                                        const bf16x8 (&qf)[C::T], f32x16& s_nxt, const f32x16& s_cur, float k0,
                                        float& acc, u32x4 (&pk)[2]) {
  constexpr int NM = DO_QK ? C::T : 0, NPAIR = FIN_HI - FIN_LO;
  // Pairs done before the first MFMA: they cover the latency of the first
  // fragment reads, which cannot be issued before the tile is published.
  constexpr int FRONT = !DO_QK ? NPAIR : (NPAIR >= 4 ? 1 : 0);
  constexpr int PF = kFragAhead < NM ? kFragAhead : NM;

  bf16x8 ring[PF > 0 ? PF : 1];
#pragma unroll
  for (int g = 0; g < PF; ++g) ring[g] = read_k_frag(kaddr[g] + krow_off);
#pragma unroll
  for (int q = FIN_LO; q < FIN_LO + FRONT; ++q) pk[q / 4][q % 4] = finish_pair<C>(p, q, s_cur, k0, acc);
  sched_fence();

#pragma unroll
  for (int g = 0; g < NM; ++g) {
    if (g == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s_nxt[r] = 0.f;
    }
    s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[g % PF], qf[g], s_nxt, 0, 0, 0);
    if (g + PF < NM) ring[g % PF] = read_k_frag(kaddr[g + PF] + krow_off);  // refill the slot just consumed
#pragma unroll
    for (int q = FIN_LO + FRONT; q < FIN_HI; ++q)
      if ((q - FIN_LO - FRONT) * NM / (NPAIR - FRONT) == g) pk[q / 4][q % 4] = finish_pair<C>(p, q, s_cur, k0, acc);
    sched_fence();
  }
}

// ---- phase B: O^T += V_sub^T P^T  ||  weight pairs [FIN_LO, 8) of s_cur, then the
//      modification / row max of s_nxt ---------------------------------------------
//   DO_PV    aggregate sub-tile `vsub` (0/1) of the V tile vaddr points into
//   DO_POST  mask / modify / reduce the freshly scored s_nxt (sub-tile starting at j0)
// The aggregation MFMAs run key-step major: the first DB of them need weight
// pairs 0..3 only, so pairs 4..7 may still be computed next to those.
template <class C, bool DO_PV, int FIN_LO, bool DO_POST, bool MASKED>
__device__ __forceinline__ void phase_b(const Params& p, const uint32_t (&vaddr)[C::VA], int vsub, u32x4 (&pk)[2],
                                        RowState<C>& st, const f32x16& s_cur, float k0, float& acc, f32x16& s_nxt,
                                        int i, int j0, int off, float g2, bool& moved, float& xm) {
  constexpr int DB = C::DB, NM = DO_PV ? 2 * DB : 0;
  constexpr int NFIN = DO_PV ? 8 - FIN_LO : 0, NPOST = DO_POST ? 8 : 0;
  static_assert(FIN_LO >= 4 || !DO_PV, "pairs 0..3 must be complete before aggregation starts");
  constexpr int PF = kFragAhead < NM ? kFragAhead : NM;
  // MFMAs [0, DB) carry the remaining weight pairs, MFMAs [DB, 2*DB) the post work;
  // with nothing to aggregate the post work simply runs.
  constexpr int POST_FRONT = !DO_PV ? NPOST : 0;

  bf16x8 ring[PF > 0 ? PF : 1];
#pragma unroll
  for (int g = 0; g < PF; ++g) ring[g] = load_v_frag<C>(vaddr, vsub, g / DB, g % DB);

  TileCtx tc;
  if constexpr (DO_POST) tc = tile_ctx<C, MASKED>(p, i, j0, off, g2);
  float mx = -INFINITY;
#pragma unroll
  for (int q = 0; q < POST_FRONT; ++q) post_pair<C, MASKED>(p, q, s_nxt, tc, g2, mx);
  sched_fence();

#pragma unroll
  for (int g = 0; g < NM; ++g) {
    const int t = g / DB, db = g % DB;
    st.o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[g % PF], __builtin_bit_cast(bf16x8, pk[t]), st.o[db], 0, 0, 0);
    if (g + PF < NM)  // refill the slot just consumed
      ring[g % PF] = load_v_frag<C>(vaddr, vsub, (g + PF) / DB, (g + PF) % DB);
    if (g < DB) {
#pragma unroll
      for (int q = FIN_LO; q < 8; ++q)
        if ((q - FIN_LO) * DB / (NFIN > 0 ? NFIN : 1) == g) pk[q / 4][q % 4] = finish_pair<C>(p, q, s_cur, k0, acc);
    } else {
#pragma unroll
      for (int q = 0; q < NPOST; ++q)
        if (q * DB / 8 == g - DB) post_pair<C, MASKED>(p, q, s_nxt, tc, g2, mx);
    }
    sched_fence();
  }
  if constexpr (DO_POST) post_done<C>(p, st, mx, moved, xm);
}

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
  const __bf16* vbase = C::VT ? p.V + ((int64_t)b * p.H_kv + hkv) * C::DV * p.ldvt : p.V + b * p.vs[0] + hkv * p.vs[1];
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
  for (int db = 0; db < C::DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) st.o[db][r] = 0.f;

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
  // wave-uniform: does sub-tile u cross the causal diagonal or the end of the keys?
  auto needs_mask = [&](int u) {
    const int j0 = u * C::SUB_N;
    return (j0 + C::SUB_N > p.L_k) || (C::CAUSAL && (j0 + C::SUB_N - 1 > iw0 + off));
  };

  // LDS: K_STAGES K buffers, then V_STAGES V buffers; tile j lives in buffer j % stages.
  const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_char*)smem);
  const uint32_t vlds0 = lds0 + C::K_STAGES * C::K_BYTES;
  uint32_t kaddr[C::T], vaddr[C::VA];  // fragment addresses inside the K / V buffer in use
  k_frag_offsets<C>(lds0, kaddr);
  v_frag_offsets<C>(vlds0, vaddr);
  uint32_t kgoff[C::KI], vgoff[C::VI];
  int kgrow[C::KI], vgrow[C::VI];
  dma_offsets<C::WAVES, C::BLOCK_N, C::CPR_K, false>(wave, p.ks[2], kgoff, kgrow);
  if constexpr (C::VT)  // tile = D_v rows of 64 keys out of rows of ldvt keys; swizzled like K
    dma_offsets<C::WAVES, C::DV, 8, false>(wave, p.ldvt, vgoff, vgrow);
  else
    dma_offsets<C::WAVES, C::BLOCK_N, C::CPR_V, true>(wave, p.vs[2], vgoff, vgrow);
  // Tile indices past the last tile are clamped: the copy is redundant but keeps
  // every wave's stream of loads identical.
  const int last_tile = max(n_tiles - 1, 0);
  auto load_k = [&](int jt) {
    dma_tile<C::WAVES, C::BLOCK_N, C::CPR_K>(kbase, p.ks[2], min(jt, last_tile) * C::BLOCK_N, p.L_k,
                                             lds0 + (jt % C::K_STAGES) * C::K_BYTES, wave, kgoff, kgrow);
  };
  auto load_v = [&](int jt) {
    const uint32_t dst = vlds0 + (jt % C::V_STAGES) * C::V_BYTES;
    if constexpr (C::VT) {
      // key columns [64*jt, +64) of every row of the transposed copy (zero filled past L_k)
      const __bf16* tile = vbase + (int64_t)min(jt, last_tile) * C::BLOCK_N;
#pragma unroll
      for (int n = 0; n < C::VI; ++n) dma16(tile, vgoff[n], dst + ((wave + n * C::WAVES) % C::NB_V) * 1024);
    } else {
      dma_tile<C::WAVES, C::BLOCK_N, C::CPR_V>(vbase, p.vs[2], min(jt, last_tile) * C::BLOCK_N, p.L_k, dst, wave, vgoff,
                                               vgrow);
    }
  };

  f32x16 s_a, s_b;  // scores of the even / odd sub-tile in flight (without PIPE only s_a)
  u32x4 pk[2];      // packed weights of the sub-tile being aggregated
  bool moved = false;
  float xm = 0.f;

#ifdef AE_PROFILE
  uint64_t prof_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  uint64_t prof_last = __builtin_readcyclecounter();
#endif

  // ---- prologue: K(0), K(1), V(0) -> LDS; score and reduce sub-tile 0 ------------
  if (n_tiles > 0) {
    load_k(0);
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    load_k(1);
    load_v(0);
    if (n_vis > 0) {
      float acc0 = 0.f;
      phase_a<C, true, 0, 0>(p, kaddr, 0, qf, s_a, s_a, 0.f, acc0, pk);
      if (needs_mask(0))
        phase_b<C, false, 8, true, true>(p, vaddr, 0, pk, st, s_a, 0.f, acc0, s_a, i, 0, off, g2, moved, xm);
      else
        phase_b<C, false, 8, true, false>(p, vaddr, 0, pk, st, s_a, 0.f, acc0, s_a, i, 0, off, g2, moved, xm);
      lazy_rescale<C>(st, moved, xm);
    }
    wait_dma_and_sync();
  }

  // One sub-step: sub-tile u (scores in s_cur, already modified / reduced) is
  // turned into weights and aggregated from V rows [vrow_off, +32) of the
  // current V buffer (sub-tile vsub of it) while sub-tile u+1 is scored from K rows [krow_off, +32)
  // of the buffer kaddr points into, into s_nxt.
  auto sub_step = [&](int u, f32x16& s_cur, f32x16& s_nxt, int krow_off, int vsub) {
    if (u >= n_vis) return;
    const bool more = u + 1 < n_vis;
    const float k0 = finish_k0<C>(p, st);
    float acc = 0.f;
    if constexpr (C::PIPE) {
      if (more) {
        AE_TICK(0);
        phase_a<C, true, 0, 4>(p, kaddr, krow_off, qf, s_nxt, s_cur, k0, acc, pk);
        AE_TICK(1);
        if (needs_mask(u + 1))
          phase_b<C, true, 4, true, true>(p, vaddr, vsub, pk, st, s_cur, k0, acc, s_nxt, i, (u + 1) * C::SUB_N, off,
                                          g2, moved, xm);
        else
          phase_b<C, true, 4, true, false>(p, vaddr, vsub, pk, st, s_cur, k0, acc, s_nxt, i, (u + 1) * C::SUB_N, off,
                                           g2, moved, xm);
        AE_TICK(2);
        finish_done<C>(st, acc);
        lazy_rescale<C>(st, moved, xm);
        AE_TICK(3);
      } else {
        // this wave's last visible sub-tile: nothing further to score
        phase_a<C, false, 0, 4>(p, kaddr, krow_off, qf, s_nxt, s_cur, k0, acc, pk);
        phase_b<C, true, 4, false, false>(p, vaddr, vsub, pk, st, s_cur, k0, acc, s_nxt, i, 0, off, g2, moved, xm);
        finish_done<C>(st, acc);
      }
    } else {
      // one score buffer: weights and aggregation of sub-tile u, then the scores
      // of sub-tile u+1 into the same registers
      AE_TICK(0);
      phase_a<C, false, 0, 8>(p, kaddr, krow_off, qf, s_cur, s_cur, k0, acc, pk);
      finish_done<C>(st, acc);
      AE_TICK(1);
      phase_b<C, true, 8, false, false>(p, vaddr, vsub, pk, st, s_cur, k0, acc, s_cur, i, 0, off, g2, moved, xm);
      AE_TICK(2);
      if (more) {
        phase_a<C, true, 0, 0>(p, kaddr, krow_off, qf, s_cur, s_cur, k0, acc, pk);
        AE_TICK(3);
        if (needs_mask(u + 1))
          phase_b<C, false, 8, true, true>(p, vaddr, vsub, pk, st, s_cur, k0, acc, s_cur, i, (u + 1) * C::SUB_N, off,
                                           g2, moved, xm);
        else
          phase_b<C, false, 8, true, false>(p, vaddr, vsub, pk, st, s_cur, k0, acc, s_cur, i, (u + 1) * C::SUB_N, off,
                                            g2, moved, xm);
        lazy_rescale<C>(st, moved, xm);
        AE_TICK(4);
      }
    }
  };

  // ---- main loop over LDS tiles -------------------------------------------------
  // On entry to iteration jt LDS holds K(jt), K(jt+1) and V(jt); kaddr points
  // into K(jt)'s buffer and vaddr into V(jt)'s; s_a holds sub-tile 2*jt.
  int kbuf = 0, vbuf = 0;  // buffer index of tile jt
  for (int jt = 0; jt < n_tiles; ++jt) {
    // K(jt+2) replaces K(jt-1), V(jt+1) replaces V(jt-1): nobody reads those any more
    load_k(jt + 2);
    load_v(jt + 1);
    AE_TICK(5);

    f32x16& s_odd = C::PIPE ? s_b : s_a;
    sub_step(2 * jt, s_a, s_odd, 32 * C::RB_K, 0);  // scores rows 32..63 of K(jt)
    {
      const int nk = (kbuf + 1 == C::K_STAGES) ? 0 : kbuf + 1;
      const uint32_t dk = (uint32_t)((nk - kbuf) * C::K_BYTES);
#pragma unroll
      for (int t = 0; t < C::T; ++t) kaddr[t] += dk;
      kbuf = nk;
    }
    sub_step(2 * jt + 1, s_odd, s_a, 0, 1);  // scores rows 0..31 of K(jt+1)
    {
      const int nv = (vbuf + 1 == C::V_STAGES) ? 0 : vbuf + 1;
      const uint32_t dv = (uint32_t)((nv - vbuf) * C::V_BYTES);
#pragma unroll
      for (int a = 0; a < C::VA; ++a) vaddr[a] += dv;
      vbuf = nv;
    }
    AE_TICK(6);
    wait_dma_and_sync();  // K(jt+2) and V(jt+1) have landed everywhere
    AE_TICK(7);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // redundant tail copies must land before LDS is released

#ifdef AE_PROFILE
  if (p.prof && lane == 0)
    for (int k = 0; k < 8; ++k) p.prof[((size_t)blockIdx.x * C::WAVES + wave) * 8 + k] = prof_acc[k];
#endif

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
