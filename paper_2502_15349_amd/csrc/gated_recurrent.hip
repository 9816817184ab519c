// Recurrent pattern with per-token gates, in one pass (paper Section 4.1, "Attention Patterns and Templates": K@V,
// then Q@h, iterated over a compressed state; "Examples of Attention variants": Mamba2's k_mod = k x gate and
// h_mod = h x decay x gate; Table 2: "Mamba2 SSM", "Gated Retention", "Retention Recurrent"; Section 4.2: chunk
// parallelism for the matrix units):
//     h_t = a_t h_{t-1} + (g_t k_t)^T v_t,     o_t = scale q_t h_t,        a_t = exp(log_decay_t) in (0, 1].
//
// One workgroup per (batch, value head) walks the sequence in chunks of 64 tokens with the state in registers
// (fp32 MFMA accumulators) from the first token to the last: Q, K, V are read once, O is written once, the state
// never touches memory (only h_in / h_out at the ends).  With b_i the sum of the log-decays from the chunk's first
// token to token i (b_i <= 0, decreasing), for token i of the chunk and H the state in front of the chunk:
//     o_i   = scale e^{b_i} q_i H  +  sum_{j <= i} scale e^{b_i - b_j} g_j (q_i . k_j) v_j
//     H_new = e^{b_last} H + sum_j (e^{b_last - b_j} g_j) k_j^T v_j
// Every exponent is <= 0: nothing overflows, nothing is divided by a decay.
//
// A wavefront owns 32 of the D_v output columns and keeps, for its columns, the state slab [D_qk x 32] as D_qk / 32
// accumulator tiles.  It takes both of the chunk's two blocks of 32 queries (QS = 1: D_v / 32 wavefronts per head,
// each alone on its SIMD with the whole register file) or one of them (QS = 2: two wavefronts per column block that
// both hold the slab and both apply every update to it -- the same instructions on the same operands, so the copies
// stay bit-identical -- where the registers allow two wavefronts per SIMD: 64 / 128).  The path is bound by memory
// and by the latency chain of a chunk, not by MFMAs.
// All products are transposed so that a lane owns one column -- a
// query in S^T and O^T, a value column in H -- and the registers run over the contracted index:
//     S^T [keys x queries]   = K Q^T          A: K rows, B: Q rows (16-byte row pieces in the d order below)
//     R^T [v x queries]      = H^T Q^T        A: the state accumulators themselves, packed to bf16 (lane = value
//                                                column, registers = d: an accumulator tile IS an A operand whose
//                                                contraction runs over its rows), B: the same Q fragments
//     O^T += V^T P^T                          A: V through the transposing LDS read, B: the S^T accumulators,
//                                                weighted and packed (no data movement)
//     H   += K^T (w . V)                      A: K through the transposing read, B: the same V fragments times
//                                                the per-token weights w_j = e^{b_last - b_j} g_j
// The contraction order over d is free, so Q and K rows are read in the order the accumulator layout of H
// dictates (register r of a tile is row 8 (r / 4) + 4 (lane / 32) + r % 4): two 8-byte pieces per fragment.
// Of the three 32 x 32 blocks of S^T that the causal order inside a chunk leaves, a wavefront computes those of
// its query block itself (cheaper than an exchange through LDS and a barrier).
// Q, K, V tiles and the chunk's gates arrive by LDS-DMA into a ring of three stages (chunk c is worked on while
// c + 1 and c + 2 are in flight), one barrier per chunk, the wavefronts issuing their shares of the copies at
// different points of the iteration.  The output of a chunk is stored before the state update, whose MFMAs cover
// the stores.  The same kernel serves the backward pass (other operands, a walk from the last token to the first,
// see GatedParams::reverse) and walks cut into segments (GatedParams::nseg).
#include <hip/hip_runtime.h>

#include "attn_bwd_kernel.hpp"  // bswz, read_tr_frag
#include "gated.hpp"

#ifndef AE_GATED_QS_128
#define AE_GATED_QS_128 1  // wavefronts per block of 32 value columns at 128/128 (build-time knob of the sweeps)
#endif

namespace ae {
namespace {

// HPW_: value heads per workgroup.  Heads of one q/k group (Mamba2: every head of a group reads the same B and C)
// can share the Q and K tiles of a workgroup: HPW_ consecutive heads, each with its own V tile, gates and state.
// QS_: wavefronts per block of 32 value columns: 2 (one per query block of the chunk, see above) or 1 (both query
// blocks in one wavefront: half the wavefronts, each with the whole register file where 2 would spill).
template <int DQK_, int DV_, int HPW_ = 1, int QS_ = 2>
struct GCfg {
  static constexpr int DQK = DQK_, DV = DV_, HPW = HPW_, QS = QS_, WPH = QS_ * (DV_ / 32), WAVES = HPW_ * WPH, THREADS = 64 * WAVES, CH = 64;
  static constexpr int RBQ = DQK * 2, RBV = DV * 2, CPRQ = DQK / 8, CPRV = DV / 8;
  static constexpr int Q_BYTES = CH * RBQ, V_BYTES = CH * RBV, STAGE_BYTES = 2 * Q_BYTES + HPW * V_BYTES;
  static constexpr int STAGES = 3;                // chunk c is worked on while c + 1 and c + 2 are arriving
  static constexpr int GATE_BYTES = 3 * CH * 4;   // per wavefront: b, g, w of the chunk's tokens
  static constexpr int RAW_BYTES = 2 * CH * 4;    // per head and stage: the chunk's log-decays and key gates as they arrive
  static constexpr int LDS_BYTES = STAGES * (STAGE_BYTES + HPW * RAW_BYTES) + WAVES * GATE_BYTES + 256;  // (+ a row nobody reads)
  // copy instructions per wavefront and chunk: its shares of the Q, K and V tiles and one of the two gate rows
  static constexpr int NDMA = 2 * (CPRQ / WAVES) + CPRV / WPH + 1;
  static constexpr int NST = 4 * (3 - QS);        // store instructions per wavefront and (whole) chunk
  static constexpr int T = DQK / 16, DBQ = DQK / 32;
  static_assert(CPRQ % WAVES == 0 && CPRV % WPH == 0, "every wave copies the same number of 1 KB blocks");
  static_assert(LDS_BYTES <= 160 * 1024, "tiles do not fit LDS");
};

__device__ __forceinline__ u32x2 lds_read8(uint32_t addr) {
  return *reinterpret_cast<__attribute__((address_space(3))) const u32x2*>((lds_char*)(uintptr_t)addr);
}
__device__ __forceinline__ void lds_write4(uint32_t addr, float v) {
  *reinterpret_cast<__attribute__((address_space(3))) float*>((lds_char*)(uintptr_t)addr) = v;
}

// 64 lanes x 4 bytes from base + byte_off (per lane) to LDS bytes [lds_addr, lds_addr + 256)
__device__ __forceinline__ void dma4(const void* base_uniform, uint32_t byte_off, uint32_t lds_addr_uniform) {
  base_uniform = uniform_ptr(base_uniform);
  lds_addr_uniform = __builtin_amdgcn_readfirstlane(lds_addr_uniform);
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dword %1, %2"
      :
      : "s"(lds_addr_uniform), "v"(byte_off), "s"(base_uniform)
      : "memory", "m0");
}

// x of the lane that the control word selects, 0 where it selects none or the masks switch the lane off
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ float dpp_f(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, BANK_MASK, false));
}

template <class C>
__global__ __launch_bounds__(C::THREADS) void gated_recurrent_kernel(const GatedParams p, const DecayTable dt) {
  __shared__ __attribute__((aligned(1024))) char smem[C::LDS_BYTES];
  const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_char*)smem);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ln = lane & 31, half = lane >> 5;
  // workgroup -> batch entry and HPW consecutive value heads of one q/k group; wave -> (head, 32 value columns,
  // query block of the chunk)
  const int hw = wave / C::WPH, wh = wave % C::WPH, vblk = wh / C::QS, ib = wh % C::QS;
  const int seg = blockIdx.x % p.nseg;
  const int bh0 = (blockIdx.x / p.nseg) * C::HPW, b = bh0 / p.H, h = bh0 % p.H + hw, bh = bh0 + hw;
  const int hqk = h / (p.H / p.H_qk);
  const bool rev = p.reverse != 0;
  // the tokens this workgroup walks: L of them from position `first` of the walk (the whole sequence unless it is
  // cut into segments); row_lo: the one with the lowest address, where all base pointers below stand
  const int64_t Lt = p.L, first = (int64_t)seg * p.seg_len;
  const int64_t L = p.nseg > 1 ? min(Lt - first, (int64_t)p.seg_len) : Lt;
  const int64_t row_lo = rev ? Lt - first - L : first;
  const __bf16* Qh = p.Q + (((int64_t)b * p.H_qk + hqk) * Lt + row_lo) * C::DQK;
  const __bf16* Kh = p.K + (((int64_t)b * p.H_qk + hqk) * Lt + row_lo) * C::DQK;
  const __bf16* Vh = p.V + (((int64_t)b * p.H_v + h / (p.H / p.H_v)) * Lt + row_lo) * C::DV;
  const float* lah = p.log_decay ? p.log_decay + (int64_t)bh * Lt + row_lo : nullptr;
  const float la_const = lah ? 0.f : dt.log2_gamma[h] * 0.6931471805599453f;  // constant decay per head: ln gamma
  const float* gh = p.key_gate ? p.key_gate + (int64_t)bh * Lt + row_lo : nullptr;
  const int64_t slot = (int64_t)bh * p.nseg + seg;  // of this segment's states
  const uint32_t raw0 = lds0 + C::STAGES * C::STAGE_BYTES + hw * C::RAW_BYTES;  // the head's raw gates, stage 0
  const uint32_t gate0 = lds0 + C::STAGES * (C::STAGE_BYTES + C::HPW * C::RAW_BYTES) + wave * C::GATE_BYTES;  // this wave's b[64], g[64], w[64]
  const uint32_t scrap0 = lds0 + C::LDS_BYTES - 256;

  // ---- the state slab of this wavefront: rows d, columns 32 * wave .. + 31 ----
  f32x16 H[C::DBQ];
#pragma unroll
  for (int db = 0; db < C::DBQ; ++db) {
    if (p.h_in) {
      const float* src = p.h_in + slot * C::DQK * C::DV + 32 * vblk + ln;
#pragma unroll
      for (int r = 0; r < 16; ++r) H[db][r] = src[(int64_t)(32 * db + key_offset(r) + 4 * half) * C::DV];
    } else {
      H[db] = zero16();
    }
    pin(H[db]);  // (the loads of the initial state are awaited here, not by a wait inside the loop)
  }

  // ---- copies: chunk c -> stage c % 3 ----
  // Per copy instruction of this wave the lane's byte offset inside a chunk is fixed (row r of the tile, chunk slot
  // with the tile's swizzle); the chunk's first row moves the wave-uniform base pointer.  The last chunk, if short,
  // takes the offsets with its rows clamped to the last token (their gates are zero).
  constexpr int NQ = C::CPRQ / C::WAVES, NV = C::CPRV / C::WPH;
  uint32_t qoff[NQ], voff[NV];  // whole chunks: the lane's byte offsets from the chunk's first row (Q and K tiles alike)
  auto lane_off = [&](auto cprc, int nb, int t0, bool whole) {
    constexpr int CPR = decltype(cprc)::value;
    const int pos = nb * 64 + lane, r = pos / CPR, pc = pos % CPR;
    int row = whole ? r : min(r, (int)L - 1 - t0);
    // walking backwards, tile row r is the token r in front of the chunk's first one, and the base pointer stands at
    // the chunk's lowest address: its last row (row 63 of a whole chunk, token 0 of a short one)
    if (rev) row = (whole ? C::CH - 1 : (int)L - 1 - t0) - row;
    return (uint32_t)((row * (CPR * 8) + ((pc ^ bswz<CPR>(r)) * 8)) * 2);
  };
  uint32_t qoff_t[NQ], voff_t[NV];  // the same for the last chunk, if it is short
  const int n_chunks = (int)((L + C::CH - 1) / C::CH);
  const int t0_last = (n_chunks - 1) * C::CH;
#pragma unroll
  for (int i = 0; i < NQ; ++i) {
    qoff[i] = lane_off(std::integral_constant<int, C::CPRQ>{}, wave + i * C::WAVES, 0, true);
    qoff_t[i] = lane_off(std::integral_constant<int, C::CPRQ>{}, wave + i * C::WAVES, t0_last, false);
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    voff[i] = lane_off(std::integral_constant<int, C::CPRV>{}, wh + i * C::WPH, 0, true);
    voff_t[i] = lane_off(std::integral_constant<int, C::CPRV>{}, wh + i * C::WPH, t0_last, false);
  }
  auto issue_chunk = [&](int c) {
    const int t0 = c * C::CH;
    const bool whole = t0 + C::CH <= L;
    const uint32_t base = lds0 + (c % C::STAGES) * C::STAGE_BYTES;
    const int64_t r0 = rev ? max((int)L - C::CH - t0, 0) : t0;  // the chunk's row with the lowest address
    const __bf16 *qc = Qh + r0 * C::DQK, *kc = Kh + r0 * C::DQK, *vc = Vh + r0 * C::DV;
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const int nb = wave + i * C::WAVES;
      const uint32_t off = whole ? qoff[i] : qoff_t[i];  // (only the last chunk can be short)
      dma16(qc, off, base + nb * 1024);
      dma16(kc, off, base + C::Q_BYTES + nb * 1024);
    }
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int nb = wh + i * C::WPH;
      const uint32_t off = whole ? voff[i] : voff_t[i];
      dma16(vc, off, base + 2 * C::Q_BYTES + hw * C::V_BYTES + nb * 1024);
    }
    // the head's gates, one token per lane: its first wave fetches the log-decays, its second the key gates; the
    // others (and a row that does not exist: constant decay, no key gate) fetch a word they never look at, so that
    // every wave issues the same number of copies
    const float* grow = wh == 0 && lah ? lah : wh == 1 && gh ? gh : nullptr;
    const uint32_t gdst = raw0 + (c % C::STAGES) * (C::HPW * C::RAW_BYTES) + (wh == 1 ? 256 : 0);
    // walking backwards: the decay of the token one later in the sequence (the walk's first token has none: its
    // word is replaced by 0 where it is read), the gate of the token itself
    // (cut into segments, the first token of a later segment does have a successor: the word behind the segment)
    int gi = min(t0 + lane, (int)L - 1);
    if (rev) gi = wh == 0 ? min((int)L - gi, first > 0 ? (int)L : (int)L - 1) : (int)L - 1 - gi;
    const uint32_t goff = grow ? (uint32_t)gi * 4u : 0u;
    dma4(grow ? (const void*)grow : (const void*)Qh, goff, grow ? gdst : scrap0);
  };

  // Per-lane parts of the fragment addresses, relative to a stage (see attn_bwd_kernel.hpp for the two read patterns
  // of a tile).  Whatever depends on the lane sits in these registers; the stage adds one uniform offset per chunk
  // (below), and tile, row block and token step are compile-time offsets that the LDS instructions carry themselves.
  const int li = lane & 15, blk = (lane >> 4) & 1;
  const int trow = 4 * half + (li >> 2), tcl = 2 * blk + ((li & 3) >> 1);
  // row fragment of Q or K for d-step t (d = 16 t + 4 half + {0..3} and + 8), row ln of a 32-row block: two 8-byte pieces
  uint32_t rq0[C::T][2];
#pragma unroll
  for (int t = 0; t < C::T; ++t)
#pragma unroll
    for (int j = 0; j < 2; ++j) rq0[t][j] = ln * C::RBQ + 8 * half + (((2 * t + j) ^ bswz<C::CPRQ>(ln)) << 4);
  // transposed fragment: 32 columns of block k, rows trow and trow + 8 of a 16-token step (lane = column, registers =
  // rows in accumulator order)
  auto tr_lane = [&](auto cprc, int k, int j) {
    constexpr int CPR = decltype(cprc)::value, RB = CPR * 16;
    const int r = trow + 8 * j;
    return (uint32_t)((li & 1) * 8 + r * RB + (((4 * k + tcl) ^ bswz<CPR>(r)) << 4));
  };
  uint32_t kt0[C::DBQ][2], vt0[2];
#pragma unroll
  for (int k = 0; k < C::DBQ; ++k)
#pragma unroll
    for (int j = 0; j < 2; ++j) kt0[k][j] = C::Q_BYTES + tr_lane(std::integral_constant<int, C::CPRQ>{}, k, j);
#pragma unroll
  for (int j = 0; j < 2; ++j) vt0[j] = 2 * C::Q_BYTES + hw * C::V_BYTES + tr_lane(std::integral_constant<int, C::CPRV>{}, vblk, j);

  float seg_b = 0.f;  // sum of the log-decays walked so far
  issue_chunk(0);
  if (n_chunks > 1) issue_chunk(1);

  for (int c = 0; c < n_chunks; ++c) {
    const int t0 = c * C::CH;
    // this chunk's fragment addresses: the lane parts plus the stage
    uint32_t rq[C::T][2], kt[C::DBQ][2], vt[2];
    {
      const uint32_t sb = lds0 + (c % C::STAGES) * C::STAGE_BYTES;
#pragma unroll
      for (int t = 0; t < C::T; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          rq[t][j] = rq0[t][j] + sb;
          pin(rq[t][j]);
        }
#pragma unroll
      for (int k = 0; k < C::DBQ; ++k)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          kt[k][j] = kt0[k][j] + sb;
          pin(kt[k][j]);
        }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        vt[j] = vt0[j] + sb;
        pin(vt[j]);
      }
    }
    // rows row0 + ln of the Q tile (tile 0) or the K tile (tile 1), d-step t
    auto row_frag = [&](int tile, int row0, int t) {
      const uint32_t o = tile * C::Q_BYTES + row0 * C::RBQ;
      const u32x2 lo = lds_read8(rq[t][0] + o), hi = lds_read8(rq[t][1] + o);
      return __builtin_bit_cast(bf16x8, (u32x4){lo[0], lo[1], hi[0], hi[1]});
    };
    auto k_tr_frag = [&](int k, int s) { return read_tr_frag(kt[k][0] + 16 * s * C::RBQ, kt[k][1] + 16 * s * C::RBQ); };
    auto v_tr_frag = [&](int s) { return read_tr_frag(vt[0] + 16 * s * C::RBV, vt[1] + 16 * s * C::RBV); };
    // Chunk c has landed: of this wave's memory operations only those issued after its copies may still be in
    // flight -- the copies of chunk c + 1 (if there is one) and the stores of chunk c - 1 (if there was one; it was
    // a whole chunk: four stores).  The counter runs in issue order.  Then the barrier: everybody's copies have
    // landed and every wave is done with chunk c - 1, whose stage chunk c + 2 may now overwrite.
    {
      const bool nxt = c + 1 < n_chunks, prv = c > 0;
      const bool st = prv && !p.state_only;  // (a walk that only updates the state stores nothing)
      if (nxt && st) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::NDMA + C::NST) : "memory");
      else if (nxt) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::NDMA) : "memory");
      else if (st) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(C::NST) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      asm volatile("s_barrier" ::: "memory");
    }
    // The copies of chunk c + 2 (its stage is free from the barrier on).  The compute unit's memory pipe takes 64
    // bytes per clock, a chunk's tiles are 48 KB: if all wavefronts queued their copies here, they would wait for the
    // pipe and for each other.  Each issues its share at a different point of the iteration instead (the counts
    // in the waits above do not care in which order a wavefront's copies and stores were issued: both are younger
    // than the copies it waits for).
    const bool more = c + 2 < n_chunks;
    const int turn = wave & 3;
    if (more && turn == 0) issue_chunk(c + 2);
    // gates of this lane's token: log-decay (0 past the end: the state is carried unchanged; at least -20: a token
    // that lets less than e^-20 through lets nothing through at the precision of the path, and the bound keeps the
    // factorised weights below in range) and key gate (0 past the end)
    float la = 0.f, g = 0.f;
    if (t0 + lane < L) {
      const uint32_t raw = raw0 + (c % C::STAGES) * (C::HPW * C::RAW_BYTES) + lane * 4;
      la = lah ? fmaxf(*reinterpret_cast<__attribute__((address_space(3))) const float*>((lds_char*)(uintptr_t)raw), -20.f) : la_const;
      g = gh ? *reinterpret_cast<__attribute__((address_space(3))) const float*>((lds_char*)(uintptr_t)(raw + 256)) : 1.f;
      if (rev && t0 + lane == 0 && first == 0) la = lah ? 0.f : la;  // (a constant decay is the same for every token: nothing to shift)
    }
    // the gate as a factor on the output rows instead of the keys: the two query tokens of this lane
    float og0 = 1.f, og1 = 1.f;
    if (p.gate_on_output) {
      swap_halves(g, og0, og1);
      g = t0 + lane < L ? 1.f : 0.f;
    }

    // ---- gates: b = inclusive prefix sum of the log-decays over the chunk's 64 tokens (lane = token) ----
    // (data-parallel-primitive steps: within rows of 16 lanes by shifts of 1, 2, 4, 8, then the row totals onward)
    float bcum = la;
    bcum += dpp_f<0x111, 0xf, 0xf>(bcum);
    bcum += dpp_f<0x112, 0xf, 0xf>(bcum);
    bcum += dpp_f<0x114, 0xf, 0xe>(bcum);
    bcum += dpp_f<0x118, 0xf, 0xc>(bcum);
    bcum += dpp_f<0x142, 0xa, 0xf>(bcum);
    bcum += dpp_f<0x143, 0xc, 0xf>(bcum);
    const float b_last = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, bcum), 63));
    // Weights inside the chunk, factorised per group of four tokens: with ref_j the sum in front of token j's group
    // (ref_j >= b_i for every i in or behind the group),  e^{b_i - b_j} g_j = e^{b_i - ref_j} * u_j,
    // u_j = g_j e^{ref_j - b_j}: one exponential per token here and four per lane and block of keys below instead of
    // one per score.  ref_j - b_j is at most four log-decays: with the bound of 20 above u_j stays finite.
    {
      const float ref = dpp_f<0x00, 0xf, 0xf>(bcum - la);  // the sum in front of lane (lane & ~3): quad broadcast of the exclusive sum
      lds_write4(gate0 + lane * 4, ref);
      lds_write4(gate0 + 256 + lane * 4, g * __expf(ref - bcum));
      lds_write4(gate0 + 512 + lane * 4, g * __expf(b_last - bcum));
    }
    if (more && turn == 1) issue_chunk(c + 2);
    float bi0, bi1;  // b of tokens ln and 32 + ln
    swap_halves(bcum, bi0, bi1);
    // The state in front of the chunk, rounded to bf16: the A operands of the read-out (an accumulator tile is an A
    // operand whose contraction runs over its rows).  In the same pass over the accumulators the state takes the
    // chunk's whole decay, as the update at the end of the iteration needs it.
    bf16x8 hp[C::DBQ][2];
    {
      const float dec = __expf(b_last);
#pragma unroll
      for (int db = 0; db < C::DBQ; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float x = H[db][r];
          hp[db][r / 8][r % 8] = (__bf16)x;
          H[db][r] = x * dec;
        }
    }
    bf16x8 vf[4];  // the V fragments of the chunk's four 16-token steps (this wave's 32 value columns)
    // The wave's query block as a compile-time constant (register arrays indexed by it stay in registers).
    auto query_block = [&](auto ibc) {
    constexpr int IB = decltype(ibc)::value;
    const float bi = IB ? bi1 : bi0;  // of this lane's query: token 32 IB + ln of the chunk
    const float og = IB ? og1 : og0;
    // ---- Q fragments of the wave's query block (B operands of S^T and of the read-out) ----
    bf16x8 qf[C::T];
#pragma unroll
    for (int t = 0; t < C::T; ++t) qf[t] = row_frag(0, 32 * IB, t);

    // ---- read-out of the state in front of the chunk: O^T = H^T Q^T, times scale e^{b_i} ----
    f32x16 o = zero16();
#pragma unroll
    for (int db = 0; db < C::DBQ; ++db)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) o = mfma(hp[db][tt], qf[2 * db + tt], o);
    {
      const float f = p.scale * __expf(bi);
#pragma unroll
      for (int r = 0; r < 16; ++r) o[r] *= f;
    }

    // weights of one S^T block: scale e^{b_i - b_j} g_j s for key j <= query i (positions inside the chunk), else 0
    auto weigh = [&](const f32x16& s, int kblk, bool diag, u32x4 (&pk)[2]) {
      float ref[4];
      f32x4 uj[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) {  // (all eight reads first: one LDS latency for the block, not four)
        const uint32_t off = (32 * kblk + 8 * a + 4 * half) * 4;
        ref[a] = *reinterpret_cast<__attribute__((address_space(3))) const float*>((lds_char*)(uintptr_t)(gate0 + off));
        uj[a] = lds_read16(gate0 + 256 + off);
      }
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        // (groups past the lane's query have bi > ref: whatever the factor becomes there, the mask below discards it)
        const float qfac = p.scale * __expf(bi - ref[a]);
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          x[e] = s[4 * a + e] * (qfac * uj[a][e]);
          if (diag && 8 * a + 4 * half + e > ln) x[e] = 0.f;
        }
        bf16x2 lo, hi;
        lo[0] = (__bf16)x[0];
        lo[1] = (__bf16)x[1];
        hi[0] = (__bf16)x[2];
        hi[1] = (__bf16)x[3];
        pk[a / 2][2 * (a % 2)] = __builtin_bit_cast(uint32_t, lo);
        pk[a / 2][2 * (a % 2) + 1] = __builtin_bit_cast(uint32_t, hi);
      }
    };
    // ---- scores and aggregation inside the chunk: the diagonal block of the wave's queries, and for the second
    //      query block also the block below the diagonal (keys 0-31) ----
    {
      f32x16 sd = zero16();
#pragma unroll
      for (int t = 0; t < C::T; ++t) sd = mfma(row_frag(1, 32 * IB, t), qf[t], sd);
      u32x4 pd[2];
      weigh(sd, IB, true, pd);
      // the V fragments of the chunk's four 16-token steps (this wave's 32 value columns): A operands of the
      // aggregation and, weighted, B operands of the state update
      if constexpr (IB == 0 || C::QS == 2) {
#pragma unroll
        for (int s = 0; s < 4; ++s) vf[s] = v_tr_frag(s);
      }
      o = mfma(vf[2 * IB], __builtin_bit_cast(bf16x8, pd[0]), o);
      o = mfma(vf[2 * IB + 1], __builtin_bit_cast(bf16x8, pd[1]), o);
    }
    if constexpr (IB == 1) {
      f32x16 sl = zero16();
#pragma unroll
      for (int t = 0; t < C::T; ++t) sl = mfma(row_frag(1, 0, t), qf[t], sl);
      u32x4 pl[2];
      weigh(sl, 0, false, pl);
      o = mfma(vf[0], __builtin_bit_cast(bf16x8, pl[0]), o);
      o = mfma(vf[1], __builtin_bit_cast(bf16x8, pl[1]), o);
    }

    // ---- store: lane = query row, four 16-byte pieces of the wave's 32 columns ----
    {
      const int64_t i = t0 + 32 * IB + ln;
      if (i < L) {
        if (p.gate_on_output) {
#pragma unroll
          for (int r = 0; r < 16; ++r) o[r] *= og;
        }
        const int64_t e0 = ((int64_t)bh * Lt + row_lo + (rev ? L - 1 - i : i)) * C::DV + 32 * vblk + 4 * half;
        if (p.out_bf16) {
#pragma unroll
          for (int a = 0; a < 4; ++a) {
            bf16x4 hv;
#pragma unroll
            for (int e = 0; e < 4; ++e) hv[e] = (__bf16)o[4 * a + e];
            *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.O) + e0 + 8 * a) = hv;
          }
        } else {
#pragma unroll
          for (int a = 0; a < 4; ++a)
            *reinterpret_cast<f32x4*>(static_cast<float*>(p.O) + e0 + 8 * a) = (f32x4){o[4 * a], o[4 * a + 1], o[4 * a + 2], o[4 * a + 3]};
        }
      }
    }

    };
    if (!p.state_only) {
      if (C::QS == 1 || ib == 0) query_block(std::integral_constant<int, 0>{});
      if (more && turn == 2) issue_chunk(c + 2);
      if (C::QS == 1 || ib == 1) query_block(std::integral_constant<int, 1>{});
    } else {
      if (more && turn == 2) issue_chunk(c + 2);
      // (the V fragments that a query block would have left behind for the update)
#pragma unroll
      for (int s = 0; s < 4; ++s) vf[s] = v_tr_frag(s);
    }
    seg_b += b_last;
    if (more && turn == 3) issue_chunk(c + 2);

    // ---- state update: H (already e^{b_last} times the old state) += K^T (w . V) ----
    f32x4 wv[8];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      wv[2 * s] = lds_read16(gate0 + 512 + (16 * s + 4 * half) * 4);
      wv[2 * s + 1] = lds_read16(gate0 + 512 + (16 * s + 8 + 4 * half) * 4);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      // the V fragment of token step s times the tokens' weights (element e of the fragment: token 16 s + 8 (e / 4) + 4 half + e % 4)
      bf16x8 vw;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        vw[e] = (__bf16)((float)vf[s][e] * wv[2 * s][e]);
        vw[4 + e] = (__bf16)((float)vf[s][4 + e] * wv[2 * s + 1][e]);
      }
#pragma unroll
      for (int db = 0; db < C::DBQ; ++db)
        H[db] = mfma(k_tr_frag(db, s), vw, H[db]);
    }
  }

  if (p.seg_decay && wh == 0 && lane == 0) p.seg_decay[slot] = seg_b;
  if (p.h_out && ib == 0 && (!p.h_out_last_only || seg == p.nseg - 1)) {  // (the slab's other copy is identical)
    float* dst = p.h_out + (p.h_out_last_only ? (int64_t)bh : slot) * C::DQK * C::DV + 32 * vblk + ln;
#pragma unroll
    for (int db = 0; db < C::DBQ; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[(int64_t)(32 * db + key_offset(r) + 4 * half) * C::DV] = H[db][r];
  }
}

template <int DQK, int DV, int HPW = 1, int QS = 2>
hipError_t launch(const GatedParams& p, const DecayTable& dt, hipStream_t s) {
  typedef GCfg<DQK, DV, HPW, QS> C;
  hipLaunchKernelGGL(gated_recurrent_kernel<C>, dim3((unsigned)(p.B * p.H / HPW * p.nseg)), dim3(C::THREADS), 0, s, p, dt);
  return hipGetLastError();
}

// ---- segments: from the final states of the segments (each from a zero start) to the states in front of them ----
__global__ __launch_bounds__(256) void gated_combine_segments_kernel(float* buf, const float* seg_decay, const float* h_in, int nseg,
                                                                      int state_elems) {
  const int64_t bh = blockIdx.y;
  const int e = blockIdx.x * 256 + threadIdx.x;
  if (e >= state_elems) return;
  float x = h_in ? h_in[bh * state_elems + e] : 0.f;
  for (int s = 0; s < nseg; ++s) {
    float* slot = buf + (bh * nseg + s) * state_elems + e;
    const float local = *slot;
    *slot = x;
    x = __expf(seg_decay[bh * nseg + s]) * x + local;
  }
}

// ---- epilogue of the backward pass ----
// A group of DQK / 4 lanes owns a token (16 bytes of an fp32 row, 8 of a bf16 row, per lane); a wavefront takes
// 64 / (DQK / 4) tokens of one (batch, q/k head) at a time and loops over the value heads of the group.
template <int DQK>
__global__ __launch_bounds__(256) void gated_bwd_rows_kernel(const GatedBwdEpilogueParams p) {
  constexpr int LPR = DQK / 4, TPW = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane % LPR;
  const int grp = p.H / p.H_qk;
  const int64_t blocks_per_head = ((int64_t)p.L + 4 * TPW - 1) / (4 * TPW);
  const int64_t bhq = blockIdx.x / blocks_per_head;  // (batch, q/k head)
  const int64_t t = (blockIdx.x % blocks_per_head) * (4 * TPW) + (threadIdx.x >> 6) * TPW + lane / LPR;
  const bool live = t < p.L;
  const int64_t tc = live ? t : p.L - 1;
  const int b = (int)(bhq / p.H_qk), hq = (int)(bhq % p.H_qk);
  const int64_t qrow = (bhq * p.L + tc) * DQK + 4 * sub;
  const bf16x4 q4 = *reinterpret_cast<const bf16x4*>(p.Q + qrow), k4 = *reinterpret_cast<const bf16x4*>(p.K + qrow);
  f32x4 dq = {0.f, 0.f, 0.f, 0.f}, dk = {0.f, 0.f, 0.f, 0.f};
  for (int j = 0; j < grp; ++j) {
    const int64_t bh = (int64_t)b * p.H + (int64_t)hq * grp + j;
    const int64_t row = (bh * p.L + tc) * DQK + 4 * sub;
    const f32x4 u = *reinterpret_cast<const f32x4*>(p.dQu + row), x = *reinterpret_cast<const f32x4*>(p.X + row);
    const float g = p.key_gate ? p.key_gate[bh * p.L + tc] : 1.f;
    float qd = 0.f, kx = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      qd += (float)q4[e] * u[e];
      kx += (float)k4[e] * x[e];
      dq[e] += u[e];
      dk[e] += g * x[e];
    }
#pragma unroll
    for (int s = LPR / 2; s >= 1; s >>= 1) {
      qd += __shfl_xor(qd, s);
      kx += __shfl_xor(kx, s);
    }
    if (live && sub == 0) {
      p.dB[bh * p.L + t] = qd - g * kx;
      if (p.dkey_gate) p.dkey_gate[bh * p.L + t] = kx;
    }
  }
  if (live) {
    // (where dQu is dQ itself the values are already in place; dK is rewritten only if something changed it)
    if (p.dQu != p.dQ) *reinterpret_cast<f32x4*>(p.dQ + qrow) = dq;
    if (p.X != p.dK || p.key_gate) *reinterpret_cast<f32x4*>(p.dK + qrow) = dk;
  }
}

// dlog_decay[t] = sum_{i >= t} dB[i]: one wavefront per (batch, head) walks from the end in blocks of 256 tokens,
// four per lane; the running total is kept in double (the terms change sign and the sum is long).
__global__ __launch_bounds__(64) void gated_bwd_suffix_sum_kernel(const GatedBwdEpilogueParams p) {
  const int lane = threadIdx.x;
  const float* src = p.dB + (int64_t)blockIdx.x * p.L;
  float* dst = p.dlog_decay + (int64_t)blockIdx.x * p.L;
  double carry = 0.0;
  const int nblk = (p.L + 255) / 256;
  for (int blk = nblk - 1; blk >= 0; --blk) {
    const int t0 = blk * 256 + 4 * lane;
    float x[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = t0 + e < p.L ? src[t0 + e] : 0.f;
    // suffix sums inside the lane, then over the lanes behind this one
    x[2] += x[3];
    x[1] += x[2];
    x[0] += x[1];
    float tot = x[0];  // inclusive suffix sum over lanes: lane l gets the sum of the totals of lanes >= l
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      const float o = __shfl_down(tot, s);
      if (lane + s < 64) tot += o;
    }
    const float behind = tot - x[0];  // the lanes strictly behind
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (t0 + e < p.L) dst[t0 + e] = (float)(carry + (double)(x[e] + behind));
    carry += (double)__shfl(tot, 0);
  }
}

}  // namespace

hipError_t launch_gated_combine_segments(float* buf, const float* seg_decay, const float* h_in, int BH, int nseg, int state_elems,
                                         hipStream_t s) {
  if (BH < 1 || BH > 65535 || nseg < 1 || state_elems < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gated_combine_segments_kernel, dim3((unsigned)((state_elems + 255) / 256), (unsigned)BH), dim3(256), 0, s, buf,
                     seg_decay, h_in, nseg, state_elems);
  return hipGetLastError();
}

hipError_t launch_gated_backward_epilogue(const GatedBwdEpilogueParams& p, int dqk, hipStream_t s) {
  const int tpb = 4 * (64 / (dqk / 4));
  const int64_t grid = (int64_t)p.B * p.H_qk * (((int64_t)p.L + tpb - 1) / tpb);
  if (grid > 0x7fffffffLL || (dqk != 64 && dqk != 128)) return hipErrorInvalidValue;
  if (dqk == 64) hipLaunchKernelGGL(gated_bwd_rows_kernel<64>, dim3((unsigned)grid), dim3(256), 0, s, p);
  else hipLaunchKernelGGL(gated_bwd_rows_kernel<128>, dim3((unsigned)grid), dim3(256), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(gated_bwd_suffix_sum_kernel, dim3((unsigned)(p.B * p.H)), dim3(64), 0, s, p);
  return hipGetLastError();
}

bool gated_supported(int dqk, int dv) { return (dqk == 64 || dqk == 128) && (dv == 64 || dv == 128); }

hipError_t launch_gated_recurrent(const GatedParams& p_in, const DecayTable& dt, int dqk, int dv, hipStream_t s) {
  GatedParams p = p_in;
  if (p.H_v == 0) p.H_v = p.H;
  if (p.H_qk < 1 || p.H % p.H_qk != 0 || p.H % p.H_v != 0) return hipErrorInvalidValue;
  if (p.nseg < 1 || (p.nseg > 1 && (p.seg_len < 64 || p.seg_len % 64 != 0 || (int64_t)(p.nseg - 1) * p.seg_len >= p.L)))
    return hipErrorInvalidValue;
  if ((int64_t)p.B * p.H * p.nseg > 0x7fffffffLL) return hipErrorInvalidValue;
  if (dqk == 64 && dv == 64) return launch<64, 64>(p, dt, s);
  if (dqk == 128 && dv == 64) {
    // value heads that share their q/k head (Mamba2's groups) share the Q and K tiles of a workgroup, two at a time
    const int grp = p.H / p.H_qk;
    if (grp % 2 == 0 && p.H_v == p.H) return launch<128, 64, 2, 1>(p, dt, s);
    return launch<128, 64>(p, dt, s);
  }
  if (dqk == 64 && dv == 128) return launch<64, 128>(p, dt, s);
  if (dqk == 128 && dv == 128) return launch<128, 128, 1, AE_GATED_QS_128>(p, dt, s);
  return hipErrorInvalidValue;
}

}  // namespace ae
