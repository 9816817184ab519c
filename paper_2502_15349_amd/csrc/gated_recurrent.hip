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
// A wavefront owns 32 of the D_v output columns (D_v / 32 wavefronts per workgroup) and, for them, the state slab
// [D_qk x 32] as D_qk / 32 accumulator tiles.  All products are transposed so that a lane owns one column -- a
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
// The three 32 x 32 blocks of S^T that the causal order inside a chunk leaves are computed by every wavefront
// itself (cheaper than an exchange through LDS and a barrier: the path is bound by memory, not by the MFMAs).
// Q, K, V tiles arrive by LDS-DMA, double buffered, one barrier per chunk; the gates of the next chunk are
// fetched a chunk ahead.  The output of a chunk is stored before the state update, whose MFMAs cover the stores.
#include <hip/hip_runtime.h>

#include "attn_bwd_kernel.hpp"  // bswz, read_tr_frag
#include "gated.hpp"

namespace ae {
namespace {

// HPW_: value heads per workgroup.  Heads of one q/k group (Mamba2: every head of a group reads the same B and C)
// can share the Q and K tiles of a workgroup: HPW_ consecutive heads, each with its own V tile, gates and state.
template <int DQK_, int DV_, int HPW_ = 1>
struct GCfg {
  static constexpr int DQK = DQK_, DV = DV_, HPW = HPW_, WPH = DV_ / 32, WAVES = HPW_ * WPH, THREADS = 64 * WAVES, CH = 64;
  static constexpr int RBQ = DQK * 2, RBV = DV * 2, CPRQ = DQK / 8, CPRV = DV / 8;
  static constexpr int Q_BYTES = CH * RBQ, V_BYTES = CH * RBV, STAGE_BYTES = 2 * Q_BYTES + HPW * V_BYTES;
  static constexpr int GATE_BYTES = 3 * CH * 4;  // per wavefront: b, g, w of the chunk's tokens
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES + WAVES * GATE_BYTES;
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
  // workgroup -> batch entry and HPW consecutive value heads of one q/k group; wave -> (head, 32 value columns)
  const int hw = wave / C::WPH, vblk = wave % C::WPH;
  const int bh0 = blockIdx.x * C::HPW, b = bh0 / p.H, h = bh0 % p.H + hw, bh = bh0 + hw;
  const int hqk = h / (p.H / p.H_qk);
  const int64_t L = p.L;
  const __bf16* Qh = p.Q + ((int64_t)b * p.H_qk + hqk) * L * C::DQK;
  const __bf16* Kh = p.K + ((int64_t)b * p.H_qk + hqk) * L * C::DQK;
  const __bf16* Vh = p.V + (int64_t)bh * L * C::DV;
  const float* lah = p.log_decay ? p.log_decay + (int64_t)bh * L : nullptr;
  const float la_const = lah ? 0.f : dt.log2_gamma[h] * 0.6931471805599453f;  // constant decay per head: ln gamma
  const float* gh = p.key_gate ? p.key_gate + (int64_t)bh * L : nullptr;
  const uint32_t gate0 = lds0 + 2 * C::STAGE_BYTES + wave * C::GATE_BYTES;  // this wave's b[64], g[64], w[64]

  // ---- the state slab of this wavefront: rows d, columns 32 * wave .. + 31 ----
  f32x16 H[C::DBQ];
#pragma unroll
  for (int db = 0; db < C::DBQ; ++db) {
    if (p.h_in) {
      const float* src = p.h_in + (int64_t)bh * C::DQK * C::DV + 32 * vblk + ln;
#pragma unroll
      for (int r = 0; r < 16; ++r) H[db][r] = src[(int64_t)(32 * db + key_offset(r) + 4 * half) * C::DV];
    } else {
      H[db] = zero16();
    }
  }

  // ---- copies: chunk c -> stage c % 2 (rows past the end repeat the last row; their gates are zero) ----
  auto issue_chunk = [&](int c) {
    const int t0 = c * C::CH;
    const uint32_t base = lds0 + (c & 1) * C::STAGE_BYTES;
    auto tile = [&](const __bf16* src, auto cprc, uint32_t dst, auto nwc, int w) {
      constexpr int CPR = decltype(cprc)::value, NW = decltype(nwc)::value;  // copied by NW waves, this one being number w
#pragma unroll
      for (int i = 0; i < CPR / NW; ++i) {
        const int nb = w + i * NW, pos = nb * 64 + lane;
        const int r = pos / CPR, pc = pos % CPR;
        const int row = min(t0 + r, (int)L - 1);
        dma16(src, (uint32_t)((row * (CPR * 8) + ((pc ^ bswz<CPR>(r)) * 8)) * 2), dst + nb * 1024);
      }
    };
    tile(Qh, std::integral_constant<int, C::CPRQ>{}, base, std::integral_constant<int, C::WAVES>{}, wave);
    tile(Kh, std::integral_constant<int, C::CPRQ>{}, base + C::Q_BYTES, std::integral_constant<int, C::WAVES>{}, wave);
    tile(Vh, std::integral_constant<int, C::CPRV>{}, base + 2 * C::Q_BYTES + hw * C::V_BYTES, std::integral_constant<int, C::WPH>{}, vblk);
  };
  // gates of chunk c for token lane: log-decay (0 past the end: the state is carried unchanged) and key gate (0 past the end)
  auto load_gates = [&](int c, float& la, float& g) {
    const int t = c * C::CH + lane;
    la = 0.f;
    g = 0.f;
    if (t < L) {
      la = lah ? lah[t] : la_const;
      g = gh ? gh[t] : 1.f;
    }
  };

  // per-lane pieces of the fragment addresses (stage 0; see attn_bwd_kernel.hpp for the two read patterns of a tile)
  const int fq = bswz<C::CPRQ>(ln);
  const int li = lane & 15, blk = (lane >> 4) & 1;
  const int trow = 4 * half + (li >> 2), tcl = 2 * blk + ((li & 3) >> 1);
  // row fragment of Q or K for d-step t, rows `row0 + ln` of the tile at `tb`: d = 16 t + 4 half + {0..3} and + 8
  auto row_frag = [&](uint32_t tb, int row0, int t) {
    const uint32_t a = tb + (row0 + ln) * C::RBQ + 8 * half;
    const u32x2 lo = lds_read8(a + (((2 * t) ^ fq) << 4)), hi = lds_read8(a + (((2 * t + 1) ^ fq) << 4));
    return __builtin_bit_cast(bf16x8, (u32x4){lo[0], lo[1], hi[0], hi[1]});
  };
  // transposed fragment: 32 columns of block k, 16 rows of step s (lane = column, registers = rows in accumulator order)
  auto tr_frag = [&](uint32_t tb, auto cprc, int k, int s) {
    constexpr int CPR = decltype(cprc)::value, RB = CPR * 16;
    const int rlo = 16 * s + trow, rhi = rlo + 8;
    const uint32_t alo = tb + (li & 1) * 8 + rlo * RB + (((4 * k + tcl) ^ bswz<CPR>(rlo)) << 4);
    const uint32_t ahi = tb + (li & 1) * 8 + rhi * RB + (((4 * k + tcl) ^ bswz<CPR>(rhi)) << 4);
    return read_tr_frag(alo, ahi);
  };

  const int n_chunks = (int)((L + C::CH - 1) / C::CH);
  float la_next, g_next;
  issue_chunk(0);
  load_gates(0, la_next, g_next);

  for (int c = 0; c < n_chunks; ++c) {
    const int t0 = c * C::CH;
    const uint32_t sb = lds0 + (c & 1) * C::STAGE_BYTES;
    const uint32_t qb = sb, kb_ = sb + C::Q_BYTES, vb_ = sb + 2 * C::Q_BYTES + hw * C::V_BYTES;
    const float la = la_next, g = g_next;
    // chunk c has landed (this wave's copies; the barrier: everybody's), and every wave is done with chunk c - 1
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
    if (c + 1 < n_chunks) {
      issue_chunk(c + 1);
      load_gates(c + 1, la_next, g_next);
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
    lds_write4(gate0 + lane * 4, bcum);
    lds_write4(gate0 + 256 + lane * 4, g);
    lds_write4(gate0 + 512 + lane * 4, __expf(b_last - bcum) * g);
    float bi0, bi1;  // of this lane's two queries: tokens ln and 32 + ln
    swap_halves(bcum, bi0, bi1);

    // ---- Q fragments of both query blocks (B operands of S^T and of the read-out) ----
    bf16x8 qf[2][C::T];
#pragma unroll
    for (int ib = 0; ib < 2; ++ib)
#pragma unroll
      for (int t = 0; t < C::T; ++t) qf[ib][t] = row_frag(qb, 32 * ib, t);

    // ---- read-out of the state in front of the chunk: O^T = H^T Q^T, times scale e^{b_i} ----
    f32x16 o[2] = {zero16(), zero16()};
#pragma unroll
    for (int db = 0; db < C::DBQ; ++db)
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        bf16x8 hfrag;
#pragma unroll
        for (int e = 0; e < 8; ++e) hfrag[e] = (__bf16)H[db][8 * tt + e];
        o[0] = mfma(hfrag, qf[0][2 * db + tt], o[0]);
        o[1] = mfma(hfrag, qf[1][2 * db + tt], o[1]);
      }
    {
      const float f0 = p.scale * __expf(bi0), f1 = p.scale * __expf(bi1);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        o[0][r] *= f0;
        o[1][r] *= f1;
      }
    }

    // ---- scores inside the chunk: S^T blocks (keys 0-31 | queries 0-31), (0-31 | 32-63), (32-63 | 32-63) ----
    f32x16 s00 = zero16(), s01 = zero16(), s11 = zero16();
#pragma unroll
    for (int t = 0; t < C::T; ++t) {
      const bf16x8 k0 = row_frag(kb_, 0, t), k1 = row_frag(kb_, 32, t);
      s00 = mfma(k0, qf[0][t], s00);
      s01 = mfma(k0, qf[1][t], s01);
      s11 = mfma(k1, qf[1][t], s11);
    }
    // weights: scale e^{b_i - b_j} g_j s for key j <= query i (positions inside the chunk), else 0
    u32x4 p00[2], p01[2], p11[2];
    auto weigh = [&](const f32x16& s, int kblk, float bi, int iq, bool diag, u32x4 (&pk)[2]) {
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const uint32_t off = (32 * kblk + 8 * a + 4 * half) * 4;
        const f32x4 bj = lds_read16(gate0 + off), gj = lds_read16(gate0 + 256 + off);
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = 32 * kblk + 8 * a + 4 * half + e;
          x[e] = s[4 * a + e] * (p.scale * gj[e]) * __expf(bi - bj[e]);
          if (diag && j > iq) x[e] = 0.f;
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
    weigh(s00, 0, bi0, ln, true, p00);
    weigh(s01, 0, bi1, 32 + ln, false, p01);
    weigh(s11, 1, bi1, 32 + ln, true, p11);

    // ---- aggregation inside the chunk: O^T += V^T P^T (this wave's 32 value columns) ----
    bf16x8 vf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) vf[s] = tr_frag(vb_, std::integral_constant<int, C::CPRV>{}, vblk, s);
    o[0] = mfma(vf[0], __builtin_bit_cast(bf16x8, p00[0]), o[0]);
    o[0] = mfma(vf[1], __builtin_bit_cast(bf16x8, p00[1]), o[0]);
    o[1] = mfma(vf[0], __builtin_bit_cast(bf16x8, p01[0]), o[1]);
    o[1] = mfma(vf[1], __builtin_bit_cast(bf16x8, p01[1]), o[1]);
    o[1] = mfma(vf[2], __builtin_bit_cast(bf16x8, p11[0]), o[1]);
    o[1] = mfma(vf[3], __builtin_bit_cast(bf16x8, p11[1]), o[1]);

    // ---- store: lane = query row, four 16-byte pieces of the wave's 32 columns ----
#pragma unroll
    for (int ib = 0; ib < 2; ++ib) {
      const int64_t i = t0 + 32 * ib + ln;
      if (i < L) {
        const int64_t e0 = ((int64_t)bh * L + i) * C::DV + 32 * vblk + 4 * half;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          const f32x4 v = {o[ib][4 * a], o[ib][4 * a + 1], o[ib][4 * a + 2], o[ib][4 * a + 3]};
          if (p.out_bf16) {
            bf16x4 hv;
#pragma unroll
            for (int e = 0; e < 4; ++e) hv[e] = (__bf16)v[e];
            *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.O) + e0 + 8 * a) = hv;
          } else {
            *reinterpret_cast<f32x4*>(static_cast<float*>(p.O) + e0 + 8 * a) = v;
          }
        }
      }
    }

    // ---- state update: H = e^{b_last} H + K^T (w . V) ----
    {
      const float dec = __expf(b_last);
#pragma unroll
      for (int db = 0; db < C::DBQ; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) H[db][r] *= dec;
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      // the V fragment of token step s times the tokens' weights (element e of the fragment: token 16 s + 8 (e / 4) + 4 half + e % 4)
      const f32x4 w0 = lds_read16(gate0 + 512 + (16 * s + 4 * half) * 4), w1 = lds_read16(gate0 + 512 + (16 * s + 8 + 4 * half) * 4);
      bf16x8 vw;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        vw[e] = (__bf16)((float)vf[s][e] * w0[e]);
        vw[4 + e] = (__bf16)((float)vf[s][4 + e] * w1[e]);
      }
#pragma unroll
      for (int db = 0; db < C::DBQ; ++db)
        H[db] = mfma(tr_frag(kb_, std::integral_constant<int, C::CPRQ>{}, db, s), vw, H[db]);
    }
  }

  if (p.h_out) {
    float* dst = p.h_out + (int64_t)bh * C::DQK * C::DV + 32 * vblk + ln;
#pragma unroll
    for (int db = 0; db < C::DBQ; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) dst[(int64_t)(32 * db + key_offset(r) + 4 * half) * C::DV] = H[db][r];
  }
}

template <int DQK, int DV, int HPW = 1>
hipError_t launch(const GatedParams& p, const DecayTable& dt, hipStream_t s) {
  typedef GCfg<DQK, DV, HPW> C;
  hipLaunchKernelGGL(gated_recurrent_kernel<C>, dim3((unsigned)(p.B * p.H / HPW)), dim3(C::THREADS), 0, s, p, dt);
  return hipGetLastError();
}

}  // namespace

bool gated_supported(int dqk, int dv) { return (dqk == 64 || dqk == 128) && (dv == 64 || dv == 128); }

hipError_t launch_gated_recurrent(const GatedParams& p, const DecayTable& dt, int dqk, int dv, hipStream_t s) {
  if (dqk == 64 && dv == 64) return launch<64, 64>(p, dt, s);
  if (dqk == 128 && dv == 64) {
    // value heads that share their q/k head (Mamba2's groups) share the Q and K tiles of a workgroup, up to four
    const int grp = p.H / p.H_qk;
    if (grp % 4 == 0) return launch<128, 64, 4>(p, dt, s);
    if (grp % 2 == 0) return launch<128, 64, 2>(p, dt, s);
    return launch<128, 64>(p, dt, s);
  }
  if (dqk == 64 && dv == 128) return launch<64, 128>(p, dt, s);
  if (dqk == 128 && dv == 128) return launch<128, 128>(p, dt, s);
  return hipErrorInvalidValue;
}

}  // namespace ae
