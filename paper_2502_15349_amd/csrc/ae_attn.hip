// C ABI of the fused parallel-pattern attention forward operator: descriptor
// validation, kernel/tile selection, launch.  See include/ae_attn.h.
#include "../../include/ae_attn.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <cstdlib>
#include <new>

#include "bwd.hpp"
#include "dispatch.hpp"
#include "attn_decode.hpp"
#include "gated.hpp"
#include "recurrent.hpp"

// ---- static device scratch for the entry point that allocates nothing -----------------------
// ae_attn_forward_split_static keeps the partial rows of the split-key forward in this array instead of a
// caller's workspace.  The array's name is a host-side stand-in, not a device address: each device that
// loads the library holds its own copy at its own address, which hipGetSymbolAddress returns for the
// device that is current; host code uses that pointer only.
static __device__ __align__(256) unsigned char scratch[AE_ATTN_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[256] = "";

ae_status_t fail(ae_status_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

const ae::KernelEntry* find_kernel(int dqk, int dv, int norm, int mod, int mask, int fold) {
  typedef const ae::KernelEntry* (*table_fn)(int*);
  static const table_fn tables[] = {ae::table_64_64, ae::table_128_128, ae::table_128_256, ae::table_192_128, ae::table_256_128};
  for (table_fn tf : tables) {
    int n = 0;
    const ae::KernelEntry* t = tf(&n);
    for (int i = 0; i < n; ++i)
      if (t[i].dqk == dqk && t[i].dv == dv && t[i].norm == norm && t[i].mod == mod && t[i].mask == mask && t[i].fold == fold)
        return &t[i];
  }
  return nullptr;
}

bool dims_supported(int dqk, int dv) {
  return (dqk == 64 && dv == 64) || (dqk == 128 && dv == 128) || (dqk == 128 && dv == 256) ||
         (dqk == 192 && dv == 128) || (dqk == 256 && (dv == 128 || dv == 512));
}

void fill_strides(int64_t dst[3], const int64_t src[3], int H, int L, int D) {
  if (src[0] == 0 && src[1] == 0 && src[2] == 0) {
    dst[2] = D;
    dst[1] = (int64_t)L * D;
    dst[0] = (int64_t)H * L * D;
  } else {
    dst[0] = src[0];
    dst[1] = src[1];
    dst[2] = src[2];
  }
}

// ---- split keys: combining the partial results -----------------------------------------
// Softmax over a union of key sets: with lse_c = ln sum_{j in set c} exp(x_j) and O_c the
// normalised partial rows, O = sum_c exp(lse_c - LSE) O_c and LSE = ln sum_c exp(lse_c) (the
// rule by which the online row-norm state of two key blocks is combined, Section 4.1).  A
// split without a visible key has lse_c = -inf and weight 0.
struct MergeParams {
  const float* ws_o;    // [n_splits, rows, D_v]
  const float* ws_lse;  // [n_splits, rows]
  void* O;              // fp32 or bf16, strides os[] in elements
  float* stats;         // optional [rows]
  int n_splits, B, H_q, L_q, D_v, out_bf16;
  int64_t os[3];
};
__global__ __launch_bounds__(256) void attn_merge_kernel(const MergeParams p) {
  const int64_t rows = (int64_t)p.B * p.H_q * p.L_q;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // one wavefront per row
  if (r >= rows) return;
  const int lane = threadIdx.x & 63;
  // the ranges' log-sum-exp: range c in lane c % 64, slot c / 64 (at most kMaxSplits ranges), all loads at once
  constexpr int kSlots = 4;  // kMaxSplits / 64
  float lc[kSlots];
  float mx = -INFINITY;
#pragma unroll
  for (int k = 0; k < kSlots; ++k) {
    const int c = lane + 64 * k;
    lc[k] = c < p.n_splits ? p.ws_lse[c * rows + r] : -INFINITY;
    mx = fmaxf(mx, lc[k]);
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) mx = fmaxf(mx, __shfl_xor(mx, s));
  float tot = 0.f;
#pragma unroll
  for (int k = 0; k < kSlots; ++k) tot += lc[k] == -INFINITY ? 0.f : __expf(lc[k] - mx);
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) tot += __shfl_xor(tot, s);
  const float lse = mx == -INFINITY ? -INFINITY : mx + __logf(tot);
  float wc[kSlots];  // the ranges' weights
#pragma unroll
  for (int k = 0; k < kSlots; ++k) wc[k] = lc[k] == -INFINITY ? 0.f : __expf(lc[k] - lse);
  const int i = (int)(r % p.L_q), hq = (int)((r / p.L_q) % p.H_q), b = (int)(r / ((int64_t)p.L_q * p.H_q));
  const int64_t obase = b * p.os[0] + hq * p.os[1] + (int64_t)i * p.os[2];
  for (int d = lane; d < p.D_v; d += 64) {
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < kSlots; ++k) {
      if (64 * k >= p.n_splits) break;
      const int n = min(64, p.n_splits - 64 * k);
#pragma unroll 8
      for (int cc = 0; cc < n; ++cc)  // (independent loads: the unrolled ones are in flight together)
        acc += __shfl(wc[k], cc) * p.ws_o[((64 * k + cc) * rows + r) * p.D_v + d];
    }
    if (p.out_bf16) static_cast<__bf16*>(p.O)[obase + d] = (__bf16)acc;
    else static_cast<float*>(p.O)[obase + d] = acc;
  }
  if (p.stats != nullptr && lane == 0) p.stats[r] = lse;
}

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// The current device's copy of `scratch` (looked up once per device); null with g_err set on failure.
void* static_scratch() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fail(AE_ERR_HIP, "ae_attn_forward_split_static: hipGetDevice: %s (device %d)", hipGetErrorString(e), dev);
    return nullptr;
  }
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (ptr) return ptr;
  e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !ptr) {
    fail(AE_ERR_HIP, "ae_attn_forward_split_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    return nullptr;
  }
  g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // two first calls racing store the same address
  return ptr;
}

}  // namespace

struct ae_attn {
  ae_attn_desc_t desc;
  const ae::KernelEntry* kernel;
  ae::Params params;  // pointers filled in per call
  ae::DecayTable decay;
  int grid;
  size_t ws_bytes;  // workspace the split-key forward needs (0: keys are not split)
  // D_v = 512 (Table 2, "Retention Parallel" 256 / 512): the output accumulators of 512 columns do not fit the
  // register file beside the 256-wide query fragments, so the forward pass is v_slices launches of the 256 / 128
  // kernel, each over 128 columns of V and O (the scores and the row normalizer are the same in every launch)
  int v_slices;
  // One query row per head, softmax, every key visible (a decoding step): with split keys the ranges are walked by
  // the streaming kernel of attn_decode.hip instead of the 256-row attention kernel
  bool decode;
};

extern "C" {

ae_status_t ae_attn_create(const ae_attn_desc_t* d, ae_attn_t** out) {
  if (out) *out = nullptr;
  if (!d || !out) return fail(AE_ERR_INVALID_ARG, "ae_attn_create: null argument");
  if (d->B <= 0 || d->H_q <= 0 || d->H_kv <= 0 || d->L_q <= 0 || d->L_k <= 0 || d->D_qk <= 0 || d->D_v <= 0)
    return fail(AE_ERR_INVALID_ARG, "ae_attn_create: every size must be positive");
  if (d->H_q % d->H_kv != 0)
    return fail(AE_ERR_INVALID_ARG, "ae_attn_create: H_q (%d) is not a multiple of H_kv (%d)", d->H_q, d->H_kv);
  if (!std::isfinite(d->scale) || d->scale == 0.f)
    return fail(AE_ERR_INVALID_ARG, "ae_attn_create: scale must be finite and non-zero");
  if ((int)d->score_mod < 0 || (int)d->score_mod > AE_MOD_BIAS_TENSOR)
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: unknown score_mod %d", (int)d->score_mod);
  if ((int)d->norm < 0 || (int)d->norm > AE_NORM_NONE)
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: unknown norm %d", (int)d->norm);
  if ((int)d->mask < 0 || (int)d->mask > AE_MASK_SLIDING_WINDOW)
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: unknown mask %d", (int)d->mask);
  if (d->mask == AE_MASK_SLIDING_WINDOW && d->window < 1)
    return fail(AE_ERR_INVALID_ARG, "ae_attn_create: the sliding window must hold at least one key");
  if (d->out_dtype != AE_OUT_F32 && d->out_dtype != AE_OUT_BF16)
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: unknown out_dtype %d", (int)d->out_dtype);
  if (d->kv_splits < AE_KV_SPLITS_AUTO || d->kv_splits > 256)
    return fail(AE_ERR_INVALID_ARG, "ae_attn_create: kv_splits must be AE_KV_SPLITS_AUTO or between 0 and 256");
  if (d->kv_splits > 1 && (d->norm != AE_NORM_SOFTMAX || d->mask == AE_MASK_SLIDING_WINDOW))
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: split keys come with softmax and the masks NONE and CAUSAL only");
  if (d->score_mod == AE_MOD_BIAS && !std::isfinite(d->bias))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_create: bias must be finite");
  if ((int64_t)d->B * d->H_kv > (1 << 24) || (int64_t)d->L_q > (1 << 28) || (int64_t)d->L_k > (1 << 28))
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: problem too large for 32-bit tile indices");

  if (!dims_supported(d->D_qk, d->D_v))
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: head dims %d/%d not in the tile table (64/64, 128/128, 128/256, 192/128; 256/128 and 256/512 for retention)",
                d->D_qk, d->D_v);

  int mod = ae::MOD_PLAIN;
  if (d->score_mod == AE_MOD_HEAD_DECAY) mod = ae::MOD_DECAY;
  if (d->score_mod == AE_MOD_RELU) mod = ae::MOD_RELU;
  if (d->score_mod == AE_MOD_BIAS_TENSOR) {
    mod = ae::MOD_BIAS_T;
    if (d->mask == AE_MASK_SLIDING_WINDOW || d->kv_splits > 1)
      return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: BIAS_TENSOR comes with the masks NONE and CAUSAL and without split keys");
  }
  if (d->score_mod == AE_MOD_HEAD_DECAY) {
    if (d->mask != AE_MASK_CAUSAL)
      return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: HEAD_DECAY needs the causal mask");
    if (!d->gamma) return fail(AE_ERR_INVALID_ARG, "ae_attn_create: HEAD_DECAY needs gamma[H_q]");
    if (d->H_q > AE_MAX_DECAY_HEADS)
      return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: HEAD_DECAY supports at most %d query heads", AE_MAX_DECAY_HEADS);
    for (int h = 0; h < d->H_q; ++h)
      if (!std::isfinite(d->gamma[h]) || !(d->gamma[h] > 0.f))
        return fail(AE_ERR_INVALID_ARG, "ae_attn_create: gamma[%d] must be finite and > 0", h);
  }
  // Softmax and sigmoid without a bias tensor: the kernels that take the scale on Q (rounded to bf16 again, as the
  // paper's own modification of q does) and the rest of the exponent from the accumulator's initial value -- where
  // that second rounding is harmless: it moves an exponent by about 2^-9 |scale| log2(e) |q||k| / sqrt(D_qk), which
  // for unit-variance inputs and |scale| sqrt(D_qk) <= 2 stays below the bf16 rounding of the weight itself.
  // Larger scales keep the scale in fp32 on the scores.
  const bool fold = (d->norm == AE_NORM_SOFTMAX || d->norm == AE_NORM_SIGMOID) && mod == ae::MOD_PLAIN &&
                    std::fabs(d->scale) * std::sqrt((float)d->D_qk) <= 2.f;
  const int v_slices = d->D_v == 512 ? 4 : 1;
  if (v_slices > 1 && d->kv_splits > 1) return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: D_v = 512 comes without split keys");
  const ae::KernelEntry* k = find_kernel(d->D_qk, d->D_v / v_slices, (int)d->norm, mod, (int)d->mask, fold ? 1 : 0);
  if (!k && fold) k = find_kernel(d->D_qk, d->D_v / v_slices, (int)d->norm, mod, (int)d->mask, 0);
  if (!k)
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: no kernel for score_mod %d with norm %d and mask %d",
                (int)d->score_mod, (int)d->norm, (int)d->mask);

  ae_attn* h = new (std::nothrow) ae_attn;
  if (!h) return fail(AE_ERR_NOMEM, "ae_attn_create: out of host memory");
  std::memset(h, 0, sizeof(*h));
  h->desc = *d;
  h->desc.gamma = nullptr;  // the caller's array is not kept
  h->kernel = k;
  h->v_slices = v_slices;

  ae::Params& p = h->params;
  p.B = d->B; p.H_q = d->H_q; p.H_kv = d->H_kv; p.L_q = d->L_q; p.L_k = d->L_k;
  p.g = d->H_q / d->H_kv;
  p.n_qtiles = (d->L_q + k->block_m - 1) / k->block_m;
  p.n_groups = d->B * d->H_kv;
  fill_strides(p.qs, d->q_stride, d->H_q, d->L_q, d->D_qk);
  fill_strides(p.ks, d->k_stride, d->H_kv, d->L_k, d->D_qk);
  fill_strides(p.vs, d->v_stride, d->H_kv, d->L_k, d->D_v);
  fill_strides(p.os, d->o_stride, d->H_q, d->L_q, d->D_v);
  fill_strides(p.bs, d->bias_stride, d->H_q, d->L_q, d->L_k);
  if (mod == ae::MOD_BIAS_T && (p.bs[0] < 0 || p.bs[1] < 0 || p.bs[2] < d->L_k || p.bs[2] % 8 != 0 || p.bs[0] % 8 != 0 || p.bs[1] % 8 != 0)) {
    delete h;
    return fail(AE_ERR_INVALID_ARG, "ae_attn_create: bias strides must be non-negative multiples of 8 elements, the row stride >= L_k");
  }
  const int64_t* in_strides[3] = {p.qs, p.ks, p.vs};
  const int in_d[3] = {d->D_qk, d->D_qk, d->D_v};
  for (int t = 0; t < 3; ++t) {
    for (int a = 0; a < 3; ++a)
      if (in_strides[t][a] < 0 || in_strides[t][a] % 8 != 0) {
        delete h;
        return fail(AE_ERR_INVALID_ARG, "ae_attn_create: Q/K/V strides must be non-negative multiples of 8 elements");
      }
    if (in_strides[t][2] < in_d[t]) {
      delete h;
      return fail(AE_ERR_INVALID_ARG, "ae_attn_create: a Q/K/V row stride is smaller than the head dim");
    }
  }
  // the kernels address the rows of one (batch, head) slab with 32-bit byte offsets
  {
    const int64_t lim = (int64_t)1 << 32;
    if ((int64_t)d->L_q * p.qs[2] * 2 >= lim || (int64_t)d->L_k * p.ks[2] * 2 >= lim || (int64_t)d->L_k * p.vs[2] * 2 >= lim ||
        (mod == ae::MOD_BIAS_T && (int64_t)d->L_q * p.bs[2] * 2 >= lim)) {
      delete h;
      return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: one (batch, head) slab of Q, K, V or the bias spans 4 GiB or more");
    }
  }
  for (int a = 0; a < 3; ++a)
    if (p.os[a] < 0 || p.os[a] % 4 != 0) {
      delete h;
      return fail(AE_ERR_INVALID_ARG, "ae_attn_create: O strides must be non-negative multiples of 4 elements");
    }
  if (p.os[2] < d->D_v) {
    delete h;
    return fail(AE_ERR_INVALID_ARG, "ae_attn_create: the O row stride is smaller than D_v");
  }

  const float log2e = 1.4426950408889634f;
  const float a = std::fabs(d->scale);
  const float bias = d->score_mod == AE_MOD_BIAS ? d->bias : 0.f;
  if (d->norm == AE_NORM_SOFTMAX || d->norm == AE_NORM_SIGMOID) {
    p.c = a * log2e;
    p.b2 = bias * log2e;
  } else {
    p.c = a;
    p.b2 = bias;
  }
  if (mod == ae::MOD_BIAS_T) {
    p.b2 = (d->norm == AE_NORM_SOFTMAX || d->norm == AE_NORM_SIGMOID) ? log2e : 1.f;  // the unit of the bias values
    if (d->norm == AE_NORM_SOFTMAX) p.c = a;  // biased scores in natural units until the exponent (see post_pair)
  }
  p.neg_q = d->scale < 0.f ? 1 : 0;
  p.out_bf16 = d->out_dtype == AE_OUT_BF16 ? 1 : 0;
  // a window wider than every row's reach hides nothing more than the causal mask; clamped so that
  // the kernel's row + offset - window arithmetic stays inside 32 bits
  p.window = d->mask == AE_MASK_SLIDING_WINDOW ? (int)std::min<int64_t>(d->window, (int64_t)d->L_q + d->L_k) : 0;
  if (mod == ae::MOD_DECAY)
    for (int hh = 0; hh < d->H_q; ++hh) h->decay.log2_gamma[hh] = std::log2(d->gamma[hh]);

  // Workgroup -> tile mapping (see attn_fwd_kernel): groups are dealt to the 8
  // XCDs round-robin and walked `interleave` at a time per XCD.  Measured: a group
  // whose workgroups fill the XCD's 32 CUs on their own runs best with 1-2 groups
  // walked together, smaller groups with 8 (more K/V streams spread the reads
  // over more L2 channels).
  const int64_t per_group = (int64_t)p.n_qtiles * p.g;
  const int64_t rounds = (p.n_groups + 7) / 8;  // groups per XCD
#ifdef AE_TUNE_INTERLEAVE  // build-time knob of the mapping sweeps, like the AE_SHAPE_* entries of the tile table
  int interleave = AE_TUNE_INTERLEAVE;
#else
  int interleave = per_group >= 32 ? 2 : 8;
#endif
  if (interleave < 1) interleave = 1;
  if (interleave > rounds) interleave = (int)rounds;
  p.interleave = interleave;
  const int64_t blocks = (rounds + interleave - 1) / interleave;
  const int64_t grid = blocks * interleave * 8 * per_group;
  if (grid > 0x7fffffffLL) {
    delete h;
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: grid of %lld workgroups exceeds the launch limit", (long long)grid);
  }
  h->grid = (int)grid;
  // Split keys: n_splits copies of the grid, each over its own range of key tiles.
  p.n_splits = 1;
  p.split_tiles = 0;
  p.base_grid = (int)grid;
  h->ws_bytes = 0;
  int kv_splits = d->kv_splits;
  h->decode = d->L_q == 1 && d->norm == AE_NORM_SOFTMAX && mod == ae::MOD_PLAIN && d->mask != AE_MASK_SLIDING_WINDOW &&
              v_slices == 1 && ae::decode_supported(d->D_qk, d->D_v);
  if (kv_splits == AE_KV_SPLITS_AUTO && h->decode) {
    // Measured on the decoding row of Table 2 (16 heads, batch 1 and 8, 2k-8k keys): fastest with 128-256
    // workgroups (8 ranges at batch 1, 2 at batch 8) -- every workgroup pays the latency of its first loads and of
    // the combination at its end, and every range costs the merge kernel a row to read -- and with ranges of at
    // least four key tiles.
    const int key_tiles = (d->L_k + h->kernel->block_n - 1) / h->kernel->block_n;
    const int64_t rows = (int64_t)d->B * d->H_q, want = (192 + rows / 2) / rows;
    kv_splits = (int)std::min<int64_t>(std::min<int64_t>(want, key_tiles / 4), 256);
  } else if (kv_splits == AE_KV_SPLITS_AUTO) {
    // Measured on decoding shapes (one query row, 16 heads, 2k-8k keys, batch 1 and 8): the
    // fastest launches hold some 128-256 workgroups with at least 8 key tiles each; more
    // ranges cost a start and an end of a workgroup apiece.  Only where the keys may be split
    // and the query tiles alone leave most of the device idle.
    kv_splits = 0;
    if (d->norm == AE_NORM_SOFTMAX && d->mask != AE_MASK_SLIDING_WINDOW && mod != ae::MOD_BIAS_T && v_slices == 1 && grid < 160) {
      const int key_tiles = (d->L_k + h->kernel->block_n - 1) / h->kernel->block_n;
      const int64_t want = (192 + grid / 2) / grid;  // round(192 / workgroups)
      kv_splits = (int)std::min<int64_t>(std::min<int64_t>(want, key_tiles / 8), 256);
    }
  }
  if (kv_splits > 1) {
    const int key_tiles = (d->L_k + h->kernel->block_n - 1) / h->kernel->block_n;
    p.split_tiles = (key_tiles + kv_splits - 1) / kv_splits;
    p.n_splits = (key_tiles + p.split_tiles - 1) / p.split_tiles;
    if (p.n_splits > 1) {
      if (grid * p.n_splits > 0x7fffffffLL) {
        delete h;
        return fail(AE_ERR_UNSUPPORTED, "ae_attn_create: grid of %lld workgroups exceeds the launch limit",
                    (long long)(grid * p.n_splits));
      }
      h->grid = (int)(grid * p.n_splits);
      const size_t rows = (size_t)d->B * d->H_q * d->L_q;
      h->ws_bytes = (size_t)p.n_splits * rows * ((size_t)d->D_v + 1) * sizeof(float);
    }
  }
  *out = h;
  return AE_OK;
}

// Recurrent pattern: where the chunk-as-batch launch finds the state in front of each chunk (see ae::Params::state).
struct CarriedState {
  const __bf16* state;
  int64_t batch_stride, head_stride;
  int first_batch;
};

static ae_status_t forward_impl(const ae_attn_t* h, const void* Q, const void* K, const void* V, void* O, float* stats,
                                hipStream_t stream, void* workspace = nullptr, size_t workspace_bytes = 0,
                                const void* bias = nullptr, const CarriedState* carried = nullptr) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward: null handle");
  if (!Q || !K || !V || !O) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward: null device pointer");
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15)
    return fail(AE_ERR_INVALID_ARG, "ae_attn_forward: device pointers must be 16-byte aligned");
  if (O == Q || O == K || O == V) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward: O aliases an input");
  if ((h->kernel->mod == ae::MOD_BIAS_T) != (bias != nullptr))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_forward: a handle with AE_MOD_BIAS_TENSOR, and only such a handle, runs through "
                                    "ae_attn_forward_bias with its bias tensor");
  if (bias && (((uintptr_t)bias & 15) || bias == O)) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_bias: the bias tensor must be 16-byte aligned and must not alias O");
  ae::Params p = h->params;
  p.bias = static_cast<const __bf16*>(bias);
  p.state = nullptr;
  if (carried) {
    p.state = carried->state;
    p.state_bs = carried->batch_stride;
    p.state_hs = carried->head_stride;
    p.state_b0 = carried->first_batch;
  }
  p.Q = static_cast<const __bf16*>(Q);
  p.K = static_cast<const __bf16*>(K);
  p.V = static_cast<const __bf16*>(V);
  p.O = O;
  p.stats = stats;
  if (p.n_splits > 1) {
    if (!workspace || ((uintptr_t)workspace & 15) || workspace_bytes < h->ws_bytes)
      return fail(AE_ERR_INVALID_ARG,
                  "ae_attn_forward: keys are split: call ae_attn_forward_split with a 16-byte aligned workspace of "
                  "ae_attn_workspace_bytes() bytes");
    const size_t rows = (size_t)p.B * p.H_q * p.L_q;
    p.ws_o = static_cast<float*>(workspace);
    p.ws_lse = p.ws_o + (size_t)p.n_splits * rows * h->desc.D_v;
  }
  hipError_t e = hipSuccess;
  const bool decode = h->decode && p.n_splits > 1 && !carried && !bias;
  if (decode) {
    ae::DecodeParams q;
    q.Q = p.Q;
    q.K = p.K;
    q.V = p.V;
    q.ws_o = p.ws_o;
    q.ws_lse = p.ws_lse;
    for (int a = 0; a < 3; ++a) {
      if (a < 2) q.qs[a] = p.qs[a];
      q.ks[a] = p.ks[a];
      q.vs[a] = p.vs[a];
    }
    q.rows = (int64_t)p.B * p.H_q;
    q.H_q = p.H_q;
    q.g = p.g;
    q.L_k = p.L_k;
    q.n_splits = p.n_splits;
    q.split_keys = p.split_tiles * h->kernel->block_n;
    q.c = h->desc.scale * 1.4426950408889634f;
    q.b2 = (h->desc.score_mod == AE_MOD_BIAS ? h->desc.bias : 0.f) * 1.4426950408889634f;
    e = ae::launch_decode(q, h->desc.D_qk, h->desc.D_v, static_cast<hipStream_t>(stream));
  }
  for (int sl = 0; sl < h->v_slices && e == hipSuccess && !decode; ++sl) {
    if (sl > 0) {  // the next 128 columns of V and O
      p.V += h->kernel->dv;
      p.O = static_cast<char*>(p.O) + (size_t)h->kernel->dv * (p.out_bf16 ? 2 : 4);
    }
    e = h->kernel->launch(p, h->decay, h->grid, static_cast<hipStream_t>(stream));
  }
  if (e != hipSuccess) return fail(AE_ERR_HIP, "ae_attn_forward: launch failed: %s", hipGetErrorString(e));
  if (p.n_splits > 1) {
    MergeParams m;
    m.ws_o = p.ws_o;
    m.ws_lse = p.ws_lse;
    m.O = O;
    m.stats = stats;
    m.n_splits = p.n_splits;
    m.B = p.B;
    m.H_q = p.H_q;
    m.L_q = p.L_q;
    m.D_v = h->desc.D_v;
    m.out_bf16 = p.out_bf16;
    for (int a = 0; a < 3; ++a) m.os[a] = p.os[a];
    const int64_t rows = (int64_t)p.B * p.H_q * p.L_q;
    hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, static_cast<hipStream_t>(stream), m);
    e = hipGetLastError();
    if (e != hipSuccess) return fail(AE_ERR_HIP, "ae_attn_forward: merge launch failed: %s", hipGetErrorString(e));
  }
  return AE_OK;
}

ae_status_t ae_attn_forward(const ae_attn_t* h, const void* Q, const void* K, const void* V, void* O, hipStream_t stream) {
  return forward_impl(h, Q, K, V, O, nullptr, stream);
}

ae_status_t ae_attn_forward_stats(const ae_attn_t* h, const void* Q, const void* K, const void* V, void* O, void* stats,
                                  hipStream_t stream) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_stats: null handle");
  if (!stats || ((uintptr_t)stats & 3)) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_stats: stats must be a 4-byte aligned device pointer");
  if (stats == O || stats == Q || stats == K || stats == V)
    return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_stats: stats aliases another buffer");
  const int norm = h->kernel->norm;
  if (norm != ae::NORM_SOFTMAX && norm != ae::NORM_ABSSUM && norm != ae::NORM_ABS_OF_SUM)
    return fail(AE_ERR_UNSUPPORTED, "ae_attn_forward_stats: this normalization keeps no row statistic");
  return forward_impl(h, Q, K, V, O, static_cast<float*>(stats), stream);
}

ae_status_t ae_attn_forward_bias(const ae_attn_t* h, const void* Q, const void* K, const void* V, const void* bias, void* O,
                                 void* stats, hipStream_t stream) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_bias: null handle");
  if (!bias) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_bias: null bias tensor");
  if (stats) {
    if (((uintptr_t)stats & 3) || stats == O || stats == Q || stats == K || stats == V || stats == bias)
      return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_bias: stats must be 4-byte aligned and must not alias another buffer");
    if (h->kernel->norm != ae::NORM_SOFTMAX)
      return fail(AE_ERR_UNSUPPORTED, "ae_attn_forward_bias: this normalization keeps no row statistic");
  }
  return forward_impl(h, Q, K, V, O, static_cast<float*>(stats), stream, nullptr, 0, bias);
}

ae_status_t ae_attn_workspace_bytes(const ae_attn_t* h, size_t* bytes) {
  if (!h || !bytes) return fail(AE_ERR_INVALID_ARG, "ae_attn_workspace_bytes: null argument");
  *bytes = h->ws_bytes;
  return AE_OK;
}

ae_status_t ae_attn_forward_split(const ae_attn_t* h, const void* Q, const void* K, const void* V, void* O, void* stats,
                                  void* workspace, size_t workspace_bytes, hipStream_t stream) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_split: null handle");
  if (stats && (((uintptr_t)stats & 3) || stats == O || stats == Q || stats == K || stats == V))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_split: stats must be 4-byte aligned and must not alias another buffer");
  if (h->params.n_splits > 1 && (workspace == O || workspace == Q || workspace == K || workspace == V || (stats && workspace == stats)))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_split: the workspace aliases another buffer");
  return forward_impl(h, Q, K, V, O, static_cast<float*>(stats), stream, workspace, workspace_bytes);
}

ae_status_t ae_attn_forward_split_static(const ae_attn_t* h, const void* Q, const void* K, const void* V, void* O, void* stats,
                                         hipStream_t stream) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_split_static: null handle");
  if (stats && (((uintptr_t)stats & 3) || stats == O || stats == Q || stats == K || stats == V))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_forward_split_static: stats must be 4-byte aligned and must not alias another buffer");
  if (h->ws_bytes > (size_t)AE_ATTN_STATIC_SCRATCH_BYTES)
    return fail(AE_ERR_UNSUPPORTED,
                "ae_attn_forward_split_static: this handle's partial results take %zu bytes, the static scratch holds %zu; "
                "use ae_attn_forward_split with a workspace",
                h->ws_bytes, (size_t)AE_ATTN_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  if (h->params.n_splits > 1) {
    ws = static_scratch();
    if (!ws) return AE_ERR_HIP;
  }
  // every partial row and statistic that the merge kernel reads is written by the attention kernel of the
  // same call (ranges without a visible key write zeros and -inf), so nothing has to be cleared
  return forward_impl(h, Q, K, V, O, static_cast<float*>(stats), stream, ws, AE_ATTN_STATIC_SCRATCH_BYTES);
}

ae_status_t ae_attn_backward_workspace_bytes(const ae_attn_t* h, size_t* bytes) {
  if (!h || !bytes) return fail(AE_ERR_INVALID_ARG, "ae_attn_backward_workspace_bytes: null argument");
  const bool rows = h->desc.norm == AE_NORM_SOFTMAX || h->desc.norm == AE_NORM_ABSSUM || h->desc.norm == AE_NORM_ABS_OF_SUM;
  *bytes = rows ? (size_t)h->desc.B * h->desc.H_q * h->desc.L_q * sizeof(float) : 0;
  return AE_OK;
}

}  // extern "C"

static ae_status_t backward_impl(const ae_attn_t* h, const void* Q, const void* K, const void* V, const void* bias, const void* O,
                                 const void* dO, const void* stats, void* dQ, void* dK, void* dV, void* workspace,
                                 size_t workspace_bytes, hipStream_t stream, void* dBias = nullptr, int64_t dbias_ld = 0) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_attn_backward: null handle");
  if ((h->desc.score_mod == AE_MOD_BIAS_TENSOR) != (bias != nullptr))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_backward: a handle with AE_MOD_BIAS_TENSOR, and only such a handle, runs through "
                                    "ae_attn_backward_bias with its bias tensor");
  if (bias && (((uintptr_t)bias & 15) || bias == dQ || bias == dK || bias == dV || bias == workspace))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_backward_bias: the bias tensor must be 16-byte aligned and must not alias an output");
  const ae_attn_desc_t& d = h->desc;
  // no normalization + ReLU is one kernel variant of its own
  const int norm = d.norm == AE_NORM_NONE && d.score_mod == AE_MOD_RELU ? ae::BWD_NORM_NONE_RELU : h->kernel->norm;
  const bool abs_family = norm == ae::NORM_ABSSUM || norm == ae::NORM_ABS_OF_SUM;
  const bool mod_ok = d.score_mod == AE_MOD_NONE || d.score_mod == AE_MOD_BIAS || d.score_mod == AE_MOD_BIAS_TENSOR ||
                      norm == ae::BWD_NORM_NONE_RELU ||
                      ((abs_family || norm == ae::NORM_NONE) && d.score_mod == AE_MOD_HEAD_DECAY);
  if (!ae::backward_supported(d.D_qk, d.D_v, norm) || !mod_ok)
    return fail(AE_ERR_UNSUPPORTED,
                "ae_attn_backward: unsupported (score_mod, norm) pair or head dims");
  const bool softmax = norm == ae::NORM_SOFTMAX || abs_family;  // the variants that read O, the row statistic and a workspace
  if (!Q || !K || !V || !dO || !dQ || !dK || !dV || (softmax && (!O || !stats || !workspace)))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_backward: null device pointer");
  if ((((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)dO | (uintptr_t)dQ | (uintptr_t)dK | (uintptr_t)dV) & 15) ||
      (softmax && ((((uintptr_t)O | (uintptr_t)workspace) & 15) || ((uintptr_t)stats & 3))))
    return fail(AE_ERR_INVALID_ARG, "ae_attn_backward: device pointers must be 16-byte aligned (stats: 4-byte)");
  const void* ins[] = {Q, K, V, dO, softmax ? O : nullptr, softmax ? stats : nullptr};
  void* outs[] = {dQ, dK, dV, softmax ? workspace : nullptr};
  for (int a = 0; a < 4; ++a) {
    if (!outs[a]) continue;
    for (const void* in : ins)
      if (in == outs[a]) return fail(AE_ERR_INVALID_ARG, "ae_attn_backward: an output aliases an input");
    for (int c = a + 1; c < 4; ++c)
      if (outs[c] == outs[a]) return fail(AE_ERR_INVALID_ARG, "ae_attn_backward: two outputs alias");
  }
  size_t need = 0;
  ae_attn_backward_workspace_bytes(h, &need);
  if (workspace_bytes < need)
    return fail(AE_ERR_INVALID_ARG, "ae_attn_backward: the workspace holds %zu bytes, %zu are needed", workspace_bytes, need);
  ae::BwdParams p;
  p.Q = static_cast<const __bf16*>(Q);
  p.K = static_cast<const __bf16*>(K);
  p.V = static_cast<const __bf16*>(V);
  p.dO = static_cast<const __bf16*>(dO);
  p.O = O;
  p.lse = static_cast<const float*>(stats);
  p.delta = static_cast<float*>(workspace);
  p.bias = static_cast<const __bf16*>(bias);
  p.dbias = static_cast<__bf16*>(dBias);
  p.dbias_ld = dbias_ld;
  for (int a = 0; a < 3; ++a) p.bs[a] = h->params.bs[a];
  p.dQ = static_cast<float*>(dQ);
  p.dK = static_cast<float*>(dK);
  p.dV = static_cast<float*>(dV);
  p.B = d.B;
  p.H_q = d.H_q;
  p.H_kv = d.H_kv;
  p.L_q = d.L_q;
  p.L_k = d.L_k;
  p.g = d.H_q / d.H_kv;
  p.o_bf16 = d.out_dtype == AE_OUT_BF16;
  for (int a = 0; a < 3; ++a) {
    p.qs[a] = h->params.qs[a];
    p.ks[a] = h->params.ks[a];
    p.vs[a] = h->params.vs[a];
    p.os[a] = h->params.os[a];
  }
  const float log2e = 1.4426950408889634f;
  // softmax and sigmoid work in powers of two; without a normalization the modified score itself is the weight
  const float unit = norm == ae::NORM_SOFTMAX || norm == ae::NORM_SIGMOID ? log2e : 1.f;
  p.c2 = d.scale * unit;
  p.b2 = (d.score_mod == AE_MOD_BIAS ? d.bias : 0.f) * unit;
  p.bunit = unit;
  p.scale = d.scale;
  p.window = d.mask == AE_MASK_SLIDING_WINDOW ? std::min(d.window, d.L_q + d.L_k) : d.L_q + d.L_k;
  p.has_decay = d.score_mod == AE_MOD_HEAD_DECAY ? 1 : 0;
  // (batch, k/v head) groups walked side by side per XCD.  The workgroups of a group stream the same rows of the
  // other side, so a tile is fetched from memory once per group and XCD-resident set: few groups side by side mean
  // few fetches (measured on 1 x 128 heads x 8k, 192/128: 16 side by side 11.7 ms, 4: 10.5 ms).  Enough of them to
  // put a workgroup on every compute unit of the XCD, though, and with a causal mask four at least, so that the
  // last set to run -- heaviest workgroups first within a set -- is a small part of the grid.
  {
    const int64_t tiles_q = (d.L_q + 127) / 128 * (int64_t)p.g, tiles_kv = (d.L_k + 127) / 128;
    const int64_t rounds = ((int64_t)d.B * d.H_kv + 7) / 8;
#ifdef AE_TUNE_BWD_TOGETHER_Q  // build-time knobs of the mapping sweeps
    int64_t tq = AE_TUNE_BWD_TOGETHER_Q, tk = AE_TUNE_BWD_TOGETHER_KV;
#else
    const int64_t least = d.mask != AE_MASK_NONE ? 4 : 1;
    int64_t tq = std::max(least, (64 + tiles_q - 1) / tiles_q), tk = std::max(least, (32 + tiles_kv - 1) / tiles_kv);
#endif
    p.together[0] = (int)std::max<int64_t>(1, std::min(tq, rounds));
    p.together[1] = (int)std::max<int64_t>(1, std::min(tk, rounds));
  }
  hipError_t e = ae::launch_backward(p, h->decay, d.D_qk, d.D_v, norm, d.mask != AE_MASK_NONE, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(AE_ERR_HIP, "ae_attn_backward: launch failed: %s", hipGetErrorString(e));
  return AE_OK;
}

extern "C" {

ae_status_t ae_attn_backward(const ae_attn_t* h, const void* Q, const void* K, const void* V, const void* O, const void* dO,
                             const void* stats, void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                             hipStream_t stream) {
  return backward_impl(h, Q, K, V, nullptr, O, dO, stats, dQ, dK, dV, workspace, workspace_bytes, stream);
}

ae_status_t ae_attn_backward_bias(const ae_attn_t* h, const void* Q, const void* K, const void* V, const void* bias,
                                  const void* O, const void* dO, const void* stats, void* dQ, void* dK, void* dV,
                                  void* dBias, int64_t dbias_row_stride, void* workspace, size_t workspace_bytes,
                                  hipStream_t stream) {
  if (!bias) return fail(AE_ERR_INVALID_ARG, "ae_attn_backward_bias: null bias tensor");
  if (dBias) {
    if (!h) return fail(AE_ERR_INVALID_ARG, "ae_attn_backward_bias: null handle");
    if (((uintptr_t)dBias & 7) || dbias_row_stride < h->desc.L_k || dbias_row_stride % 4 != 0)
      return fail(AE_ERR_INVALID_ARG,
                  "ae_attn_backward_bias: dBias must be 8-byte aligned, its row stride a multiple of 4 elements and >= L_k");
    if (dBias == bias || dBias == dQ || dBias == dK || dBias == dV || dBias == workspace || dBias == Q || dBias == K ||
        dBias == V || dBias == O || dBias == dO)
      return fail(AE_ERR_INVALID_ARG, "ae_attn_backward_bias: dBias aliases another buffer");
  }
  return backward_impl(h, Q, K, V, bias, O, dO, stats, dQ, dK, dV, workspace, workspace_bytes, stream, dBias, dbias_row_stride);
}

ae_status_t ae_attn_destroy(ae_attn_t* h) {
  delete h;
  return AE_OK;
}

ae_status_t ae_attn_query(const ae_attn_t* h, int32_t* block_m, int32_t* block_n, int32_t* lds_bytes,
                          int32_t* grid_size, int32_t* block_threads) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_attn_query: null handle");
  if (block_m) *block_m = h->kernel->block_m;
  if (block_n) *block_n = h->kernel->block_n;
  if (lds_bytes) *lds_bytes = h->kernel->lds_bytes;
  if (grid_size) *grid_size = h->grid;
  if (block_threads) *block_threads = h->kernel->threads;
  return AE_OK;
}

const char* ae_attn_kernel_name(const ae_attn_t* h) { return h ? h->kernel->name : ""; }

const char* ae_attn_last_error(void) { return g_err; }

int32_t ae_attn_version(void) { return 1; }

}  // extern "C"

// ---- recurrent pattern: chunk-parallel retention -----------------------------------------------------------
// The intra-chunk part is the parallel-pattern kernel (per-head decay, causal, no normalization) run on the
// chunks as if they were batch entries: batch' = chunk index (stride chunk * D), heads' = `fold` batch entries x H
// heads (stride L * D, which is uniform over (batch, head) in a contiguous [B, H, L, D] tensor).  The decay table
// of that kernel holds 256 heads, so larger B * H take one launch per batch entry.
// Segments for a walk of L tokens by `workgroups` workgroups of the single-pass recurrent kernel: enough of them to
// give every compute unit one, none shorter than 512 tokens (each segment is walked twice, the first time for its
// state only).  nseg = 1: not cut.
static void gated_segments(int64_t workgroups, int L, int* nseg, int* seg_len) {
  *nseg = 1;
  *seg_len = 0;
  if (workgroups >= 192 || L < 1024) return;
  int64_t n = std::min<int64_t>((256 + workgroups - 1) / workgroups, L / 512);
  if (n < 2) return;
  const int len = (int)(((L + n - 1) / n + 63) / 64 * 64);
  *seg_len = len;
  *nseg = (L + len - 1) / len;
}

static size_t gated_segments_ws(int B, int H, int nseg, int dqk, int dv) {
  if (nseg == 1) return 0;
  const size_t slots = (size_t)B * H * nseg;
  return slots * dqk * dv * 4 + ((slots * 4 + 255) & ~(size_t)255);
}

// The walk described by p (whole sequence, caller's h_in / h_out), cut into segments: every segment's final state
// from a zero start and the sum of its log-decays; those chained into the state in front of every segment; the
// segments walked again, side by side, for their outputs.
static hipError_t launch_gated_segmented(const ae::GatedParams& p, const ae::DecayTable& dt, int dqk, int dv, int nseg, int seg_len,
                                         void* workspace, hipStream_t stream) {
  const size_t slots = (size_t)p.B * p.H * nseg;
  float* dec = static_cast<float*>(workspace);
  float* buf = reinterpret_cast<float*>(static_cast<char*>(workspace) + ((slots * 4 + 255) & ~(size_t)255));
  ae::GatedParams s1 = p;
  s1.nseg = nseg;
  s1.seg_len = seg_len;
  s1.state_only = 1;
  s1.h_in = nullptr;
  s1.h_out = buf;
  s1.seg_decay = dec;
  s1.O = nullptr;
  hipError_t e = ae::launch_gated_recurrent(s1, dt, dqk, dv, stream);
  if (e != hipSuccess) return e;
  e = ae::launch_gated_combine_segments(buf, dec, p.h_in, p.B * p.H, nseg, dqk * dv, stream);
  if (e != hipSuccess) return e;
  ae::GatedParams s2 = p;
  s2.nseg = nseg;
  s2.seg_len = seg_len;
  s2.h_in = buf;
  s2.h_out_last_only = 1;
  return ae::launch_gated_recurrent(s2, dt, dqk, dv, stream);
}

struct ae_recurrent {
  ae_recurrent_desc_t desc;
  ae_attn_t* full;  // all chunks of full length; null if L < chunk
  ae_attn_t* tail;  // the short last chunk; null if L is a multiple of chunk
  ae::DecayTable decay;
  int fold, n_full, n_chunks, tail_len;
  size_t ws_bytes;
  bool single_pass;  // forward runs as one kernel with the state on chip (see ae_recurrent_forward_state)
  int nseg, seg_len;  // ... or, with few (batch, head) pairs and a long sequence, as that kernel on segments (nseg > 1)
};

extern "C" {

ae_status_t ae_recurrent_create(const ae_recurrent_desc_t* d, ae_recurrent_t** out) {
  if (out) *out = nullptr;
  if (!d || !out) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_create: null argument");
  if (d->B < 1 || d->H < 1 || d->L < 1) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_create: B, H, L must be >= 1");
  if (!std::isfinite(d->scale) || d->scale == 0.f) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_create: scale must be finite and non-zero");
  if (!d->gamma) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_create: gamma missing");
  if (d->H > AE_MAX_DECAY_HEADS) return fail(AE_ERR_UNSUPPORTED, "ae_recurrent_create: at most %d heads", AE_MAX_DECAY_HEADS);
  for (int i = 0; i < d->H; ++i)
    if (!std::isfinite(d->gamma[i]) || d->gamma[i] <= 0.f || d->gamma[i] > 1.f)
      return fail(AE_ERR_INVALID_ARG, "ae_recurrent_create: gamma[%d] must be in (0, 1]", i);
  if (d->chunk != 64 && d->chunk != 128 && d->chunk != 256)
    return fail(AE_ERR_UNSUPPORTED, "ae_recurrent_create: chunk must be 64, 128 or 256");
  if (d->out_dtype != AE_OUT_F32 && d->out_dtype != AE_OUT_BF16)
    return fail(AE_ERR_INVALID_ARG, "ae_recurrent_create: unknown out_dtype");
  if (!ae::recurrent_supported(d->D_qk, d->D_v))
    return fail(AE_ERR_UNSUPPORTED, "ae_recurrent_create: head dims %d/%d not built (64/64, 128/128)", d->D_qk, d->D_v);
  if ((int64_t)d->L * std::max(d->D_qk, d->D_v) * 2 >= (int64_t)1 << 32)
    return fail(AE_ERR_UNSUPPORTED, "ae_recurrent_create: one (batch, head) slab must span less than 4 GiB");
  ae_recurrent* h = new (std::nothrow) ae_recurrent();
  if (!h) return fail(AE_ERR_NOMEM, "ae_recurrent_create: out of host memory");
  h->desc = *d;
  h->desc.gamma = nullptr;
  h->full = h->tail = nullptr;
  h->fold = (int64_t)d->B * d->H <= AE_MAX_DECAY_HEADS ? d->B : 1;
  h->n_full = d->L / d->chunk;
  h->tail_len = d->L % d->chunk;
  h->n_chunks = h->n_full + (h->tail_len ? 1 : 0);
  std::memset(&h->decay, 0, sizeof(h->decay));
  for (int i = 0; i < d->H; ++i) h->decay.log2_gamma[i] = std::log2(d->gamma[i]);
  float gam[AE_MAX_DECAY_HEADS];
  for (int i = 0; i < h->fold * d->H; ++i) gam[i] = d->gamma[i % d->H];
  ae_attn_desc_t a;
  std::memset(&a, 0, sizeof(a));
  a.H_q = a.H_kv = h->fold * d->H;
  a.D_qk = d->D_qk;
  a.D_v = d->D_v;
  a.score_mod = AE_MOD_HEAD_DECAY;
  a.gamma = gam;
  a.norm = AE_NORM_NONE;
  a.mask = AE_MASK_CAUSAL;
  a.scale = d->scale;
  a.out_dtype = d->out_dtype;
  const int64_t L = d->L;
  auto strides = [&](int64_t* st, int D) { st[0] = (int64_t)d->chunk * D; st[1] = L * D; st[2] = D; };
  strides(a.q_stride, d->D_qk);
  strides(a.k_stride, d->D_qk);
  strides(a.v_stride, d->D_v);
  strides(a.o_stride, d->D_v);
  ae_status_t st = AE_OK;
  if (h->n_full) {
    a.B = h->n_full;
    a.L_q = a.L_k = d->chunk;
    st = ae_attn_create(&a, &h->full);
  }
  if (st == AE_OK && h->tail_len) {
    a.B = 1;
    a.L_q = a.L_k = h->tail_len;
    st = ae_attn_create(&a, &h->tail);
  }
  if (st != AE_OK) {
    ae_attn_destroy(h->full);
    ae_attn_destroy(h->tail);
    delete h;
    return st;  // the message of the inner call stands
  }
  h->ws_bytes = (size_t)d->B * d->H * h->n_chunks * d->D_qk * d->D_v * 2;  // one bf16 state per chunk
  // Measured (8 x 32 heads x 8192 tokens, 128/128): one workgroup per (batch, head) walking the whole sequence with
  // the state on chip beats the two-kernel form once there is about a workgroup per compute unit; with few pairs
  // (batch 1) the sequential walk leaves the device idle and the chunk-parallel form wins.
  h->single_pass = ae::gated_supported(d->D_qk, d->D_v) && (int64_t)d->B * d->H >= 192;
  h->nseg = 1;
  h->seg_len = 0;
  if (!h->single_pass && ae::gated_supported(d->D_qk, d->D_v)) {
    gated_segments((int64_t)d->B * d->H, d->L, &h->nseg, &h->seg_len);
    h->ws_bytes = std::max(h->ws_bytes, gated_segments_ws(d->B, d->H, h->nseg, d->D_qk, d->D_v));
  }
  *out = h;
  return AE_OK;
}

ae_status_t ae_recurrent_workspace_bytes(const ae_recurrent_t* h, size_t* bytes) {
  if (!h || !bytes) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_workspace_bytes: null argument");
  *bytes = h->ws_bytes;
  return AE_OK;
}

ae_status_t ae_recurrent_forward_state(const ae_recurrent_t* h, const void* Q, const void* K, const void* V,
                                       const void* h_in, void* O, void* h_out, void* workspace, size_t workspace_bytes,
                                       hipStream_t stream) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_forward: null handle");
  if (!Q || !K || !V || !O) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_forward: null pointer");
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O | (uintptr_t)h_in | (uintptr_t)h_out) & 15)
    return fail(AE_ERR_INVALID_ARG, "ae_recurrent_forward: Q, K, V, O and the states must be 16-byte aligned");
  if (O == Q || O == K || O == V) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_forward: O aliases an input");
  if (h_out && (h_out == O || h_out == Q || h_out == K || h_out == V || h_out == workspace))
    return fail(AE_ERR_INVALID_ARG, "ae_recurrent_forward: the final state aliases another buffer");
  if (h_in && (h_in == O || h_in == workspace)) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_forward: the initial state aliases an output");
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < h->ws_bytes)
    return fail(AE_ERR_INVALID_ARG, "ae_recurrent_forward: workspace missing, not 256-byte aligned, or smaller than %zu bytes", h->ws_bytes);
  if (workspace == O || workspace == Q || workspace == K || workspace == V)
    return fail(AE_ERR_INVALID_ARG, "ae_recurrent_forward: workspace aliases another buffer");
  const ae_recurrent_desc_t& d = h->desc;
  const int64_t L = d.L, state_elems = (int64_t)d.D_qk * d.D_v;
  if (h->single_pass || h->nseg > 1) {
    // enough (batch, head) pairs to fill the device with one workgroup each: the kernel of the gated pattern with a
    // constant decay per head -- state on chip, Q, K, V read once, the workspace untouched; or few pairs and a long
    // sequence: the same kernel on segments of the sequence, whose states pass through the workspace
    ae::GatedParams g;
    g.Q = static_cast<const __bf16*>(Q);
    g.K = static_cast<const __bf16*>(K);
    g.V = static_cast<const __bf16*>(V);
    g.log_decay = nullptr;
    g.key_gate = nullptr;
    g.h_in = static_cast<const float*>(h_in);
    g.h_out = static_cast<float*>(h_out);
    g.O = O;
    g.B = d.B;
    g.H = g.H_qk = d.H;
    g.L = d.L;
    g.scale = d.scale;
    g.out_bf16 = d.out_dtype == AE_OUT_BF16;
    const hipError_t e = h->nseg > 1 ? launch_gated_segmented(g, h->decay, d.D_qk, d.D_v, h->nseg, h->seg_len, workspace, stream)
                                     : ae::launch_gated_recurrent(g, h->decay, d.D_qk, d.D_v, stream);
    if (e != hipSuccess) return fail(AE_ERR_HIP, "ae_recurrent_forward: %s", hipGetErrorString(e));
    return AE_OK;
  }
  ae::RecParams p;
  p.K = static_cast<const __bf16*>(K);
  p.V = static_cast<const __bf16*>(V);
  p.HT = static_cast<__bf16*>(workspace);
  p.h_in = static_cast<const float*>(h_in);
  p.h_out = static_cast<float*>(h_out);
  p.B = d.B;
  p.H = d.H;
  p.L = d.L;
  p.chunk = d.chunk;
  p.n_chunks = h->n_chunks;
  if (h->n_chunks > 1 || h_in || h_out) {
    // the state in front of every chunk (slot c of a (batch, head): chunk c; slot 0 only from h_in): one workgroup
    // per (batch, head, slice of D_v) walks the chunks
    const hipError_t e = ae::launch_recurrent_states(p, h->decay, d.D_qk, d.D_v, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(AE_ERR_HIP, "ae_recurrent_forward: %s", hipGetErrorString(e));
  }
  // O = read-out of the carried state + decay-masked causal attention inside the chunk, in one pass of the
  // parallel-pattern kernel over the chunks
  for (int b = 0; b < d.B; b += h->fold) {
    const int64_t e0 = (int64_t)b * d.H * L;  // first row of this launch's (batch, head) slabs
    for (int part = 0; part < 2; ++part) {
      const ae_attn_t* a = part ? h->tail : h->full;
      if (!a) continue;
      const int64_t r0 = e0 + (part ? (int64_t)h->n_full * d.chunk : 0);
      CarriedState cs;  // batch entry c' of the launch is chunk c' (part 0) or chunk n_full (the short last one)
      cs.first_batch = (part == 0 && !h_in) ? 1 : 0;  // chunk 0 has a state in front of it only if the caller gave one
      // (the kernel counts slots from the first batch entry that has one)
      cs.state = p.HT + ((int64_t)b * d.H * h->n_chunks + (part ? h->n_full : cs.first_batch)) * state_elems;
      cs.batch_stride = state_elems;
      cs.head_stride = (int64_t)h->n_chunks * state_elems;
      const bool has_state = part == 0 ? (h->n_full > 1 || h_in) : (h->n_full > 0 || h_in);
      const ae_status_t st = forward_impl(a, static_cast<const __bf16*>(Q) + r0 * d.D_qk, static_cast<const __bf16*>(K) + r0 * d.D_qk,
                                          static_cast<const __bf16*>(V) + r0 * d.D_v,
                                          static_cast<char*>(O) + r0 * d.D_v * (d.out_dtype == AE_OUT_BF16 ? 2 : 4), nullptr,
                                          stream, nullptr, 0, nullptr, has_state ? &cs : nullptr);
      if (st != AE_OK) return st;
    }
  }
  return AE_OK;
}

ae_status_t ae_recurrent_forward(const ae_recurrent_t* h, const void* Q, const void* K, const void* V, void* O,
                                 void* workspace, size_t workspace_bytes, hipStream_t stream) {
  return ae_recurrent_forward_state(h, Q, K, V, nullptr, O, nullptr, workspace, workspace_bytes, stream);
}

ae_status_t ae_recurrent_step(const ae_recurrent_t* h, const void* q, const void* k, const void* v, void* state, void* o,
                              hipStream_t stream) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_step: null handle");
  if (!q || !k || !v || !state || !o) return fail(AE_ERR_INVALID_ARG, "ae_recurrent_step: null pointer");
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)state | (uintptr_t)o) & 15)
    return fail(AE_ERR_INVALID_ARG, "ae_recurrent_step: pointers must be 16-byte aligned");
  if (o == q || o == k || o == v || o == state || state == q || state == k || state == v)
    return fail(AE_ERR_INVALID_ARG, "ae_recurrent_step: an output aliases another buffer");
  ae::RecStepParams p;
  p.q = static_cast<const __bf16*>(q);
  p.k = static_cast<const __bf16*>(k);
  p.v = static_cast<const __bf16*>(v);
  p.state = static_cast<float*>(state);
  p.o = static_cast<float*>(o);
  p.B = h->desc.B;
  p.H = h->desc.H;
  p.scale = h->desc.scale;
  const hipError_t e = ae::launch_recurrent_step(p, h->decay, h->desc.D_qk, h->desc.D_v, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(AE_ERR_HIP, "ae_recurrent_step: %s", hipGetErrorString(e));
  return AE_OK;
}

ae_status_t ae_recurrent_destroy(ae_recurrent_t* h) {
  if (h) {
    ae_attn_destroy(h->full);
    ae_attn_destroy(h->tail);
    delete h;
  }
  return AE_OK;
}

}  // extern "C"

// ---- recurrent pattern with per-token gates: one kernel, state on chip ------------------------------------
struct ae_gated {
  ae_gated_desc_t desc;
  // ae_gated_forward_segmented: the walk of a (batch, head) cut into nseg segments of seg_len tokens where the
  // (batch, head) pairs alone would leave most compute units idle; 1: not cut
  int nseg, seg_len;
};

extern "C" {

ae_status_t ae_gated_create(const ae_gated_desc_t* d, ae_gated_t** out) {
  if (out) *out = nullptr;
  if (!d || !out) return fail(AE_ERR_INVALID_ARG, "ae_gated_create: null argument");
  if (d->B < 1 || d->H < 1 || d->H_qk < 1 || d->L < 1) return fail(AE_ERR_INVALID_ARG, "ae_gated_create: B, H, H_qk, L must be >= 1");
  if (d->H % d->H_qk != 0) return fail(AE_ERR_INVALID_ARG, "ae_gated_create: H (%d) is not a multiple of H_qk (%d)", d->H, d->H_qk);
  if (!std::isfinite(d->scale) || d->scale == 0.f) return fail(AE_ERR_INVALID_ARG, "ae_gated_create: scale must be finite and non-zero");
  if (d->out_dtype != AE_OUT_F32 && d->out_dtype != AE_OUT_BF16) return fail(AE_ERR_INVALID_ARG, "ae_gated_create: unknown out_dtype");
  if (!ae::gated_supported(d->D_qk, d->D_v))
    return fail(AE_ERR_UNSUPPORTED, "ae_gated_create: head dims %d/%d not built (D_qk and D_v each 64 or 128)", d->D_qk, d->D_v);
  if ((int64_t)d->L * std::max(d->D_qk, d->D_v) * 2 >= (int64_t)1 << 32)
    return fail(AE_ERR_UNSUPPORTED, "ae_gated_create: one (batch, head) slab must span less than 4 GiB");
  if ((int64_t)d->B * d->H > 0x7fffffffLL) return fail(AE_ERR_UNSUPPORTED, "ae_gated_create: too many (batch, head) pairs");
  ae_gated* h = new (std::nothrow) ae_gated;
  if (!h) return fail(AE_ERR_NOMEM, "ae_gated_create: out of host memory");
  h->desc = *d;
  {
    // (two heads of a group share a workgroup at 128/64, see launch_gated_recurrent)
    const bool pairs = d->D_qk == 128 && d->D_v == 64 && (d->H / d->H_qk) % 2 == 0;
    gated_segments((int64_t)d->B * d->H / (pairs ? 2 : 1), d->L, &h->nseg, &h->seg_len);
  }
  *out = h;
  return AE_OK;
}

}  // extern "C"

static size_t gated_forward_ws(const ae_gated* h) {
  return gated_segments_ws(h->desc.B, h->desc.H, h->nseg, h->desc.D_qk, h->desc.D_v);
}

static ae_status_t gated_forward_impl(const ae_gated_t* h, const void* Q, const void* K, const void* V, const void* log_decay,
                                      const void* key_gate, const void* h_in, void* O, void* h_out, void* workspace,
                                      size_t workspace_bytes, bool segmented, hipStream_t stream) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_gated_forward: null handle");
  if (!Q || !K || !V || !log_decay || !O) return fail(AE_ERR_INVALID_ARG, "ae_gated_forward: null pointer");
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O | (uintptr_t)h_in | (uintptr_t)h_out) & 15)
    return fail(AE_ERR_INVALID_ARG, "ae_gated_forward: Q, K, V, O and the states must be 16-byte aligned");
  if (((uintptr_t)log_decay | (uintptr_t)key_gate) & 3) return fail(AE_ERR_INVALID_ARG, "ae_gated_forward: the gates must be 4-byte aligned");
  const void* ins[] = {Q, K, V, log_decay, key_gate, h_in};
  for (const void* in : ins)
    if (in && (in == O || (h_out && in == h_out && in != h_in)))
      return fail(AE_ERR_INVALID_ARG, "ae_gated_forward: an output aliases an input");
  if (h_out && h_out == O) return fail(AE_ERR_INVALID_ARG, "ae_gated_forward: the final state aliases O");
  const ae_gated_desc_t& d = h->desc;
  ae::GatedParams p;
  p.Q = static_cast<const __bf16*>(Q);
  p.K = static_cast<const __bf16*>(K);
  p.V = static_cast<const __bf16*>(V);
  p.log_decay = static_cast<const float*>(log_decay);
  p.key_gate = static_cast<const float*>(key_gate);
  p.h_in = static_cast<const float*>(h_in);
  p.h_out = static_cast<float*>(h_out);
  p.O = O;
  p.B = d.B;
  p.H = d.H;
  p.H_qk = d.H_qk;
  p.L = d.L;
  p.scale = d.scale;
  p.out_bf16 = d.out_dtype == AE_OUT_BF16;
  static const ae::DecayTable no_table = {};
  hipError_t e;
  if (segmented && h->nseg > 1) {
    const size_t need = gated_forward_ws(h);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)
      return fail(AE_ERR_INVALID_ARG, "ae_gated_forward_segmented: workspace missing, not 256-byte aligned, or smaller than %zu bytes", need);
    for (const void* in : ins)
      if (in == workspace) return fail(AE_ERR_INVALID_ARG, "ae_gated_forward_segmented: the workspace aliases an input");
    if (workspace == O || workspace == h_out) return fail(AE_ERR_INVALID_ARG, "ae_gated_forward_segmented: the workspace aliases an output");
    e = launch_gated_segmented(p, no_table, d.D_qk, d.D_v, h->nseg, h->seg_len, workspace, stream);
  } else {
    e = ae::launch_gated_recurrent(p, no_table, d.D_qk, d.D_v, stream);
  }
  if (e != hipSuccess) return fail(AE_ERR_HIP, "ae_gated_forward: %s", hipGetErrorString(e));
  return AE_OK;
}

extern "C" {

ae_status_t ae_gated_forward(const ae_gated_t* h, const void* Q, const void* K, const void* V, const void* log_decay,
                             const void* key_gate, const void* h_in, void* O, void* h_out, hipStream_t stream) {
  return gated_forward_impl(h, Q, K, V, log_decay, key_gate, h_in, O, h_out, nullptr, 0, false, stream);
}

ae_status_t ae_gated_workspace_bytes(const ae_gated_t* h, size_t* bytes) {
  if (!h || !bytes) return fail(AE_ERR_INVALID_ARG, "ae_gated_workspace_bytes: null argument");
  *bytes = gated_forward_ws(h);
  return AE_OK;
}

ae_status_t ae_gated_forward_segmented(const ae_gated_t* h, const void* Q, const void* K, const void* V, const void* log_decay,
                                       const void* key_gate, const void* h_in, void* O, void* h_out, void* workspace,
                                       size_t workspace_bytes, hipStream_t stream) {
  return gated_forward_impl(h, Q, K, V, log_decay, key_gate, h_in, O, h_out, workspace, workspace_bytes, true, stream);
}

// Workspace of the backward pass: the per-token terms of the decay gradient, fp32 [B, H, L]; and, where value heads
// share q/k heads, the gradients of q and of the gated key per value head, fp32 [B, H, L, D_qk] each.
// Where the forward pass would cut the walks into segments, so do the three walks of the backward pass: the segments'
// states (one set, used by the walks in turn) follow.
static size_t gated_backward_ws(const ae_gated* h, size_t* per_head_off, size_t* seg_off) {
  const ae_gated_desc_t& d = h->desc;
  const size_t rows = ((size_t)d.B * d.H * d.L * 4 + 255) & ~(size_t)255;
  const size_t per_head = d.H != d.H_qk ? 2 * (size_t)d.B * d.H * d.L * d.D_qk * 4 : 0;
  if (per_head_off) *per_head_off = rows;
  if (seg_off) *seg_off = rows + per_head;
  return rows + per_head + gated_segments_ws(d.B, d.H, h->nseg, d.D_qk, d.D_v);
}

ae_status_t ae_gated_backward_workspace_bytes(const ae_gated_t* h, size_t* bytes) {
  if (!h || !bytes) return fail(AE_ERR_INVALID_ARG, "ae_gated_backward_workspace_bytes: null argument");
  *bytes = gated_backward_ws(h, nullptr, nullptr);
  return AE_OK;
}

ae_status_t ae_gated_backward(const ae_gated_t* h, const void* Q, const void* K, const void* V, const void* log_decay,
                              const void* key_gate, const void* dO, void* dQ, void* dK, void* dV, void* dlog_decay,
                              void* dkey_gate, void* workspace, size_t workspace_bytes, hipStream_t stream) {
  if (!h) return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: null handle");
  if (!Q || !K || !V || !log_decay || !dO || !dQ || !dK || !dV || !dlog_decay)
    return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: null pointer");
  if (key_gate && !dkey_gate) return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: a key gate needs a buffer for its gradient");
  if (!key_gate && dkey_gate) return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: dkey_gate without a key gate");
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)dO | (uintptr_t)dQ | (uintptr_t)dK | (uintptr_t)dV) & 15)
    return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: Q, K, V, dO, dQ, dK, dV must be 16-byte aligned");
  if (((uintptr_t)log_decay | (uintptr_t)key_gate | (uintptr_t)dlog_decay | (uintptr_t)dkey_gate) & 3)
    return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: the gates and their gradients must be 4-byte aligned");
  const ae_gated_desc_t& d = h->desc;
  size_t per_head_off = 0, seg_off = 0;
  const size_t need = gated_backward_ws(h, &per_head_off, &seg_off);
  void* seg_ws = static_cast<char*>(workspace) + seg_off;
  auto walk = [&](const ae::GatedParams& g, int dqk, int dv) {
    static const ae::DecayTable none = {};
    return h->nseg > 1 ? launch_gated_segmented(g, none, dqk, dv, h->nseg, h->seg_len, seg_ws, stream)
                       : ae::launch_gated_recurrent(g, none, dqk, dv, stream);
  };
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need)
    return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: workspace missing, not 256-byte aligned, or smaller than %zu bytes", need);
  const void* ins[] = {Q, K, V, log_decay, key_gate, dO};
  void* outs[] = {dQ, dK, dV, dlog_decay, dkey_gate, workspace};
  for (int a = 0; a < 6; ++a) {
    if (!outs[a]) continue;
    for (const void* in : ins)
      if (in == outs[a]) return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: an output aliases an input");
    for (int c = a + 1; c < 6; ++c)
      if (outs[c] == outs[a]) return fail(AE_ERR_INVALID_ARG, "ae_gated_backward: two outputs alias");
  }
  const bool grouped = d.H != d.H_qk;
  float* dB = static_cast<float*>(workspace);
  float* dQu = grouped ? reinterpret_cast<float*>(static_cast<char*>(workspace) + per_head_off) : static_cast<float*>(dQ);
  float* X = grouped ? dQu + (size_t)d.B * d.H * d.L * d.D_qk : static_cast<float*>(dK);
  static const ae::DecayTable no_table = {};
  // The three sums of the backward pass are the forward recurrence itself on other operands (see include/ae_attn.h):
  ae::GatedParams p;
  p.h_in = nullptr;
  p.h_out = nullptr;
  p.B = d.B;
  p.H = d.H;
  p.L = d.L;
  p.scale = d.scale;
  p.out_bf16 = 0;
  p.log_decay = static_cast<const float*>(log_decay);
  // (1) dq_i = scale sum_{j <= i} A_ij g_j (dO_i . v_j) k_j: queries dO, keys V (both per value head), values K
  p.Q = static_cast<const __bf16*>(dO);
  p.K = static_cast<const __bf16*>(V);
  p.V = static_cast<const __bf16*>(K);
  p.H_qk = d.H;
  p.H_v = d.H_qk;
  p.key_gate = static_cast<const float*>(key_gate);
  p.gate_on_output = 0;
  p.reverse = 0;
  p.O = dQu;
  hipError_t e = walk(p, d.D_v, d.D_qk);
  // (2) x_j = scale sum_{i >= j} A_ij (v_j . dO_i) q_i, walking backwards: queries V, keys dO, values Q, no gate
  if (e == hipSuccess) {
    p.Q = static_cast<const __bf16*>(V);
    p.K = static_cast<const __bf16*>(dO);
    p.V = static_cast<const __bf16*>(Q);
    p.key_gate = nullptr;
    p.reverse = 1;
    p.O = X;
    e = walk(p, d.D_v, d.D_qk);
  }
  // (3) dv_j = g_j scale sum_{i >= j} A_ij (k_j . q_i) dO_i, walking backwards: queries K, keys Q, values dO
  if (e == hipSuccess) {
    p.Q = static_cast<const __bf16*>(K);
    p.K = static_cast<const __bf16*>(Q);
    p.V = static_cast<const __bf16*>(dO);
    p.H_qk = d.H_qk;
    p.H_v = d.H;
    p.key_gate = static_cast<const float*>(key_gate);
    p.gate_on_output = key_gate ? 1 : 0;
    p.O = dV;
    e = walk(p, d.D_qk, d.D_v);
  }
  if (e == hipSuccess) {
    ae::GatedBwdEpilogueParams q;
    q.Q = static_cast<const __bf16*>(Q);
    q.K = static_cast<const __bf16*>(K);
    q.dQu = dQu;
    q.X = X;
    q.key_gate = static_cast<const float*>(key_gate);
    q.dQ = static_cast<float*>(dQ);
    q.dK = static_cast<float*>(dK);
    q.dkey_gate = static_cast<float*>(dkey_gate);
    q.dB = dB;
    q.dlog_decay = static_cast<float*>(dlog_decay);
    q.B = d.B;
    q.H = d.H;
    q.H_qk = d.H_qk;
    q.L = d.L;
    e = ae::launch_gated_backward_epilogue(q, d.D_qk, stream);
  }
  if (e != hipSuccess) return fail(AE_ERR_HIP, "ae_gated_backward: %s", hipGetErrorString(e));
  return AE_OK;
}

ae_status_t ae_gated_destroy(ae_gated_t* h) {
  delete h;
  return AE_OK;
}

}  // extern "C"
