// Kernel table shared by the per-head-dim instantiation units and the C ABI.
#pragma once
#include "attn_kernel.hpp"

namespace ae {

typedef hipError_t (*launch_fn)(const Params&, const DecayTable&, int grid, hipStream_t);

struct KernelEntry {
  int dqk, dv, norm, mod, mask;  // mask: 0 none, 1 causal, 2 sliding window
  int fold;                      // Cfg::FOLD: scale folded into Q, exponent offset in the accumulator's initial value
  int block_m, block_n, threads, lds_bytes;
  launch_fn launch;
  const char* name;
};

template <class C>
hipError_t launch_cfg(const Params& p, const DecayTable& dt, int grid, hipStream_t s) {
  hipLaunchKernelGGL(attn_fwd_kernel<C>, dim3(grid), dim3(C::THREADS), 0, s, p, dt);
  return hipGetLastError();
}

template <class C>
constexpr KernelEntry make_entry(const char* name) {
  return KernelEntry{C::DQK, C::DV, C::NORM, C::MOD, C::MASK, C::FOLD ? 1 : 0,
                     C::BLOCK_M, C::BLOCK_N, C::THREADS, C::LDS_BYTES, &launch_cfg<C>, name};
}

// One row of the tile-shape table: for head dims (DQK, DV) and mask MASK (false / 0: none,
// true / 1: causal, 2: sliding window) the workgroup has WAVES wavefronts of 32 query rows each.
#define AE_ENTRY(DQK, DV, NORM, MOD, MASK, WAVES)     \
  make_entry<Cfg<DQK, DV, NORM, MOD, MASK, WAVES>>(   \
      "attn_fwd<" #DQK "," #DV "," #NORM "," #MOD "," #MASK "," #WAVES ">")
#define AE_ENTRY_FOLD(DQK, DV, NORM, MASK, WAVES)             \
  make_entry<Cfg<DQK, DV, NORM, MOD_PLAIN, MASK, WAVES, 1>>(  \
      "attn_fwd<" #DQK "," #DV "," #NORM ",MOD_PLAIN," #MASK "," #WAVES ",FOLD>")

// Every (norm, mod) pair the library supports, for one (DQK, DV) and one tile
// shape (WAVES) per mask value (SHAPE_NC unmasked, SHAPE_C causal and sliding window;
// the sliding window comes with softmax, sigmoid and no normalization).
#define AE_ENTRIES_FOR_DIMS(DQK, DV, SHAPE_NC, SHAPE_C)            \
  AE_ENTRY(DQK, DV, NORM_SOFTMAX, MOD_PLAIN, false, SHAPE_NC),    \
  AE_ENTRY(DQK, DV, NORM_SIGMOID, MOD_PLAIN, false, SHAPE_NC),    \
  AE_ENTRY(DQK, DV, NORM_ABSSUM, MOD_PLAIN, false, SHAPE_NC),     \
  AE_ENTRY(DQK, DV, NORM_ABS_OF_SUM, MOD_PLAIN, false, SHAPE_NC), \
  AE_ENTRY(DQK, DV, NORM_NONE, MOD_PLAIN, false, SHAPE_NC),       \
  AE_ENTRY(DQK, DV, NORM_NONE, MOD_RELU, false, SHAPE_NC),        \
  AE_ENTRY(DQK, DV, NORM_SOFTMAX, MOD_PLAIN, true, SHAPE_C),      \
  AE_ENTRY(DQK, DV, NORM_SIGMOID, MOD_PLAIN, true, SHAPE_C),      \
  AE_ENTRY(DQK, DV, NORM_ABSSUM, MOD_PLAIN, true, SHAPE_C),       \
  AE_ENTRY(DQK, DV, NORM_ABS_OF_SUM, MOD_PLAIN, true, SHAPE_C),   \
  AE_ENTRY(DQK, DV, NORM_NONE, MOD_PLAIN, true, SHAPE_C),         \
  AE_ENTRY(DQK, DV, NORM_NONE, MOD_RELU, true, SHAPE_C),          \
  AE_ENTRY(DQK, DV, NORM_ABSSUM, MOD_DECAY, true, SHAPE_C),       \
  AE_ENTRY(DQK, DV, NORM_ABS_OF_SUM, MOD_DECAY, true, SHAPE_C),   \
  AE_ENTRY(DQK, DV, NORM_NONE, MOD_DECAY, true, SHAPE_C),          \
  AE_ENTRY(DQK, DV, NORM_SOFTMAX, MOD_PLAIN, 2, SHAPE_C),         \
  AE_ENTRY(DQK, DV, NORM_SIGMOID, MOD_PLAIN, 2, SHAPE_C),         \
  AE_ENTRY(DQK, DV, NORM_NONE, MOD_PLAIN, 2, SHAPE_C)

// The FOLD forms of softmax and sigmoid (see Cfg), for the head dims whose kernels have the 16 registers of
// the accumulator's initial value to spare (not 128/256: two waves per SIMD leave 256 registers).
#define AE_ENTRIES_FOLD(DQK, DV, SHAPE_NC, SHAPE_C)               \
  AE_ENTRY_FOLD(DQK, DV, NORM_SOFTMAX, false, SHAPE_NC),          \
  AE_ENTRY_FOLD(DQK, DV, NORM_SIGMOID, false, SHAPE_NC),          \
  AE_ENTRY_FOLD(DQK, DV, NORM_SOFTMAX, true, SHAPE_C),            \
  AE_ENTRY_FOLD(DQK, DV, NORM_SIGMOID, true, SHAPE_C),            \
  AE_ENTRY_FOLD(DQK, DV, NORM_SOFTMAX, 2, SHAPE_C),               \
  AE_ENTRY_FOLD(DQK, DV, NORM_SIGMOID, 2, SHAPE_C)

// The additive bias tensor (softmax, sigmoid, no normalization; unmasked and causal), for the head
// dims whose kernels have registers to spare for the prefetched bias values.
#define AE_ENTRIES_BIAS_TENSOR(DQK, DV, SHAPE_NC, SHAPE_C)        \
  AE_ENTRY(DQK, DV, NORM_SOFTMAX, MOD_BIAS_T, false, SHAPE_NC),   \
  AE_ENTRY(DQK, DV, NORM_SIGMOID, MOD_BIAS_T, false, SHAPE_NC),   \
  AE_ENTRY(DQK, DV, NORM_NONE, MOD_BIAS_T, false, SHAPE_NC),      \
  AE_ENTRY(DQK, DV, NORM_SOFTMAX, MOD_BIAS_T, true, SHAPE_C),     \
  AE_ENTRY(DQK, DV, NORM_SIGMOID, MOD_BIAS_T, true, SHAPE_C),     \
  AE_ENTRY(DQK, DV, NORM_NONE, MOD_BIAS_T, true, SHAPE_C)

const KernelEntry* table_64_64(int* n);
const KernelEntry* table_128_128(int* n);
const KernelEntry* table_128_256(int* n);
const KernelEntry* table_192_128(int* n);
const KernelEntry* table_256_128(int* n);

}  // namespace ae
