// Kernel instantiations for D_qk = 256, D_v = 128: the retention variants (Table 2, "Retention Parallel": 256 / 512,
// whose D_v = 512 runs as four launches over 128 value columns each, see ae_attn_create).
#include "dispatch.hpp"

namespace ae {
static const KernelEntry kTable[] = {AE_ENTRY(256, 128, NORM_ABSSUM, MOD_DECAY, true, 8), AE_ENTRY(256, 128, NORM_ABS_OF_SUM, MOD_DECAY, true, 8),
                                     AE_ENTRY(256, 128, NORM_NONE, MOD_DECAY, true, 8)};

const KernelEntry* table_256_128(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}
}  // namespace ae
