// Kernel instantiations and tile shapes for D_qk = 64, D_v = 64.
#include "dispatch.hpp"

// tile shape: wavefronts per workgroup
#ifndef AE_SHAPE_64_64_NC
#define AE_SHAPE_64_64_NC 8
#endif
#ifndef AE_SHAPE_64_64_C
#define AE_SHAPE_64_64_C 8
#endif

namespace ae {
static const KernelEntry kTable[] = {AE_ENTRIES_FOR_DIMS(64, 64, AE_SHAPE_64_64_NC, AE_SHAPE_64_64_C),
                                     AE_ENTRIES_BIAS_TENSOR(64, 64, AE_SHAPE_64_64_NC, AE_SHAPE_64_64_C),
                                     AE_ENTRIES_FOLD(64, 64, AE_SHAPE_64_64_NC, AE_SHAPE_64_64_C)};

const KernelEntry* table_64_64(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}
}  // namespace ae
