// Kernel instantiations and tile shapes for D_qk = 192, D_v = 128.
#include "dispatch.hpp"

// tile shape: wavefronts per workgroup
#ifndef AE_SHAPE_192_128_NC
#define AE_SHAPE_192_128_NC 8
#endif
#ifndef AE_SHAPE_192_128_C
#define AE_SHAPE_192_128_C 8
#endif

namespace ae {
static const KernelEntry kTable[] = {AE_ENTRIES_FOR_DIMS(192, 128, AE_SHAPE_192_128_NC, AE_SHAPE_192_128_C),
                                     AE_ENTRIES_BIAS_TENSOR(192, 128, AE_SHAPE_192_128_NC, AE_SHAPE_192_128_C),
                                     AE_ENTRIES_FOLD(192, 128, AE_SHAPE_192_128_NC, AE_SHAPE_192_128_C)};

const KernelEntry* table_192_128(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}
}  // namespace ae
