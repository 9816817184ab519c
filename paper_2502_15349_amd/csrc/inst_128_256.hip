// Kernel instantiations and tile shapes for D_qk = 128, D_v = 256.
#include "dispatch.hpp"

// tile shape: wavefronts per workgroup
#ifndef AE_SHAPE_128_256_NC
#define AE_SHAPE_128_256_NC 8
#endif
#ifndef AE_SHAPE_128_256_C
#define AE_SHAPE_128_256_C 8
#endif

namespace ae {
static const KernelEntry kTable[] = {AE_ENTRIES_FOR_DIMS(128, 256, AE_SHAPE_128_256_NC, AE_SHAPE_128_256_C)};

const KernelEntry* table_128_256(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}
}  // namespace ae
