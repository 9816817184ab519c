// Kernel instantiations and tile shapes for D_qk = 128, D_v = 128.
#include "dispatch.hpp"

namespace ae {
static const KernelEntry kTable[] = {
    //                  D_qk D_v  non-causal: waves, q-blocks/wave   causal: waves, q-blocks/wave
    AE_ENTRIES_FOR_DIMS(128, 128, 8, 1, 8, 1)};

const KernelEntry* table_128_128(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}
}  // namespace ae
