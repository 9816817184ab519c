// Kernel instantiations and tile shapes for D_qk = 64, D_v = 64.
#include "dispatch.hpp"

namespace ae {
static const KernelEntry kTable[] = {
    //                  D_qk D_v  non-causal: waves, q-blocks/wave   causal: waves, q-blocks/wave
    AE_ENTRIES_FOR_DIMS(64, 64, 8, 1, 8, 1)};

const KernelEntry* table_64_64(int* n) {
  *n = (int)(sizeof(kTable) / sizeof(kTable[0]));
  return kTable;
}
}  // namespace ae
