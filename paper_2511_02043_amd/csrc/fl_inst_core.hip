// Plain and causal softmax attention, bf16, every supported head dim, in the kernel shapes the
// tuning knobs can select.
#include "fl_registry.hpp"
namespace fl {
#define E(D, NW, BN, MASK) bf16_entry<D, D, NW, BN, kModNone, MASK, 0, false, 0>()
static const KernelEntry kEntries[] = {
    E(128, 8, 32, 0), E(128, 8, 32, kMaskCausal), E(128, 4, 32, 0), E(128, 4, 32, kMaskCausal),
    E(128, 8, 64, 0), E(128, 8, 64, kMaskCausal), E(128, 4, 64, 0), E(128, 4, 64, kMaskCausal),
    E(64, 8, 64, 0),  E(64, 8, 64, kMaskCausal),  E(64, 4, 64, 0),  E(64, 4, 64, kMaskCausal),
    E(32, 8, 64, 0),  E(32, 8, 64, kMaskCausal),  E(32, 4, 64, 0),  E(32, 4, 64, kMaskCausal),
};
#undef E
const KernelEntry* entries_core(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
