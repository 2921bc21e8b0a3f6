// Evoformer-style attention: one or two additive biases (pair bias broadcast over the row axis,
// per-row key bias) and the sigmoid output gate (Sec. 4.1, "Evoformer"), bf16.
#include "fl_registry.hpp"
namespace fl {
#define E(D, NBIAS, EPI) bf16_entry<D, D, 4, 1, 64, 2, kModNone, 0, NBIAS, false, EPI>()
static const KernelEntry kEntries[] = {
    E(32, 1, kEpiGate), E(32, 2, kEpiGate), E(32, 1, 0), E(32, 2, 0),
    E(64, 1, kEpiGate), E(64, 2, kEpiGate), E(128, 1, kEpiGate), E(128, 2, kEpiGate),
};
#undef E
const KernelEntry* entries_evo(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
