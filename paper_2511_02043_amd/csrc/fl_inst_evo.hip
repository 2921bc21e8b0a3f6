// Evoformer-style attention: one or two additive biases (pair bias broadcast over the row axis,
// per-row key bias) and the sigmoid output gate (Sec. 4.1, "Evoformer"), bf16.  The gate alone
// (no bias) is the column-wise gated self-attention named in Sec. 1.
#include "fl_registry.hpp"
namespace fl {
// D = 32 is bound by the vector work per score, not by registers: 32-key tiles and four waves per
// SIMD measured best on the Evoformer benchmark shape.
#define E(D, NBIAS, EPI, BN, WPE) bf16_entry<D, D, 4, 1, BN, WPE, kModNone, 0, NBIAS, false, EPI>()
static const KernelEntry kEntries[] = {
    E(32, 1, kEpiGate, 32, 4), E(32, 2, kEpiGate, 32, 4), E(32, 1, 0, 32, 4), E(32, 2, 0, 32, 4),
    E(32, 1, kEpiGate, 64, 2),
    E(64, 1, kEpiGate, 64, 2), E(64, 2, kEpiGate, 64, 2),
    // short key loops at D = 64 (the paper's 256 x 256 shape: 71.7 against 78.5 us); four waves per SIMD spill here
    E(64, 1, kEpiGate, 32, 3), E(64, 2, kEpiGate, 32, 3), E(128, 1, kEpiGate, 32, 2), E(128, 2, kEpiGate, 32, 2),
    E(32, 0, kEpiGate, 32, 4), E(64, 0, kEpiGate, 64, 2), E(128, 0, kEpiGate, 64, 2),
};
#undef E
const KernelEntry* entries_evo(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
