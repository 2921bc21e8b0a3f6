// Differential attention: two softmax streams over one V, subtraction with lambda, optional
// per-head RMSNorm (differential-attention listing, Sec. 3), bf16.
#include "fl_registry.hpp"
namespace fl {
// 8 waves: waves 0-3 run stream 0, waves 4-7 stream 1 of the same 128 query rows
#define E(D, DV, MASK, EPI) bf16_entry<D, DV, 8, 1, (D == 128 ? 32 : 64), 2, kModNone, MASK, 0, true, EPI>()
static const KernelEntry kEntries[] = {
    E(64, 128, kMaskCausal, kEpiRms), E(64, 128, kMaskCausal, 0), E(64, 128, 0, kEpiRms), E(64, 128, 0, 0),
    E(128, 128, kMaskCausal, kEpiRms), E(128, 128, kMaskCausal, 0),
    E(64, 64, kMaskCausal, kEpiRms), E(64, 64, kMaskCausal, 0),
    E(64, 64, 0, 0), E(128, 128, 0, 0),   // the paper's DiffAttn benchmark shapes: no mask, no normalisation
    bf16_entry<64, 64, 8, 1, 32, 4, kModNone, 0, 0, true, 0>(),   // short key loops: two workgroups per CU
};
#undef E
const KernelEntry* entries_diff(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
