// Backward kernels, head dim 64: the variants of the forward pass that have no bias, gate or
// second softmax stream.
#include "fl_bwd_registry.hpp"
namespace fl {
#define E(MOD, MASK) bwd_entry<64, MOD, MASK, 64, 2, 64, 2, false>()
constexpr uint32_t CW = kMaskCausal | kMaskWindow;
static const BwdEntry kEntries[] = {
    E(kModNone, 0),        E(kModNone, kMaskCausal),        E(kModAlibi, 0),       E(kModAlibi, kMaskCausal),
    E(kModSoftcap, 0),     E(kModSoftcap, kMaskCausal),     E(kModNone, CW),       E(kModNone, CW | kMaskDoc),
    E(kModNone, kMaskDoc), E(kModNone, kMaskCausal | kMaskDoc), E(kModNone, kMaskPrefix),
    E(kModNone, kMaskPrefix | kMaskDoc),
};
#undef E
const BwdEntry* entries_bwd64(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
