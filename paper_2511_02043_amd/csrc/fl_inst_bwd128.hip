// Backward kernels, head dim 128.  The dK/dV kernel keeps K, V and both accumulators of its 32
// keys in registers and runs one wave per SIMD.
#include "fl_bwd_registry.hpp"
namespace fl {
#define E(MOD, MASK) bwd_entry<128, MOD, MASK, 64, 2, 64, 2, true>()
constexpr uint32_t CW = kMaskCausal | kMaskWindow;
static const BwdEntry kEntries[] = {
    E(kModNone, 0),  E(kModNone, kMaskCausal), E(kModAlibi, 0), E(kModSoftcap, 0), E(kModNone, CW),
    E(kModNone, CW | kMaskDoc), E(kModNone, kMaskDoc), E(kModNone, kMaskCausal | kMaskDoc), E(kModNone, kMaskPrefix),
    // additive biases: plain and causal, one or two biases
    bwd_entry<128, kModNone, 0, 64, 2, 64, 2, true, 1>(), bwd_entry<128, kModNone, 0, 64, 2, 64, 2, true, 2>(),
    bwd_entry<128, kModNone, kMaskCausal, 64, 2, 64, 2, true, 1>(), bwd_entry<128, kModNone, kMaskCausal, 64, 2, 64, 2, true, 2>(),
};
#undef E
const BwdEntry* entries_bwd128(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
