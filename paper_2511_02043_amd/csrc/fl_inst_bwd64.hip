// Backward kernels, head dim 64: the variants of the forward pass that have no bias, gate or
// second softmax stream.
#include "fl_bwd_registry.hpp"
namespace fl {
constexpr uint32_t CW = kMaskCausal | kMaskWindow;
// The dQ kernel needs 128 - 165 registers at this head dim: three waves per SIMD instead of two measured 4 - 18 %
// faster on whole backward calls; the three variants that fit 128 registers run four.
constexpr int dq_waves(int mod, uint32_t mask) {
  return mod == kModNone && (mask == kMaskCausal || mask == CW || mask == kMaskPrefix) ? 4 : 3;
}
#define E(MOD, MASK) bwd_entry<64, MOD, MASK, 64, dq_waves(MOD, MASK), 64, 2, false>()
static const BwdEntry kEntries[] = {
    E(kModNone, 0),        E(kModNone, kMaskCausal),        E(kModAlibi, 0),       E(kModAlibi, kMaskCausal),
    E(kModSoftcap, 0),     E(kModSoftcap, kMaskCausal),     E(kModNone, CW),       E(kModNone, CW | kMaskDoc),
    E(kModNone, kMaskDoc), E(kModNone, kMaskCausal | kMaskDoc), E(kModNone, kMaskPrefix),
    E(kModNone, kMaskPrefix | kMaskDoc),
    // additive biases (Evoformer pair / row biases): plain and causal, one or two biases
    bwd_entry<64, kModNone, 0, 64, 2, 64, 2, false, 1>(), bwd_entry<64, kModNone, 0, 64, 2, 64, 2, false, 2>(),
    bwd_entry<64, kModNone, kMaskCausal, 64, 2, 64, 2, false, 1>(), bwd_entry<64, kModNone, kMaskCausal, 64, 2, 64, 2, false, 2>(),
};
#undef E
const BwdEntry* entries_bwd64(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
