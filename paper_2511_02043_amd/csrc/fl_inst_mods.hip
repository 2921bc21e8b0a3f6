// Score modifications (ALiBi, tanh soft-cap; Eq. 4) and the mask family (sliding window,
// PrefixLM, document mask; Sec. 4.1 benchmark variants), bf16.
#include "fl_registry.hpp"
namespace fl {
// Document masks at D = 128 keep 32-key tiles: their id registers do not fit beside two 64-key score tiles.
#define E(D, MOD, MASK) bf16_entry<D, D, 4, 1, (D == 128 && ((MASK) & kMaskDoc) != 0) ? 32 : 64, 2, MOD, MASK, 0, false, 0>()
constexpr uint32_t CW = kMaskCausal | kMaskWindow;
static const KernelEntry kEntries[] = {
    E(64, kModAlibi, 0),   E(64, kModAlibi, kMaskCausal),   E(64, kModSoftcap, 0), E(64, kModSoftcap, kMaskCausal),
    // sliding window: short key loops, most tiles partly masked; 32-key tiles at four waves per SIMD (four
    // resident workgroups per CU) measured 10 % faster than the common shape, which stays selectable
    bf16_entry<64, 64, 4, 1, 32, 4, kModNone, CW, 0, false, 0>(),
    // window and document mask: three waves per SIMD (the document ids do not fit four), 7 % faster at every length
    bf16_entry<64, 64, 4, 1, 32, 3, kModNone, CW | kMaskDoc, 0, false, 0>(),
    E(64, kModNone, CW),   E(64, kModNone, CW | kMaskDoc),  E(64, kModNone, kMaskDoc),
    E(64, kModNone, kMaskCausal | kMaskDoc),
    bf16_entry<64, 64, 4, 2, 32, 2, kModNone, kMaskPrefix, 0, false, 0>(),   // long key loops: two row blocks per wave, as for plain / causal
    E(64, kModNone, kMaskPrefix), E(64, kModNone, kMaskPrefix | kMaskDoc),
    // 32-key tiles for the short key loops of other variants (chosen by the host for Sk <= 2048, where they
    // measured 2 - 11 % faster): four waves per SIMD, or three where the document ids need the registers.
    // ALiBi gains only at S = 512 and keeps one shape.
    bf16_entry<64, 64, 4, 1, 32, 4, kModSoftcap, 0, 0, false, 0>(), bf16_entry<64, 64, 4, 1, 32, 4, kModNone, kMaskPrefix, 0, false, 0>(),
    bf16_entry<64, 64, 4, 1, 32, 3, kModNone, kMaskDoc, 0, false, 0>(), bf16_entry<64, 64, 4, 1, 32, 3, kModNone, kMaskCausal | kMaskDoc, 0, false, 0>(),
    E(128, kModAlibi, 0),  E(128, kModSoftcap, 0), E(128, kModNone, CW), E(128, kModNone, CW | kMaskDoc),
    E(128, kModNone, kMaskDoc), E(128, kModNone, kMaskCausal | kMaskDoc), E(128, kModNone, kMaskPrefix),
};
#undef E
const KernelEntry* entries_mods(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
