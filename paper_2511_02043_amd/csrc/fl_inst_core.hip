// Plain and causal softmax attention, bf16, every supported head dim, in the kernel shapes the
// tuning knobs can select.
#include "fl_registry.hpp"
namespace fl {
#define E(D, NW, RB, BN, WPE, MASK) bf16_entry<D, D, NW, RB, BN, WPE, kModNone, MASK, 0, false, 0>()
#define BOTH(D, NW, RB, BN, WPE) E(D, NW, RB, BN, WPE, 0), E(D, NW, RB, BN, WPE, kMaskCausal)
#define R4(D, NW, RB, BN, WPE, MASK) bf16_entry<D, D, NW, RB, BN, WPE, kModNone, MASK, 0, false, 0, 4>()
#define BOTH4(D, NW, RB, BN, WPE) R4(D, NW, RB, BN, WPE, 0), R4(D, NW, RB, BN, WPE, kMaskCausal)
static const KernelEntry kEntries[] = {
    // first entry of a head dim = default shape; the others are selectable with fl_set_tuning
    BOTH(128, 8, 1, 64, 2), BOTH4(128, 8, 1, 64, 2), BOTH(128, 4, 1, 64, 2), BOTH(128, 4, 2, 32, 1),
    // D = 64, long key loops: two row blocks per wave on 32-key tiles (every K / V fragment read from LDS feeds
    // two MFMAs; 225 registers, two waves per SIMD) measured 2 - 4 % faster than one row block on 64-key tiles.
    // (64, 4, 1, 32, 4): 32-key tiles at four waves per SIMD, four resident workgroups per CU: the host picks
    // it for short key loops (Sk <= 4096 unmasked, <= 2048 causal), where it measured 3 - 12 % faster
    BOTH(64, 4, 2, 32, 2),  BOTH(64, 4, 1, 64, 2),  BOTH(64, 8, 1, 64, 2),  BOTH(64, 4, 1, 32, 4),
    BOTH(32, 4, 1, 64, 2),  BOTH(32, 4, 2, 64, 2),
    // causal attention with keys and values read in place from a paged cache (chunked prefill; other variants of it are
    // instantiated on first use): the default shapes with two ring slots
    bf16_entry<128, 128, 8, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true>(),
    bf16_entry<128, 128, 4, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true>(),
    bf16_entry<64, 64, 4, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true>(),
    // ... and with the query heads of a kv head packed into one workgroup, for chunks shorter than a workgroup's rows:
    // 8 waves x 4 heads x 64 rows, 8 waves x 8 heads x 32 rows, 8 waves x 2 heads x 128 rows, 4 waves x 4 heads x 32 rows,
    // 4 waves x 2 heads x 64 rows
    bf16_entry<128, 128, 8, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true, 4>(),
    bf16_entry<128, 128, 8, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true, 8>(),
    bf16_entry<128, 128, 8, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true, 2>(),
    bf16_entry<128, 128, 4, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true, 4>(),
    bf16_entry<128, 128, 4, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true, 2>(),
    // head dim 64 (32 query / 8 kv heads is the model of the paper's serving experiment): the eight-wave shape and the packed ones
    bf16_entry<64, 64, 8, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true>(),
    bf16_entry<64, 64, 8, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true, 4>(),
    bf16_entry<64, 64, 4, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true, 4>(),
    bf16_entry<64, 64, 4, 1, 64, 2, kModNone, kMaskCausal, 0, false, 0, 2, true, 2>(),
};
#undef BOTH
#undef BOTH4
#undef R4
#undef E
const KernelEntry* entries_core(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
