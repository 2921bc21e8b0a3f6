// Decode-step kernels (the newest query rows of each sequence over a paged key/value cache), bf16:
// one block of 32 (query row, head) columns per kv head, and two.
#include "fl_decode_registry.hpp"
namespace fl {
static const DecodeEntry kEntries[] = {
    decode_entry<128, kModNone>(), decode_entry<128, kModSoftcap>(), decode_entry<128, kModAlibi>(),
    decode_entry<64, kModNone>(),  decode_entry<64, kModSoftcap>(),  decode_entry<64, kModAlibi>(),
    decode_entry<128, kModNone, 2>(), decode_entry<128, kModSoftcap, 2>(), decode_entry<128, kModAlibi, 2>(),
    decode_entry<64, kModNone, 2>(),  decode_entry<64, kModSoftcap, 2>(),  decode_entry<64, kModAlibi, 2>(),
};
const DecodeEntry* entries_decode(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
