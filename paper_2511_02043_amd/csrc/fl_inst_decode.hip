// Decode-step kernels (one query per sequence over a paged key/value cache), bf16.
#include "fl_decode_registry.hpp"
namespace fl {
static const DecodeEntry kEntries[] = {
    decode_entry<128, kModNone>(), decode_entry<128, kModSoftcap>(), decode_entry<128, kModAlibi>(),
    decode_entry<64, kModNone>(),  decode_entry<64, kModSoftcap>(),  decode_entry<64, kModAlibi>(),
};
const DecodeEntry* entries_decode(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
