// fp32-storage kernels: variant switches are runtime values here, only the stream count and the
// register budget for the head dim are compile-time.
#include "fl_registry.hpp"
#include "fl_kernel_f32.hpp"
namespace fl {
template <bool DIFF, int DMAX>
static hipError_t launch_f32(const FwdParams& p, int nblocks, hipStream_t stream) {
  constexpr int kLds = ((DIFF ? 2 : 1) * kF32Keys * DMAX + kF32Keys * DMAX) * 4;
  hipLaunchKernelGGL((fwd_f32_kernel<DIFF, DMAX>), dim3(nblocks), dim3(256), kLds, stream, p);
  return hipGetLastError();
}
#define E(DIFF, DMAX)                                                                        \
  KernelEntry {                                                                              \
    KernelKey{2, DMAX, DMAX, -1, -1, -1, DIFF ? 1 : 0, -1, 4, 1, kF32Keys, 0, 0, 0, 1}, kF32Rows,           \
        ((DIFF ? 2 : 1) * kF32Keys * DMAX + kF32Keys * DMAX) * 4, &launch_f32<DIFF, DMAX>    \
  }
static const KernelEntry kEntries[] = {E(false, 64), E(false, 128), E(true, 64), E(true, 128)};
#undef E
const KernelEntry* entries_f32(int* n) {
  *n = (int)(sizeof(kEntries) / sizeof(kEntries[0]));
  return kEntries;
}
}  // namespace fl
