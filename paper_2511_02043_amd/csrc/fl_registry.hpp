// Table of compiled kernel specialisations: the "variant specialisation layer".
// Each instance translation unit contributes an array of entries; fl_api.hip looks a descriptor
// up in the concatenation of those arrays.  There is deliberately no generic fallback kernel.
#pragma once
#include "fl_kernel_bf16.hpp"
#include <atomic>

namespace fl {

struct KernelKey {
  int dtype;        // 1 = bf16, 2 = f32 (values of fl_dtype)
  int D, DV;        // head dims (f32 entries: the maximum they accept)
  int mod;          // -1 in f32 entries (runtime)
  int mask;         // -1 in f32 entries
  int nbias;        // -1 in f32 entries
  int diff;
  int epi;          // -1 in f32 entries
  int nwaves, rb, bn, wpe;         // kernel shape: waves, 32-row blocks per wave, keys per tile, waves per SIMD
  int ring;                        // slots of the K / V rings in LDS (a barrier every ring / 2 tiles)
  int paged;                       // 1: keys and values are read in place from a paged cache
  int pack;                        // query heads of one kv head per workgroup (1 unless paged: short chunks)
};

typedef hipError_t (*LaunchFn)(const FwdParams& p, int nblocks, hipStream_t stream);

struct KernelEntry {
  KernelKey key;
  int bm;           // query rows per workgroup and head (the workgroup's rows / key.pack)
  int lds_bytes;    // LDS of the K/V rings per workgroup
  LaunchFn launch;  // compiled specialisations; null for one compiled at run time
  void* jit;        // run-time compiled specialisations: the loaded code object (see jit_forward_entry)
  int max_lds;      // dynamic LDS a launch of this entry may ask for (0: all of a compute unit's)
};

// Specialisations outside the compiled table are instantiated from the same kernel template on first
// use (hipRTC) and kept for the life of the process: returns the entry for (D, DV, score_mod, mask,
// n_bias, combine, epilogue), or null with the compiler's message in the thread's error detail.
// Thread-safe; the first call for a combination takes about a second on the host.
struct JitRequest {
  int D, DV, mod;
  uint32_t mask;
  int nbias;
  bool diff;
  uint32_t epi;
  bool paged = false;   // keys and values read in place from a paged cache
  bool wide = false;    // eight waves (256 query rows) per workgroup instead of four: long query tiles at head dim 128
  int pack = 1;         // paged only: query heads of one kv head per workgroup
};
const KernelEntry* jit_forward_entry(const JitRequest& r);
hipError_t jit_forward_launch(const KernelEntry& e, const FwdParams& p, int nblocks, hipStream_t stream);

constexpr int kMaxLdsBytes = 160 * 1024;           // LDS of a gfx950 compute unit

template <class C>
hipError_t launch_bf16(const FwdParams& p, int nblocks, hipStream_t stream) {
  // Raising the dynamic-LDS limit is per device and sticky; cheap enough to repeat per device.
  static std::atomic<bool> done[64];              // zero-initialised; a repeated call from a second thread is harmless
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64 || !done[dev].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute((const void*)fwd_bf16_kernel<C>, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64) done[dev].store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL(fwd_bf16_kernel<C>, dim3(nblocks), dim3(C::NT), p.lds_bytes, stream, p);
  return hipGetLastError();
}

template <int D, int DV, int NWAVES, int RB, int BN, int WPE, int MOD, uint32_t MASK, int NBIAS, bool DIFF,
          uint32_t EPI, int RING = 2, bool PAGED = false, int PACK = 1>
constexpr KernelEntry bf16_entry() {
  typedef Bf16Cfg<D, DV, NWAVES, RB, BN, WPE, MOD, MASK, NBIAS, DIFF, EPI, RING, PAGED, PACK> C;
  static_assert(C::LDS_BYTES <= kMaxLdsBytes, "rings exceed the LDS of a compute unit");
  return KernelEntry{KernelKey{1, D, DV, MOD, (int)MASK, NBIAS, DIFF ? 1 : 0, (int)EPI, NWAVES, RB, BN, WPE, RING, PAGED ? 1 : 0, PACK},
                     C::HEAD_ROWS, C::LDS_BYTES, &launch_bf16<C>};
}

// Each instance file defines one of these.
const KernelEntry* entries_core(int* n);      // plain / causal, all head dims, tuning shapes
const KernelEntry* entries_mods(int* n);      // ALiBi / soft-cap / window / prefix / document masks
const KernelEntry* entries_evo(int* n);       // biases + sigmoid gate
const KernelEntry* entries_diff(int* n);      // differential two-stream + RMSNorm
const KernelEntry* entries_f32(int* n);       // fp32 storage

}  // namespace fl
