// Table of compiled backward specialisations (one dQ kernel and one dK/dV kernel per entry).
#pragma once
#include "fl_bwd_bf16.hpp"
#include <atomic>
#include <string>
#include <vector>
#include "../../include/fl_attn.h"
#include "fl_registry.hpp"

namespace fl {

struct BwdKey {
  int D;            // head dim (D == Dv)
  int mod, mask;
  int nbias;        // additive biases the kernels read (and whose gradient the dQ kernel emits)
};

typedef hipError_t (*BwdLaunchFn)(const BwdParams& p, int nblocks, hipStream_t stream);

struct BwdEntry {
  BwdKey key;
  int bm;           // query rows per workgroup of the dQ kernel = keys per workgroup of the dK/dV kernel
  BwdLaunchFn prep, dq, dkdv, reduce;   // reduce: sum of the head-subset partials of dK / dV (nblocks of 256 threads)
  void* jit;        // entries instantiated at run time: their dq / dkdv are null and launched through jit_backward_launch
};

// A backward specialisation outside the compiled table, instantiated from the same kernel templates with hipRTC
// on first use and kept for the life of the process (null if it does not compile).  prep / reduce: the compiled
// pre-pass and partial-sum kernels of that head dim, which do not depend on the variant.
const BwdEntry* jit_backward_entry(int D, int mod, uint32_t mask, int nbias, BwdLaunchFn prep, BwdLaunchFn reduce);
// which: 0 = the dQ kernel, 1 = the dK/dV kernel
hipError_t jit_backward_launch(const BwdEntry& e, int which, const BwdParams& p, int nblocks, hipStream_t stream);
// A run-time entry around an already compiled code object with the two kernels (variants compiled from expressions);
// owned by the caller, released with jit_backward_release.
BwdEntry* jit_backward_wrap(const std::vector<char>& code, const std::string& dq_name, const std::string& dkdv_name, int D, int mod,
                            uint32_t mask, BwdLaunchFn prep, BwdLaunchFn reduce);
void jit_backward_release(BwdEntry* e);

template <class K>
hipError_t raise_lds_limit(K kernel) {
  static std::atomic<bool> done[64];              // zero-initialised; a repeated call from a second thread is harmless
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64 || !done[dev].load(std::memory_order_acquire)) {
    e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64) done[dev].store(true, std::memory_order_release);
  }
  return hipSuccess;
}

template <int DV>
hipError_t launch_bwd_prep(const BwdParams& p, int nblocks, hipStream_t stream) {
  hipLaunchKernelGGL(bwd_prep_kernel<DV>, dim3(nblocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}
template <int D>
hipError_t launch_bwd_reduce(const BwdParams& p, int nblocks, hipStream_t stream) {
  hipLaunchKernelGGL(bwd_reduce_kv_kernel<D>, dim3(nblocks), dim3(256), 0, stream, p);
  return hipGetLastError();
}
template <class C>
hipError_t launch_bwd_dq(const BwdParams& p, int nblocks, hipStream_t stream) {
  hipError_t e = raise_lds_limit(bwd_dq_kernel<C>);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_dq_kernel<C>, dim3(nblocks), dim3(C::NT), 2 * C::STAGE_DQ, stream, p);
  return hipGetLastError();
}
template <class C>
hipError_t launch_bwd_dkdv(const BwdParams& p, int nblocks, hipStream_t stream) {
  hipError_t e = raise_lds_limit(bwd_dkdv_kernel<C>);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_dkdv_kernel<C>, dim3(nblocks), dim3(C::NT), 3 * C::STAGE_KV, stream, p);
  return hipGetLastError();
}

template <class C>
hipError_t launch_bwd_dkdv_ws(const BwdParams& p, int nblocks, hipStream_t stream) {
  hipError_t e = raise_lds_limit(bwd_dkdv_ws_kernel<C>);
  if (e != hipSuccess) return e;
  constexpr int lds = 3 * C::STAGE_KV + 4 * 2 * (64 * 16 * 4);   // tile ring, then two exchange buffers per wave pair
  static_assert(lds <= kMaxLdsBytes, "LDS of the wave-specialised dK/dV kernel");
  hipLaunchKernelGGL(bwd_dkdv_ws_kernel<C>, dim3(nblocks), dim3(512), lds, stream, p);
  return hipGetLastError();
}

// CQ / CK: the shapes of the dQ kernel and of the dK/dV kernel (streamed tile rows, waves per SIMD).
// WS: the dK/dV kernel with specialised waves (eight waves, two per SIMD) instead of the plain one.
template <int D, int MOD, uint32_t MASK, int BN_Q, int WPE_Q, int BN_K, int WPE_K, bool WS, int NBIAS = 0>
constexpr BwdEntry bwd_entry() {
  typedef BwdCfg<D, MOD, MASK, BN_Q, WPE_Q, NBIAS> CQ;
  typedef BwdCfg<D, MOD, MASK, BN_K, WPE_K, NBIAS> CK;
  if constexpr (WS)
    return BwdEntry{BwdKey{D, MOD, (int)MASK, NBIAS}, CQ::BM, &launch_bwd_prep<D>, &launch_bwd_dq<CQ>, &launch_bwd_dkdv_ws<CK>, &launch_bwd_reduce<D>, nullptr};
  else
    return BwdEntry{BwdKey{D, MOD, (int)MASK, NBIAS}, CQ::BM, &launch_bwd_prep<D>, &launch_bwd_dq<CQ>, &launch_bwd_dkdv<CK>, &launch_bwd_reduce<D>, nullptr};
}

// The call behind fl_attn_bwd (fl_api.hip).  custom / user_aux: the backward kernels of a variant compiled at run time from
// expressions and the arrays its expressions read, instead of the specialisation the descriptor names.
fl_status backward_call(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_tensor* out, const fl_tensor* dout,
                        const fl_tensor* lse, const fl_variant_desc* desc, const fl_aux* aux, fl_tensor* dq, fl_tensor* dk,
                        fl_tensor* dv, void* stream, const BwdEntry* custom, const void* const* user_aux);

const BwdEntry* entries_bwd64(int* n);
const BwdEntry* entries_bwd128(int* n);

}  // namespace fl
