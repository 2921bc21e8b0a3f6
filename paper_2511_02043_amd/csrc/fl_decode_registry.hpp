// Table of compiled decode-step specialisations.
#pragma once
#include "fl_bwd_registry.hpp"
#include "fl_decode_bf16.hpp"

namespace fl {

typedef hipError_t (*DecodeLaunchFn)(const DecodeParams& p, int nblocks, hipStream_t stream);

struct DecodeEntry {
  int D, mod, cb;                 // cb: blocks of 32 (query row, head) columns per kv head
  DecodeLaunchFn main, combine;   // main: B * Hkv * nsplit workgroups; combine: B * T * H workgroups
};

template <class C>
hipError_t launch_decode(const DecodeParams& p, int nblocks, hipStream_t stream) {
  hipError_t e = raise_lds_limit(decode_kernel<C>);
  if (e != hipSuccess) return e;
  static_assert(C::LDS <= kMaxLdsBytes, "LDS of the decode kernel");
  hipLaunchKernelGGL(decode_kernel<C>, dim3(nblocks), dim3(C::NWV * 64), C::LDS, stream, p);
  return hipGetLastError();
}
template <int D>
hipError_t launch_decode_combine(const DecodeParams& p, int nblocks, hipStream_t stream) {
  hipLaunchKernelGGL(decode_combine_kernel<D>, dim3(nblocks), dim3(64), 0, stream, p);
  return hipGetLastError();
}

template <int D, int MOD, int CB = 1>
constexpr DecodeEntry decode_entry() {
  return DecodeEntry{D, MOD, CB, &launch_decode<DecodeCfg<D, MOD, CB>>, &launch_decode_combine<D>};
}

const DecodeEntry* entries_decode(int* n);

}  // namespace fl
