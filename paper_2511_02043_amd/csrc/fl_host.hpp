// Host-side helpers shared by the translation units that implement the C ABI: the thread-local
// error detail, and the checks / views of [B, G, H, S, D] tensors.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/fl_attn.h"
#include "fl_params.hpp"

namespace fl {
namespace host {

inline thread_local char g_detail[384] = "";
inline void clear_detail() { g_detail[0] = 0; }

inline fl_status fail(fl_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_detail, sizeof(g_detail), fmt, ap);
  va_end(ap);
  return st;
}



inline int elem_size(int dtype) { return dtype == FL_BF16 ? 2 : 4; }

// Common checks of a [B, G, H, S, D] data tensor (q, k, v, out, gate, q2, k2).
inline fl_status check_data_tensor(const fl_tensor* t, const char* name, int want_dtype, const int64_t want[5]) {
  if (t == nullptr || t->ptr == nullptr) return fail(FL_ERR_NULL, "%s is NULL", name);
  if (t->dtype != want_dtype) return fail(FL_ERR_DTYPE, "%s has dtype %d, expected %d", name, t->dtype, want_dtype);
  for (int a = 0; a < 5; ++a)
    if (t->size[a] != want[a])
      return fail(FL_ERR_SHAPE, "%s size[%d] = %lld, expected %lld", name, a, (long long)t->size[a],
                  (long long)want[a]);
  if (t->stride[4] != 1) return fail(FL_ERR_STRIDE, "%s innermost stride must be 1", name);
  const int es = elem_size(t->dtype);
  if (((uintptr_t)t->ptr) % 16 != 0) return fail(FL_ERR_ALIGN, "%s base pointer not 16-byte aligned", name);
  for (int a = 0; a < 4; ++a) {
    if (t->stride[a] < 0) return fail(FL_ERR_STRIDE, "%s stride[%d] negative", name, a);
    if (t->size[a] > 1 && t->stride[a] == 0) return fail(FL_ERR_STRIDE, "%s stride[%d] is 0 (no broadcast here)", name, a);
    if (t->size[a] > 1 && (t->stride[a] * es) % 16 != 0)
      return fail(FL_ERR_ALIGN, "%s stride[%d] not a multiple of 16 bytes", name, a);
  }
  // the kernels address the rows of one key tile with 32-bit byte offsets from the tile's base
  if (t->size[3] > 1 && t->stride[3] >= (int64_t)1 << 23)
    return fail(FL_ERR_STRIDE, "%s row stride %lld is not below 2^23 elements", name, (long long)t->stride[3]);
  return FL_OK;
}

inline fl::View make_view(const fl_tensor* t) {
  fl::View v;
  v.ptr = t->ptr;
  v.sb = t->size[0] > 1 ? t->stride[0] : 0;
  v.sg = t->size[1] > 1 ? t->stride[1] : 0;
  v.sh = t->size[2] > 1 ? t->stride[2] : 0;
  v.ss = t->size[3] > 1 ? t->stride[3] : 0;
  return v;
}


}  // namespace host
}  // namespace fl
