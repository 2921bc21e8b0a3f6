// Kernel-side parameter block and small device helpers shared by every kernel of the library.
#pragma once
// Under hipRTC (run-time compilation of a custom variant) the HIP built-ins are already there and
// no system header is reachable: the one library facility the kernels use is declared here.
#ifdef __HIPCC_RTC__
typedef signed char int8_t;
typedef unsigned char uint8_t;
typedef short int16_t;
typedef unsigned short uint16_t;
typedef int int32_t;
typedef unsigned int uint32_t;
typedef long long int64_t;
typedef unsigned long long uint64_t;
#ifndef INFINITY
#define INFINITY __builtin_huge_valf()
#endif
namespace std {
template <class T, T v>
struct integral_constant {
  static constexpr T value = v;
  typedef T value_type;
  constexpr operator value_type() const noexcept { return value; }
  constexpr value_type operator()() const noexcept { return value; }
};
}  // namespace std
#else
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#endif

namespace fl {

// Mask bits / enums mirror include/fl_attn.h (kept numerically identical; checked in fl_api.hip).
constexpr uint32_t kMaskCausal = 1, kMaskWindow = 2, kMaskDoc = 4, kMaskPrefix = 8;
constexpr int kModNone = 0, kModAlibi = 1, kModSoftcap = 2;
// Variants compiled at run time from user expressions (fl_compile_variant): the score_mod and the
// mask predicate are the two functions below, defined by the generated translation unit.  The
// library's own kernels never instantiate these values, so the functions need no definition there.
constexpr int kModCustom = 3;
constexpr uint32_t kMaskCustom = 16;
constexpr uint32_t kEpiRms = 1, kEpiGate = 2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Granularity (rows / keys) of the document-id summaries used by the tile skipper.
constexpr int kSumBlock = 32;

struct View {            // a [B, G, H, S, D] view: element strides of the four outer axes
  const void* ptr;
  int64_t sb, sg, sh, ss;
};

struct BiasView {        // logical [B, G, H, Sq, Sk]; any stride may be 0 (broadcast)
  const void* ptr;
  int64_t sb, sg, sh, si, sj;
  int32_t is_f32;
  int32_t vec4;          // 1: sj == 1 and every row start is 8-byte aligned -> 4 keys per load
  int32_t dma;           // 1 (bf16 kernels): rows are 16-byte aligned and differ per query -> tiles staged through LDS
};

struct FwdParams {
  View q, k, v, q2, k2, gate;
  View out;              // ptr is written
  BiasView bias[2];
  float* lse;            // may be null
  int64_t lse_sb, lse_sg, lse_sh;   // element strides of lse [B, G(or 2G), H, Sq]
  const float* alibi_slopes;
  const float* lambda;
  const float* rms_weight;
  const int32_t* q_doc;  // [B, Sq]
  const int32_t* kv_doc; // [B, Sk]
  int2* q_sum;           // [B, ceil(Sq/32)]  (min, max) of q_doc per 32-row block
  int2* kv_sum;          // [B, ceil(Sk/32)]
  int32_t B, G, H, Hkv, Sq, Sk;
  int32_t D, Dv;         // head dims (compile-time in the bf16 kernels, read by the fp32 kernel)
  int32_t window, prefix;
  float scale, softcap, rms_eps;
  int32_t out_f32;       // 1: out is float, 0: out has the input dtype
  int32_t mod, mask, n_bias, epi;   // runtime copy of the descriptor (fp32 kernel reads these)
  int32_t n_qtiles;      // ceil(Sq / rows per workgroup)
  int32_t order;         // workgroup ordering scheme
  int32_t doc_vec;       // 1: kv_doc rows are 16-byte aligned and Sk % 4 == 0 -> 4 ids per load
  int32_t lds_bytes;     // bf16 kernels: dynamic LDS size of this launch (K/V rings, then bias staging)
  int32_t bias_lds_base; // byte offset of the per-wave bias staging buffers in LDS
  int32_t bias_lds_wave; // bytes of staging per wave (two buffers for every bias up to the last staged one)
  int32_t pair;          // bf16 kernels: 1 = a workgroup takes q-tiles nq - 1 - i and i (balanced causal work)
  int32_t q_off;         // query row i sits at sequence position i + q_off (positional masks, ALiBi); >= 0
  const void* user_aux[4];   // run-time compiled variants: the caller's device arrays that the expressions read
  const unsigned char* block_map;   // run-time compiled masks, or null: tile classes [problem][key tile][query block] (block_map_kernel)
  const uint32_t* block_bits;       // ... and, or null: per block 64 words (one per lane) of hidden-score bits
  int32_t map_nqb8, map_nkt;        // query blocks per tile row (a multiple of 8) and key tiles of the map
  int32_t map_per_head;             // 1: a problem of the map is (b, g, h); 0: b (the expression reads neither g nor h)
  const int32_t* block_table;  // kernels that read keys in place from a paged cache (k, v: [pages, 1, Hkv, page_size, D]):
  int32_t table_stride;        // [B, table_stride] page of each block of tokens, or null: sequence b is page b
  int32_t page_shift, page_mask, num_pages;   // tokens per page = 1 << page_shift; entries are cut to [0, num_pages)
  const int32_t* kv_lens;    // bf16 kernels, or null: [B] keys of each sequence (cut to [0, Sk]); then q_off = kv_lens[b] - Sq
};

}  // namespace fl
// new score from the scaled score s of query i and key j (Eq. 4's score_mod); p gives the expression
// the call's sizes and the caller's captured arrays
__device__ float fl_user_score_mod(float s, int b, int g, int h, int i, int j, const fl::FwdParams& p);
// derivative of fl_user_score_mod with respect to s at the same arguments (the backward pass of a compiled variant)
__device__ float fl_user_score_mod_grad(float s, int b, int g, int h, int i, int j, const fl::FwdParams& p);
// true where the score of (i, j) is to be replaced by -inf (the mask_mod of Sec. 2.2, inverted)
__device__ bool fl_user_mask(int b, int g, int h, int i, int j, const fl::FwdParams& p);
namespace fl {

// Compile-time loop: f(std::integral_constant<int, I>) for I in [B, E).
template <int B, int E, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>());
    static_for<B + 1, E>(f);
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// Is score (i, j) masked?  MASK is the set of active mask kinds; the bf16 kernels pass a
// compile-time constant (the tests fold away), the fp32 kernel a runtime value.
__device__ __forceinline__ bool is_masked(const uint32_t MASK, int i, int j, int window, int prefix,
                                          int qdoc, int kdoc) {
  bool m = false;
  if ((MASK & kMaskPrefix) != 0) m = m || (j > i && j >= prefix);
  else if ((MASK & (kMaskCausal | kMaskWindow)) != 0) m = m || (j > i);
  if ((MASK & kMaskWindow) != 0) m = m || (i - j > window);
  if ((MASK & kMaskDoc) != 0) m = m || (qdoc != kdoc);
  return m;
}

// Key range [lo, hi) that can be visible to any query row in [i_min, i_max] under the
// positional masks (document masks are handled per tile through the summaries).
__device__ __forceinline__ void key_range(const uint32_t MASK, int i_min, int i_max, int Sk,
                                          int window, int prefix, int& lo, int& hi) {
  lo = 0;
  hi = Sk;
  if ((MASK & kMaskPrefix) != 0) {
    int h = i_max + 1 > prefix ? i_max + 1 : prefix;
    hi = h < Sk ? h : Sk;
  } else if ((MASK & (kMaskCausal | kMaskWindow)) != 0) {
    hi = i_max + 1 < Sk ? i_max + 1 : Sk;
  }
  if ((MASK & kMaskWindow) != 0) lo = i_min - window > 0 ? i_min - window : 0;
}

enum BlockClass : int { kSkip = 0, kFull = 1, kPartial = 2 };

// Classify the block of query rows [q_lo, q_hi] x keys [k_lo, k_hi] (all inclusive, k_hi may
// exceed Sk - 1 for a ragged tail): kSkip = every score masked, kFull = none masked.
__device__ __forceinline__ int classify_block(const uint32_t MASK, int q_lo, int q_hi, int k_lo,
                                              int k_hi, int Sk, int window, int prefix, int2 qs,
                                              int2 ks) {
  if (k_lo >= Sk) return kSkip;
  bool full = k_hi < Sk;
  const int k_last = k_hi < Sk ? k_hi : Sk - 1;
  if ((MASK & kMaskPrefix) != 0) {
    if (k_lo > q_hi && k_lo >= prefix) return kSkip;
    full = full && (k_last <= q_lo || k_last < prefix);
  } else if ((MASK & (kMaskCausal | kMaskWindow)) != 0) {
    if (k_lo > q_hi) return kSkip;
    full = full && (k_last <= q_lo);
  }
  if ((MASK & kMaskWindow) != 0) {
    if (q_lo - k_last > window) return kSkip;
    full = full && (q_hi - k_lo <= window);
  }
  if ((MASK & kMaskDoc) != 0) {
    if (qs.y < ks.x || ks.y < qs.x) return kSkip;     // id ranges disjoint: nothing can match
    full = full && (qs.x == qs.y && ks.x == ks.y && qs.x == ks.x);
  }
  return full ? kFull : kPartial;
}

// Tiles of BN keys that are fully visible (classify_block == kFull) to the query rows
// [q_lo, q_hi] under the positional masks form one range [lo, hi); this is that range in closed
// form (document masks need the per-tile summaries instead).
__device__ __forceinline__ void full_tile_range(const uint32_t MASK, int q_lo, int q_hi, int Sk, int window,
                                                int prefix, int BN, int& lo, int& hi) {
  lo = 0;
  hi = Sk / BN;                                    // tiles that end inside the key range
  if ((MASK & kMaskPrefix) != 0) {
    const int last = q_lo > prefix - 1 ? q_lo : prefix - 1;   // last key every row may see
    hi = min(hi, (last + 1) / BN);
  } else if ((MASK & (kMaskCausal | kMaskWindow)) != 0) {
    hi = min(hi, (q_lo + 1) / BN);
  }
  if ((MASK & kMaskWindow) != 0) {
    const int first = q_hi - window;               // first key every row may see
    lo = first > 0 ? (first + BN - 1) / BN : 0;
  }
}

}  // namespace fl
