// C-ABI entry points: argument validation, descriptor -> kernel-specialisation lookup, launch.
// Nothing here computes attention; every step of the path runs in the kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "../../include/fl_attn.h"
#include "fl_bwd_registry.hpp"
#include "fl_host.hpp"
#include "fl_decode_registry.hpp"
#include "fl_registry.hpp"

static_assert(FL_MASK_CAUSAL == fl::kMaskCausal && FL_MASK_WINDOW == fl::kMaskWindow &&
                  FL_MASK_DOC == fl::kMaskDoc && FL_MASK_PREFIX == fl::kMaskPrefix,
              "mask bits");
static_assert(FL_MOD_NONE == fl::kModNone && FL_MOD_ALIBI == fl::kModAlibi && FL_MOD_SOFTCAP == fl::kModSoftcap,
              "score_mod values");
static_assert(FL_EPI_RMSNORM == fl::kEpiRms && FL_EPI_GATE_SIGMOID == fl::kEpiGate, "epilogue bits");

// Built-in scratch of fl_attn_fwd_noalloc: the tile skipper's document-id summaries live here instead
// of in a caller-supplied workspace.  One copy per GPU, held until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; kernels get the device address it returns.
constexpr size_t kScratchBytes = 1u << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

using fl::host::check_data_tensor;
using fl::host::fail;
using fl::host::g_detail;
using fl::host::make_view;

// Shape requests of fl_set_tuning.  Per host thread: a request changes the calls of the thread that made it
// and nothing else, so the entry points share no mutable state (the error detail is per thread as well).
struct Tuning {
  int bm = 0, bn = 0, rb = 0, nw = 0, wpe = 0, ring = 0, order = -1, pair = -1;
  int decode_splits = 0;           // 0: chosen by decode_splits() from the shapes
  int prefill_pack = 0;            // fl_attn_prefill_paged in place: 1 never packs the query heads of a kv head into one workgroup
  int prefill_gather = 0;          // fl_attn_prefill_paged: 1 always copies the pages into dense tensors first, 2 never
                                   // (where the pages allow it); 0: by chunk length
  int bwd_wg_target = 0;           // 0: the default of choose_hsplit
};
thread_local Tuning g_tuning;

struct Registry {
  const fl::KernelEntry* tab[5];
  int n[5];
  Registry() {
    tab[0] = fl::entries_core(&n[0]);
    tab[1] = fl::entries_mods(&n[1]);
    tab[2] = fl::entries_evo(&n[2]);
    tab[3] = fl::entries_diff(&n[3]);
    tab[4] = fl::entries_f32(&n[4]);
  }
};
const Registry& registry() {
  static Registry r;
  return r;
}

// A window that reaches past both sequence ends changes nothing; cutting it there keeps the kernels'
// int32 arithmetic on i - window and j + window far from overflow (callers pass INT_MAX for "no limit").
int32_t clamp_window(int32_t window, int64_t Sq, int64_t Sk) {
  const int64_t lim = Sq > Sk ? Sq : Sk;
  return (int64_t)window > lim ? (int32_t)lim : window;
}

// Canonical mask bits: WINDOW implies CAUSAL.
uint32_t canonical_mask(uint32_t m) { return (m & FL_MASK_WINDOW) ? (m | FL_MASK_CAUSAL) : m; }

fl_status check_desc(const fl_variant_desc* d) {
  if (d == nullptr) return fail(FL_ERR_NULL, "desc is NULL");
  if (d->struct_size != sizeof(fl_variant_desc))
    return fail(FL_ERR_DESC, "desc->struct_size = %u, expected %zu", d->struct_size, sizeof(fl_variant_desc));
  if (!(d->scale > 0.f) || !std::isfinite(d->scale)) return fail(FL_ERR_DESC, "scale must be finite and > 0");
  if (d->score_mod > FL_MOD_SOFTCAP) return fail(FL_ERR_DESC, "unknown score_mod %u", d->score_mod);
  if (d->score_mod == FL_MOD_SOFTCAP && (!(d->softcap > 0.f) || !std::isfinite(d->softcap)))
    return fail(FL_ERR_DESC, "softcap must be finite and > 0");
  if (d->mask & ~(uint32_t)(FL_MASK_CAUSAL | FL_MASK_WINDOW | FL_MASK_DOC | FL_MASK_PREFIX))
    return fail(FL_ERR_DESC, "unknown mask bits 0x%x", d->mask);
  if ((d->mask & FL_MASK_PREFIX) && (d->mask & (FL_MASK_CAUSAL | FL_MASK_WINDOW)))
    return fail(FL_ERR_DESC, "FL_MASK_PREFIX excludes FL_MASK_CAUSAL and FL_MASK_WINDOW");
  if ((d->mask & FL_MASK_WINDOW) && d->window < 0) return fail(FL_ERR_DESC, "window must be >= 0");
  if ((d->mask & FL_MASK_PREFIX) && d->prefix_len < 0) return fail(FL_ERR_DESC, "prefix_len must be >= 0");
  if (d->n_bias > 2) return fail(FL_ERR_DESC, "n_bias must be 0..2");
  if (d->combine > FL_DIFFERENTIAL) return fail(FL_ERR_DESC, "unknown combine %u", d->combine);
  if (d->epilogue & ~(uint32_t)(FL_EPI_RMSNORM | FL_EPI_GATE_SIGMOID))
    return fail(FL_ERR_DESC, "unknown epilogue bits 0x%x", d->epilogue);
  if ((d->epilogue & FL_EPI_RMSNORM) && (!(d->rms_eps >= 0.f) || !std::isfinite(d->rms_eps)))
    return fail(FL_ERR_DESC, "rms_eps must be finite and >= 0");
  if (d->q_offset < 0 || d->q_offset > 0x3fffffff) return fail(FL_ERR_DESC, "q_offset must be in [0, 2^30)");
  return FL_OK;
}

// Sk > 0: the key length of the call, for the shape preference; <= 0: any shape of the variant will do.
// heads x Sq (both > 0): the independent rows of the call, for the size of the launch.
struct PagedShape {
  int pack;    // query heads of one kv head per workgroup
  bool wide;   // eight waves (256 rows) per workgroup instead of four (128)
};

const fl::KernelEntry* find_entry(const fl_variant_desc* d, int dtype, int D, int Dv, int64_t Sk = 0, int64_t heads = 0,
                                  int64_t Sq = 0, const PagedShape* paged = nullptr, const PagedShape* packed = nullptr) {
  const Registry& r = registry();
  const int mask = (int)canonical_mask(d->mask);
  const fl::KernelEntry* best = nullptr;
  const fl::KernelEntry* short_loop = nullptr;    // the variant's 32-key-tile shape at three or four waves per SIMD, if listed
  const fl::KernelEntry* four_waves = nullptr;    // a 4-wave, one-row-block shape of the variant (128 query rows per workgroup)
  const fl::KernelEntry* deep_ring = nullptr;     // the default shape with four-slot K / V rings (a barrier per two tiles)
  for (int t = 0; t < 5; ++t)
    for (int e = 0; e < r.n[t]; ++e) {
      const fl::KernelEntry& k = r.tab[t][e];
      if (k.key.dtype != dtype || k.key.diff != (int)d->combine || (k.key.paged != 0) != (paged != nullptr)) continue;
      if (paged != nullptr && (k.key.pack != paged->pack || k.key.nwaves != (paged->wide ? 8 : 4))) continue;
      if (paged == nullptr && k.key.pack != (packed != nullptr ? packed->pack : 1)) continue;
      if (packed != nullptr && k.key.nwaves != (packed->wide ? 8 : 4)) continue;
      if (dtype == FL_F32) {
        if (D > k.key.D || Dv > k.key.DV) continue;
        if (best == nullptr || k.key.D < best->key.D) best = &k;   // smallest register budget that fits
        continue;
      }
      if (k.key.D != D || k.key.DV != Dv || k.key.mod != (int)d->score_mod || k.key.mask != mask ||
          k.key.nbias != (int)d->n_bias || k.key.epi != (int)d->epilogue)
        continue;
      // shape preference: tuning request if it exists, else the first listed
      auto wanted = [](const fl::KernelEntry& e) {
        return (g_tuning.bm == 0 || e.bm == g_tuning.bm) && (g_tuning.bn == 0 || e.key.bn == g_tuning.bn) &&
               (g_tuning.rb == 0 || e.key.rb == g_tuning.rb) && (g_tuning.nw == 0 || e.key.nwaves == g_tuning.nw) &&
               (g_tuning.wpe == 0 || e.key.wpe == g_tuning.wpe) && (g_tuning.ring == 0 || e.key.ring == g_tuning.ring);
      };
      if (best == nullptr || (wanted(k) && !wanted(*best))) best = &k;
      if (short_loop == nullptr && k.key.bn == 32 && k.key.wpe >= 3) short_loop = &k;
      if (four_waves == nullptr && k.key.nwaves == 4 && k.key.rb == 1 && k.key.wpe == 2) four_waves = &k;
      if (deep_ring == nullptr && k.key.ring == 4) deep_ring = &k;
    }
  // Short key loops: start-up and drain of a workgroup weigh more than the per-tile cost, and four
  // small workgroups per CU hide them better than two large ones (measured on the paper's grid at
  // head dim 64; the crossover is at a few dozen key tiles per query tile).
  const bool tuned = g_tuning.bm || g_tuning.bn || g_tuning.rb || g_tuning.nw || g_tuning.wpe || g_tuning.ring;
  if (paged != nullptr || packed != nullptr) return best;   // the shape was chosen by paged_shape()
  // (it needs a launch that fills the CUs four workgroups deep: on a small launch the fewer, larger tiles win)
  const bool known = heads > 0 && Sq > 0;
  if (!tuned && best != nullptr && short_loop != nullptr && Sk > 0 && Sk <= (mask == 0 ? 4096 : 2048) &&
      (!known || heads * ((Sq + 127) / 128) >= 1024))
    best = short_loop;
  // Small launches: 256-row workgroups leave CUs idle when there are fewer than about a thousand of them (512
  // without a mask: every workgroup then carries the same load);
  // the 128-row shape measured 2 - 45 % faster there and 1 - 2 % slower on large launches.
  else if (!tuned && best != nullptr && four_waves != nullptr && best->bm == 256 && known &&
           heads * ((Sq + 255) / 256) < (mask == 0 ? 512 : 1024))
    best = four_waves;
  // Long key loops at the default shape: with four ring slots the workgroup meets at a barrier once per two
  // tiles, which measured 1.7 % faster on the causal S = 8192 benchmark shape; short loops would only pay the
  // longer prologue (three K tiles and two V tiles in flight before the first contraction).
  if (!tuned && best != nullptr && deep_ring != nullptr && best->key.ring == 2 && best->key.nwaves == deep_ring->key.nwaves &&
      best->key.rb == deep_ring->key.rb && best->key.bn == deep_ring->key.bn && best->key.wpe == deep_ring->key.wpe &&
      Sk >= 2048)
    best = deep_ring;
  return best;
}

// Shape of the kernel that reads a paged cache in place.  Unpacked: 256-row workgroups from 512 query rows on when
// that still gives 512 workgroups (measured 17 % faster there than the 128-row shape, which wins below).  A chunk that
// leaves much of such a tile empty packs the query heads of a kv head into the workgroup instead: with R rows per head
// and tile (32, 64 or 128; 256 / R or 128 / R heads, which has to divide the heads per kv head) the MFMA rows are
// filled to Sq / (ceil(Sq / R) R); the R with the best fill is taken when that beats the unpacked tile by a fifth, with
// as many heads as fit (K / V are then fetched once for all of them).
PagedShape paged_shape(int64_t heads, int64_t group, int64_t Sq) {
  PagedShape s;
  s.pack = 1;
  s.wide = heads > 0 && Sq >= 512 && heads * ((Sq + 255) / 256) >= 512;
  if (g_tuning.nw != 0) s.wide = g_tuning.nw == 8;
  if (g_tuning.prefill_pack == 1 || Sq <= 0 || group <= 1) return s;
  auto fill = [&](int64_t rows) { return (double)Sq / (double)(((Sq + rows - 1) / rows) * rows); };
  double best = fill(s.wide ? 256 : 128) * 1.2;
  for (int rows = 128; rows >= 32; rows /= 2) {
    const bool can_wide = group % (256 / rows) == 0, can_narrow = rows < 128 && group % (128 / rows) == 0;
    if (!can_wide && !can_narrow) continue;
    const double f = fill(rows);
    if (f > best) {
      best = f;
      s.wide = can_wide;
      s.pack = (can_wide ? 256 : 128) / rows;
    }
  }
  return s;
}

// Head dims the bf16 kernel template can be instantiated for at run time.
bool jit_dims_ok(int64_t D, int64_t Dv) {
  return (D == 32 || D == 64 || D == 128) && (Dv == 32 || Dv == 64 || Dv == 128);
}

size_t workspace_bytes(int64_t B, int64_t Sq, int64_t Sk, uint32_t mask) {
  if (!(mask & FL_MASK_DOC)) return 0;
  const int64_t nq = (Sq + fl::kSumBlock - 1) / fl::kSumBlock, nk = (Sk + fl::kSumBlock - 1) / fl::kSumBlock;
  return (size_t)(B * (nq + nk)) * sizeof(int2);
}

// (min, max) of the document ids of each block of 32 tokens, one wave per block; the query-side and the key-side
// summaries in one launch (waves [0, tq) and [tq, tq + tk)).
__global__ void doc_summary_kernel(const int32_t* __restrict__ q_ids, int2* __restrict__ q_sum, int Sq, int nqs, int tq,
                                   const int32_t* __restrict__ k_ids, int2* __restrict__ k_sum, int Sk, int nks, int tk) {
  int w = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  if (w >= tq + tk) return;
  const bool keys = w >= tq;                       // uniform over the wave
  if (keys) w -= tq;
  const int32_t* ids = keys ? k_ids : q_ids;
  const int S = keys ? Sk : Sq, nblk = keys ? nks : nqs;
  const int b = w / nblk, blk = w % nblk;
  const int j = blk * fl::kSumBlock + (lane & 31);
  const int jc = j < S ? j : S - 1;
  int lo = ids[(int64_t)b * S + jc], hi = lo;
#pragma unroll
  for (int o = 16; o >= 1; o >>= 1) {
    lo = min(lo, __shfl_xor(lo, o));
    hi = max(hi, __shfl_xor(hi, o));
  }
  if (lane == 0) (keys ? k_sum : q_sum)[w] = make_int2(lo, hi);
}

void launch_doc_summaries(const int32_t* q_ids, int2* q_sum, int Sq, int nqs, int tq, const int32_t* k_ids, int2* k_sum, int Sk,
                          int nks, int tk, hipStream_t stream) {
  hipLaunchKernelGGL(doc_summary_kernel, dim3((tq + tk + 3) / 4), dim3(256), 0, stream, q_ids, q_sum, Sq, nqs, tq, k_ids, k_sum, Sk,
                     nks, tk);
}

// Degenerate Sk == 0: every row is fully masked, so out = 0 and lse = -inf.
__global__ void empty_keys_kernel(fl::View out, int out_f32, float* lse, int64_t lse_sb, int64_t lse_sg,
                                  int64_t lse_sh, int G, int H, int Sq, int Dv, int n_lse_g, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int i = (int)(idx % Sq);
  const int h = (int)((idx / Sq) % H);
  const int g = (int)((idx / ((int64_t)Sq * H)) % G);
  const int b = (int)(idx / ((int64_t)Sq * H * G));
  const int64_t o = b * out.sb + g * out.sg + h * out.sh + (int64_t)i * out.ss;
  for (int c = 0; c < Dv; ++c) {
    if (out_f32) ((float*)out.ptr)[o + c] = 0.f;
    else ((uint16_t*)out.ptr)[o + c] = 0;
  }
  if (lse != nullptr)
    for (int s = 0; s < n_lse_g; ++s)
      lse[b * lse_sb + (int64_t)(g * n_lse_g + s) * lse_sg + h * lse_sh + i] = -INFINITY;
}

struct BwdRegistry {
  const fl::BwdEntry* tab[2];
  int n[2];
  BwdRegistry() {
    tab[0] = fl::entries_bwd64(&n[0]);
    tab[1] = fl::entries_bwd128(&n[1]);
  }
};

// Can the backward kernel templates be instantiated for this variant at run time (head dim of the core kernels)?
bool bwd_jit_ok(const fl_variant_desc* d, int D, int nbias) {
  return (D == 64 || D == 128) && d->score_mod <= FL_MOD_SOFTCAP && nbias >= 0 && nbias <= 2;
}

// The compiled specialisation of the variant; with `instantiate`, otherwise one built from the kernel templates on first
// use (a few seconds, once per process and variant).
const fl::BwdEntry* find_bwd_entry(const fl_variant_desc* d, int D, int nbias = 0, bool instantiate = false) {
  static const BwdRegistry reg;                    // initialised once, also under concurrent first calls
  const fl::BwdEntry* const* tab = reg.tab;
  const int* n = reg.n;
  const int mask = (int)canonical_mask(d->mask);
  const fl::BwdEntry* same_dim = nullptr;
  for (int t = 0; t < 2; ++t)
    for (int e = 0; e < n[t]; ++e) {
      const fl::BwdEntry& k = tab[t][e];
      if (k.key.D == D && same_dim == nullptr) same_dim = &k;
      if (k.key.D == D && k.key.mod == (int)d->score_mod && k.key.mask == mask && k.key.nbias == nbias) return &k;
    }
  if (!instantiate || same_dim == nullptr || !bwd_jit_ok(d, D, nbias)) return nullptr;
  return fl::jit_backward_entry(D, (int)d->score_mod, (uint32_t)mask, nbias, same_dim->prep, same_dim->reduce);
}

hipError_t run_bwd_dq(const fl::BwdEntry* be, const fl::BwdParams& p, int nblocks, hipStream_t stream) {
  return be->jit != nullptr ? fl::jit_backward_launch(*be, 0, p, nblocks, stream) : be->dq(p, nblocks, stream);
}
hipError_t run_bwd_dkdv(const fl::BwdEntry* be, const fl::BwdParams& p, int nblocks, hipStream_t stream) {
  return be->jit != nullptr ? fl::jit_backward_launch(*be, 1, p, nblocks, stream) : be->dkdv(p, nblocks, stream);
}

bool bwd_desc_ok(const fl_variant_desc* d) { return d->n_bias == 0 && d->combine == FL_SINGLE && d->epilogue == 0; }

// Workspace of the backward pass: delta, lse2 ([B, G, H, Sq] floats each, 256-byte aligned), then
// the document-id summaries of the tile skipper.
struct BwdWorkspace {
  size_t stat_bytes, sum_bytes, part_bytes, total;
  int hsplit;
};
constexpr int kBwdKeysPerWg = 128;                 // keys per workgroup of the dK/dV kernels (BwdCfg::BM)

// Grouped-query heads: a dK/dV workgroup sums over the query heads of its group.  When that leaves
// the launch with too few workgroups, the group is cut into hsplit subsets whose fp32 partial
// sums a small kernel adds up afterwards.  Cutting pays while a workgroup keeps enough (head, 64-row
// query tile) items to amortise its partial sums: up to 1024 workgroups if at least 24 items remain
// each, up to 2048 if at least 256 remain (fitted to a sweep over the paper's grouped-head shapes).
int choose_hsplit(int64_t B, int64_t G, int64_t H, int64_t Hkv, int64_t Sq, int64_t Sk, uint32_t mask, int64_t window) {
  if (Hkv <= 0 || H <= Hkv || Sk <= 0) return 1;
  const int64_t group = H / Hkv, wgs = B * G * Hkv * ((Sk + kBwdKeysPerWg - 1) / kBwdKeysPerWg);
  int64_t rows = Sq;                               // query rows that can see a workgroup's keys
  if ((mask & FL_MASK_WINDOW) && window + kBwdKeysPerWg < rows) rows = window + kBwdKeysPerWg;
  const int64_t items = group * ((rows + 63) / 64);
  int hs = 1;
  if (g_tuning.bwd_wg_target > 0) {
    while (hs < group && wgs * hs < g_tuning.bwd_wg_target && group % (hs * 2) == 0) hs *= 2;
    return hs;
  }
  while (hs < group && group % (hs * 2) == 0 &&
         ((wgs * hs < 1024 && items / (2 * hs) >= 24) || (wgs * hs < 2048 && items / (2 * hs) >= 256)))
    hs *= 2;
  return hs;
}

BwdWorkspace bwd_workspace(int64_t B, int64_t G, int64_t H, int64_t Hkv, int64_t Sq, int64_t Sk, int64_t D,
                           uint32_t mask, int64_t window) {
  BwdWorkspace w;
  w.stat_bytes = ((size_t)(B * G * H * Sq) * sizeof(float) + 255) / 256 * 256;
  w.sum_bytes = (workspace_bytes(B, Sq, Sk, mask) + 255) / 256 * 256;
  w.hsplit = choose_hsplit(B, G, H, Hkv, Sq, Sk, mask, window);
  w.part_bytes = w.hsplit > 1 ? (size_t)w.hsplit * (size_t)(B * G * Hkv * Sk * D) * sizeof(float) : 0;
  w.total = 2 * w.stat_bytes + w.sum_bytes + 2 * w.part_bytes;
  return w;
}

const fl::DecodeEntry* find_decode_entry(int D, int mod, int cb) {
  int n = 0;
  const fl::DecodeEntry* tab = fl::entries_decode(&n);
  for (int e = 0; e < n; ++e)
    if (tab[e].D == D && tab[e].mod == mod && tab[e].cb == cb) return &tab[e];
  return nullptr;
}

// The decode kernels hold the (query row, head) pairs of a kv head as MFMA columns: at most two blocks of 32.
constexpr int64_t kDecodeMaxPairs = 64;

// Splits of a sequence's key range, a function of the shapes and the host-side length bound only.
// Measured on (sequences x kv heads) = 8 ... 2048 units and 1k ... 128k cached tokens: few units want
// about 512 workgroups in all (256 when tiles are scarce: a wave has one tile in flight, so more waves are what
// hides the latency of a tile on a nearly empty chip, down to 4 tiles per split); with hundreds of
// units three or four splits (by head dim) of at least 32 tiles even out the different sequence lengths; more than
// 32 splits never paid (every workgroup pays its start-up: length, first page lookups, first tiles).
int decode_splits(int64_t B, int64_t Hkv, int64_t D, int64_t max_seq_len) {
  const int64_t tiles = (max_seq_len + 31) / 32;
  const int64_t units = B * Hkv > 0 ? B * Hkv : 1;
  int64_t ns;
  if (g_tuning.decode_splits > 0) {
    ns = g_tuning.decode_splits;
    if (ns > tiles) ns = tiles;
  } else {
    // enough tiles: about 512 workgroups in all; otherwise about 256, with splits as short as 4 tiles (one per
    // wave) while the chip is nearly empty (<= 64 units), 16 beyond
    int64_t fill = (512 + units - 1) / units;
    if (tiles / fill < 16) {
      fill = (256 + units - 1) / units;
      const int64_t least = units <= 64 ? 4 : 16;
      if (fill > tiles / least) fill = tiles / least;
    }
    int64_t even = units >= 192 && units < 768 ? (D >= 128 ? 4 : 3) : (units >= 768 && units < 1536 ? 3 : 1);
    if (even > tiles / 32) even = tiles / 32;
    ns = fill > even ? fill : even;
    if (ns > 32) ns = 32;
  }
  return (int)(ns < 1 ? 1 : ns);
}


// ------------------------------------------------------------------------------------------------
// Backward pass of the variants with biases, gate, RMSNorm or a second stream (fl_attn_bwd_ex): the
// elementwise kernels around the per-stream backward kernels.
// ------------------------------------------------------------------------------------------------

// head dim the backward kernels run at for (D, Dv): tensors with a smaller one are zero-padded to it
int core_dim(int64_t D, int64_t Dv) { return (D > Dv ? D : Dv) <= 64 ? 64 : 128; }

struct EpiBwdParams {
  fl::View dout, out, gate, dgate;  // [B, G, H, Sq, Dv]; dgate.ptr null: not wanted
  const float* o[2];                // the streams' recomputed outputs, dense [rows, Dv] fp32 (null: not needed)
  const float* lse;                 // [B, ns * G, H, Sq]: stream s of row-axis g at ns * g + s
  int64_t lse_sb, lse_sg, lse_sh;
  uint16_t* d_o[2];                 // per-stream dO, dense [rows, Dc] bf16, channels past Dv zero
  float* delta[2];                  // per-stream rowsum(dO * O)
  float* lse2[2];                   // per-stream lse * log2(e), +inf for rows without a visible key
  const float* lambda;
  const float* rms_w;
  float* dl_rows;                   // per-row terms of dlambda (summed per head by reduce_dlambda_kernel), or null
  float* dw_part;                   // per-workgroup partial sums of the rms_weight gradient, [workgroups, Dv], or null
  float rms_eps;
  int32_t B, G, H, Sq, Dv, Dc;
  int32_t ns, has_gate, has_rms, dgate_f32;
};

// One wave per (b, g, h, i) row; lane c holds channels c and c + 64.
__global__ void __launch_bounds__(256) epi_bwd_kernel(const EpiBwdParams e) {
  const int64_t rows = (int64_t)e.B * e.G * e.H * e.Sq;
  const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  // rms_weight gradient: the four rows of a workgroup are added through LDS, the workgroups by reduce_drms_kernel
  __shared__ float dw_rows[4][128];
  auto dw_finish = [&](float t0, float t1) {         // every wave of the workgroup calls this exactly once (or none does)
    dw_rows[threadIdx.x >> 6][lane] = t0;
    dw_rows[threadIdx.x >> 6][lane + 64] = t1;
    __syncthreads();
    if ((int)threadIdx.x < e.Dv)
      e.dw_part[(int64_t)blockIdx.x * e.Dv + threadIdx.x] =
          (dw_rows[0][threadIdx.x] + dw_rows[1][threadIdx.x]) + (dw_rows[2][threadIdx.x] + dw_rows[3][threadIdx.x]);
  };
  if (row >= rows) {
    if (e.dw_part != nullptr) dw_finish(0.f, 0.f);
    return;
  }
  const int i = (int)(row % e.Sq);
  const int h = (int)((row / e.Sq) % e.H);
  const int g = (int)((row / ((int64_t)e.Sq * e.H)) % e.G);
  const int b = (int)(row / ((int64_t)e.Sq * e.H * e.G));
  auto off = [&](const fl::View& v) { return b * v.sb + g * v.sg + h * v.sh + (int64_t)i * v.ss; };
  auto wsum = [](float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
  };
  const bool need_o = e.o[0] != nullptr;
  const float lam = e.ns == 2 ? e.lambda[h] : 0.f;
  float dy[2], ov[2], x[2], o1[2], o2[2], wv[2];
  float sum_x2 = 0.f, sum_wdyx = 0.f, sum_dout_out = 0.f;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int c = lane + 64 * u;
    const bool ok = c < e.Dv;
    const float dv_ = ok ? fl::bf16_to_f32(((const uint16_t*)e.dout.ptr)[off(e.dout) + c]) : 0.f;
    ov[u] = ok ? fl::bf16_to_f32(((const uint16_t*)e.out.ptr)[off(e.out) + c]) : 0.f;
    dy[u] = dv_;
    if (e.has_gate) {
      const float gv = ok ? fl::bf16_to_f32(((const uint16_t*)e.gate.ptr)[off(e.gate) + c]) : 0.f;
      const float sg = 1.f / (1.f + __expf(-gv));
      dy[u] = dv_ * sg;
      if (ok && e.dgate.ptr != nullptr) {           // dout * y * sg (1 - sg) with out = y * sg
        const float dg = dv_ * ov[u] * (1.f - sg);
        if (e.dgate_f32) ((float*)e.dgate.ptr)[off(e.dgate) + c] = dg;
        else ((uint16_t*)e.dgate.ptr)[off(e.dgate) + c] = (uint16_t)(fl::pack_bf16(dg, 0.f) & 0xFFFFu);
      }
    }
    sum_dout_out += dv_ * ov[u];
    o1[u] = need_o && ok ? e.o[0][row * e.Dv + c] : 0.f;
    o2[u] = e.ns == 2 && ok ? e.o[1][row * e.Dv + c] : 0.f;
    x[u] = o1[u] - lam * o2[u];
    wv[u] = e.has_rms && ok ? (e.rms_w != nullptr ? e.rms_w[c] : 1.f) : 0.f;
    sum_x2 += x[u] * x[u];
    sum_wdyx += wv[u] * dy[u] * x[u];
  }
  float dx[2] = {dy[0], dy[1]};
  if (e.has_rms) {
    const float ms = wsum(sum_x2) / (float)e.Dv;
    const float r = sqrtf(ms + e.rms_eps);
    const float dot = wsum(sum_wdyx);
    const float c3 = dot / ((float)e.Dv * r * r * r);
#pragma unroll
    for (int u = 0; u < 2; ++u) dx[u] = wv[u] * dy[u] / r - x[u] * c3;
    if (e.dw_part != nullptr)                      // (channels past Dv carry dy = x = 0)
      dw_finish(dy[0] * x[0] / r, dy[1] * x[1] / r);
  }
  float d1 = 0.f, d2 = 0.f, dl = 0.f;
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int c = lane + 64 * u;
    if (c < e.Dc) {
      const bool ok = c < e.Dv;
      e.d_o[0][row * e.Dc + c] = ok ? (uint16_t)(fl::pack_bf16(dx[u], 0.f) & 0xFFFFu) : (uint16_t)0;
      if (e.ns == 2) e.d_o[1][row * e.Dc + c] = ok ? (uint16_t)(fl::pack_bf16(-lam * dx[u], 0.f) & 0xFFFFu) : (uint16_t)0;
    }
    d1 += dx[u] * o1[u];
    d2 += -lam * dx[u] * o2[u];
    dl += -dx[u] * o2[u];
  }
  // without recomputed outputs (one stream, no RMSNorm): delta = rowsum(dy * y) = rowsum(dout * out)
  d1 = need_o ? wsum(d1) : wsum(sum_dout_out);
  if (e.ns == 2) {
    d2 = wsum(d2);
    dl = wsum(dl);
  }
  if (lane == 0) {
    e.delta[0][row] = d1;
    if (e.ns == 2) {
      e.delta[1][row] = d2;
      if (e.dl_rows != nullptr) e.dl_rows[row] = dl;
    }
    for (int s = 0; s < e.ns; ++s) {
      const float l = e.lse[b * e.lse_sb + (int64_t)(e.ns * g + s) * e.lse_sg + h * e.lse_sh + i];
      e.lse2[s][row] = l == -INFINITY ? INFINITY : l * fl::kLog2e;
    }
  }
}

// The same with LPR lanes per row, eight channels per lane (16-byte loads and stores), 64 / LPR rows per wave: for tensors
// whose rows are 16-byte aligned (the host checks).  LPR = Dc / 8; lanes whose channels lie past Dv only write the zero
// padding of the per-stream dO.  The rms_weight partial sums are per workgroup as above, over 4 * 64 / LPR rows.
template <int LPR>
__global__ void __launch_bounds__(256) epi_bwd_rows_kernel(const EpiBwdParams e) {
  constexpr int RPW = 64 / LPR;
  const int64_t rows = (int64_t)e.B * e.G * e.H * e.Sq;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, sub = lane % LPR;
  const int64_t row_raw = ((int64_t)blockIdx.x * 4 + wave) * RPW + lane / LPR;
  const bool live = row_raw < rows;
  const int64_t row = live ? row_raw : rows - 1;
  const int c0 = sub * 8;
  const bool ok = live && c0 < e.Dv;               // Dv is a multiple of 8: a lane's channels are all inside or all outside
  const int i = (int)(row % e.Sq);
  const int h = (int)((row / e.Sq) % e.H);
  const int g = (int)((row / ((int64_t)e.Sq * e.H)) % e.G);
  const int b = (int)(row / ((int64_t)e.Sq * e.H * e.G));
  auto off = [&](const fl::View& v) { return b * v.sb + g * v.sg + h * v.sh + (int64_t)i * v.ss + c0; };
  auto gsum = [](float x) {                        // over the lanes of a row
#pragma unroll
    for (int o = LPR / 2; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
  };
  auto load8 = [&](const fl::View& v, float (&f)[8]) {
    uint4 q = make_uint4(0, 0, 0, 0);
    if (ok) q = *(const uint4*)((const uint16_t*)v.ptr + off(v));
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      f[2 * k] = __uint_as_float(w[k] << 16);
      f[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
    }
  };
  auto load8f = [&](const float* src, float (&f)[8]) {   // dense fp32 [rows, Dv] or [Dv]
    float4 a = make_float4(0.f, 0.f, 0.f, 0.f), c = a;
    if (ok) {
      a = *(const float4*)src;
      c = *(const float4*)(src + 4);
    }
    f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = c.x; f[5] = c.y; f[6] = c.z; f[7] = c.w;
  };
  auto pack8 = [](const float (&f)[8]) {
    return make_uint4(fl::pack_bf16(f[0], f[1]), fl::pack_bf16(f[2], f[3]), fl::pack_bf16(f[4], f[5]), fl::pack_bf16(f[6], f[7]));
  };
  const bool need_o = e.o[0] != nullptr;
  const float lam = e.ns == 2 ? e.lambda[h] : 0.f;
  float dout[8], ov[8], dy[8], o1[8], o2[8], x[8], wv[8], dx[8];
  load8(e.dout, dout);
  load8(e.out, ov);
#pragma unroll
  for (int k = 0; k < 8; ++k) dy[k] = dout[k];
  if (e.has_gate) {
    float gv[8], dg[8];
    load8(e.gate, gv);
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const float sg = 1.f / (1.f + __expf(-gv[k]));
      dy[k] = dout[k] * sg;
      dg[k] = dout[k] * ov[k] * (1.f - sg);        // dout * y * sg (1 - sg) with out = y * sg
    }
    if (ok && e.dgate.ptr != nullptr) {
      if (e.dgate_f32) {
        float* dst = (float*)e.dgate.ptr + off(e.dgate);
        *(float4*)dst = make_float4(dg[0], dg[1], dg[2], dg[3]);
        *(float4*)(dst + 4) = make_float4(dg[4], dg[5], dg[6], dg[7]);
      } else {
        *(uint4*)((uint16_t*)e.dgate.ptr + off(e.dgate)) = pack8(dg);
      }
    }
  }
#pragma unroll
  for (int k = 0; k < 8; ++k) o1[k] = o2[k] = wv[k] = 0.f;
  if (need_o) load8f(e.o[0] + row * e.Dv + c0, o1);
  if (e.ns == 2) load8f(e.o[1] + row * e.Dv + c0, o2);
  if (e.has_rms) {
    if (e.rms_w != nullptr) load8f(e.rms_w + c0, wv);
    else
#pragma unroll
      for (int k = 0; k < 8; ++k) wv[k] = ok ? 1.f : 0.f;
  }
  float sum_x2 = 0.f, sum_wdyx = 0.f, sum_dout_out = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    x[k] = o1[k] - lam * o2[k];
    sum_dout_out += dout[k] * ov[k];
    sum_x2 += x[k] * x[k];
    sum_wdyx += wv[k] * dy[k] * x[k];
    dx[k] = dy[k];
  }
  if (e.has_rms) {
    const float ms = gsum(sum_x2) / (float)e.Dv;
    const float r = sqrtf(ms + e.rms_eps);
    const float dot = gsum(sum_wdyx);
    const float c3 = dot / ((float)e.Dv * r * r * r);
#pragma unroll
    for (int k = 0; k < 8; ++k) dx[k] = wv[k] * dy[k] / r - x[k] * c3;
    if (e.dw_part != nullptr) {                    // rows of the wave by shuffles, waves of the workgroup through LDS
      __shared__ float dw_rows[4][LPR * 8];
      float t[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        t[k] = dy[k] * x[k] / r;                   // (channels past Dv and rows past the end carry dy = x = 0)
#pragma unroll
        for (int o = LPR; o < 64; o <<= 1) t[k] += __shfl_xor(t[k], o);
      }
      if (lane < LPR)
#pragma unroll
        for (int k = 0; k < 8; ++k) dw_rows[wave][c0 + k] = t[k];
      __syncthreads();
      if ((int)threadIdx.x < e.Dv)
        e.dw_part[(int64_t)blockIdx.x * e.Dv + threadIdx.x] =
            (dw_rows[0][threadIdx.x] + dw_rows[1][threadIdx.x]) + (dw_rows[2][threadIdx.x] + dw_rows[3][threadIdx.x]);
    }
  }
  float d1 = 0.f, d2 = 0.f, dl = 0.f;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    d1 += dx[k] * o1[k];
    d2 += -lam * dx[k] * o2[k];
    dl += -dx[k] * o2[k];
  }
  if (live && c0 < e.Dc) {
    float z[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) z[k] = ok ? dx[k] : 0.f;
    *(uint4*)(e.d_o[0] + row * e.Dc + c0) = pack8(z);
    if (e.ns == 2) {
#pragma unroll
      for (int k = 0; k < 8; ++k) z[k] = ok ? -lam * dx[k] : 0.f;
      *(uint4*)(e.d_o[1] + row * e.Dc + c0) = pack8(z);
    }
  }
  // without recomputed outputs (one stream, no RMSNorm): delta = rowsum(dy * y) = rowsum(dout * out)
  d1 = need_o ? gsum(d1) : gsum(sum_dout_out);
  if (e.ns == 2) {
    d2 = gsum(d2);
    dl = gsum(dl);
  }
  if (live && sub == 0) {
    e.delta[0][row] = d1;
    if (e.ns == 2) {
      e.delta[1][row] = d2;
      if (e.dl_rows != nullptr) e.dl_rows[row] = dl;
    }
    for (int s = 0; s < e.ns; ++s) {
      const float l = e.lse[b * e.lse_sb + (int64_t)(e.ns * g + s) * e.lse_sg + h * e.lse_sh + i];
      e.lse2[s][row] = l == -INFINITY ? INFINITY : l * fl::kLog2e;
    }
  }
}

// drms_weight[c] = sum over the workgroups' partial sums; one workgroup per channel, fixed summation order
__global__ void __launch_bounds__(256) reduce_drms_kernel(const float* dw_part, float* dw, int64_t nwg, int Dv) {
  __shared__ float part[256];
  const int c = blockIdx.x;
  float s = 0.f;
  for (int64_t t = threadIdx.x; t < nwg; t += 256) s += dw_part[t * Dv + c];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o >= 1; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) dw[c] = part[0];
}

// dlambda[h] = sum over (b, g, i) of the per-row terms; one workgroup per head, fixed summation order
__global__ void __launch_bounds__(256) reduce_dlambda_kernel(const float* dl_rows, float* dlambda, int B, int G, int H, int Sq) {
  __shared__ float part[256];
  const int h = blockIdx.x;
  float s = 0.f;
  const int64_t n = (int64_t)B * G * Sq;
  for (int64_t t = threadIdx.x; t < n; t += 256) {
    const int64_t bg = t / Sq;
    s += dl_rows[(bg * H + h) * Sq + t % Sq];
  }
  part[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o >= 1; o >>= 1) {
    if ((int)threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) dlambda[h] = part[0];
}

// Gradient of one bias from the staged dS (bf16 dense [B, G, H, Sq, Sk]): the sum over the axes the bias
// broadcasts along (its size-1 axes), one thread per output element, fixed summation order.
__global__ void __launch_bounds__(256) reduce_dbias_kernel(const uint16_t* ds, fl::BiasView out, int B, int G, int H, int Sq, int Sk,
                                                           int ob, int og, int oh, int oi, int oj, int64_t total, int accumulate) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int j = (int)(idx % oj), i = (int)((idx / oj) % oi), h = (int)((idx / ((int64_t)oj * oi)) % oh);
  const int g = (int)((idx / ((int64_t)oj * oi * oh)) % og), b = (int)(idx / ((int64_t)oj * oi * oh * og));
  const int nb = ob == 1 ? B : 1, ng = og == 1 ? G : 1, nh = oh == 1 ? H : 1, ni = oi == 1 ? Sq : 1, nj = oj == 1 ? Sk : 1;
  float s = 0.f;
  for (int bb = 0; bb < nb; ++bb)
    for (int gg = 0; gg < ng; ++gg)
      for (int hh = 0; hh < nh; ++hh)
        for (int ii = 0; ii < ni; ++ii) {
          const uint16_t* row = ds + ((((int64_t)(b + bb) * G + (g + gg)) * H + (h + hh)) * Sq + (i + ii)) * Sk + j;
          for (int jj = 0; jj < nj; ++jj) s += fl::bf16_to_f32(row[jj]);
        }
  float* dst = (float*)out.ptr + b * out.sb + g * out.sg + h * out.sh + (int64_t)i * out.si + (int64_t)j * out.sj;
  *dst = accumulate ? *dst + s : s;                // the second softmax stream adds to the first one's sum
}

// The same for a bias that is not broadcast along the keys, Sk a multiple of 8 and a gradient tensor with unit key stride
// and 16-byte aligned rows: eight keys per thread (one 16-byte load per staged row), four rows in flight.  The terms of an
// output element are added in the same order as above.
__global__ void __launch_bounds__(256) reduce_dbias_vec8_kernel(const uint16_t* ds, fl::BiasView out, int B, int G, int H, int Sq, int Sk,
                                                                int ob, int og, int oh, int oi, int64_t total8, int accumulate) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total8) return;
  const int oj8 = Sk / 8;
  const int j = (int)(idx % oj8) * 8, i = (int)((idx / oj8) % oi), h = (int)((idx / ((int64_t)oj8 * oi)) % oh);
  const int g = (int)((idx / ((int64_t)oj8 * oi * oh)) % og), b = (int)(idx / ((int64_t)oj8 * oi * oh * og));
  const int nb = ob == 1 ? B : 1, ng = og == 1 ? G : 1, nh = oh == 1 ? H : 1, ni = oi == 1 ? Sq : 1;
  const int64_t n_terms = (int64_t)nb * ng * nh * ni;
  auto term = [&](int64_t n) -> const uint4* {     // n-th staged row of this output, in the nesting order b, g, h, i
    const int ii = (int)(n % ni), hh = (int)((n / ni) % nh), gg = (int)((n / ((int64_t)ni * nh)) % ng);
    const int bb = (int)(n / ((int64_t)ni * nh * ng));
    return (const uint4*)(ds + ((((int64_t)(b + bb) * G + (g + gg)) * H + (h + hh)) * Sq + (i + ii)) * Sk + j);
  };
  float s[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) s[k] = 0.f;
  auto add = [&](const uint4& v) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      s[2 * k] += __uint_as_float(w[k] << 16);
      s[2 * k + 1] += __uint_as_float(w[k] & 0xFFFF0000u);
    }
  };
  int64_t n = 0;
  for (; n + 4 <= n_terms; n += 4) {
    const uint4 v0 = *term(n), v1 = *term(n + 1), v2 = *term(n + 2), v3 = *term(n + 3);
    add(v0); add(v1); add(v2); add(v3);
  }
  for (; n < n_terms; ++n) add(*term(n));
  float4* dst = (float4*)((float*)out.ptr + b * out.sb + g * out.sg + h * out.sh + (int64_t)i * out.si + j);
  if (accumulate) {                                // the second softmax stream adds to the first one's sum
    const float4 a = dst[0], c = dst[1];
    s[0] += a.x; s[1] += a.y; s[2] += a.z; s[3] += a.w;
    s[4] += c.x; s[5] += c.y; s[6] += c.z; s[7] += c.w;
  }
  dst[0] = make_float4(s[0], s[1], s[2], s[3]);
  dst[1] = make_float4(s[4], s[5], s[6], s[7]);
}

// bf16 [B, G, H, S, D] view -> dense [B, G, H, S, Dc] with zero channels past D (8 channels per thread)
__global__ void __launch_bounds__(256) pad_rows_kernel(fl::View src, uint16_t* dst, int G, int H, int S, int D, int Dc, int64_t rows) {
  const int cpr = Dc / 8;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * cpr) return;
  const int64_t row = idx / cpr;
  const int c = (int)(idx % cpr) * 8;
  const int i = (int)(row % S), h = (int)((row / S) % H), g = (int)((row / ((int64_t)S * H)) % G);
  const int b = (int)(row / ((int64_t)S * H * G));
  uint4 v = make_uint4(0, 0, 0, 0);
  if (c < D) v = *(const uint4*)((const uint16_t*)src.ptr + b * src.sb + g * src.sg + h * src.sh + (int64_t)i * src.ss + c);
  *(uint4*)(dst + row * Dc + c) = v;
}

// dense fp32 [B, G, H, S, Dc] (optionally the sum of two) -> the first D channels of a [B, G, H, S, D] view, bf16 or fp32
__global__ void __launch_bounds__(256) scatter_grad_kernel(const float* a, const float* b2, fl::View dst, int dst_f32, int G, int H,
                                                           int S, int D, int Dc, int64_t rows) {
  const int cpr = D / 4;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * cpr) return;
  const int64_t row = idx / cpr;
  const int c = (int)(idx % cpr) * 4;
  const int i = (int)(row % S), h = (int)((row / S) % H), g = (int)((row / ((int64_t)S * H)) % G);
  const int b = (int)(row / ((int64_t)S * H * G));
  float4 v = *(const float4*)(a + row * Dc + c);
  if (b2 != nullptr) {
    const float4 w = *(const float4*)(b2 + row * Dc + c);
    v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w;
  }
  const int64_t o = b * dst.sb + g * dst.sg + h * dst.sh + (int64_t)i * dst.ss + c;
  if (dst_f32) *(float4*)((float*)dst.ptr + o) = v;
  else *(uint2*)((uint16_t*)dst.ptr + o) = make_uint2(fl::pack_bf16(v.x, v.y), fl::pack_bf16(v.z, v.w));
}

// zero-fill (dS staging under masks that skip blocks)
__global__ void __launch_bounds__(256) zero_f32_kernel(float* p, int64_t n) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx < n) p[idx] = 0.f;
}

inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

// Chunked prefill over the paged cache: copies each sequence's cached rows, token by token through its block table, into
// a dense [B, 1, Hkv, L, D] tensor, row j holding token j.  Rows at and after the sequence's length are left as they are:
// the forward kernel is told the length and reads no row past it.  One thread per 16-byte chunk; k and v in one launch
// (blockIdx.y).
struct GatherParams {
  const uint16_t* cache[2];
  int64_t sp[2], st[2], sh[2];
  uint16_t* dst[2];
  const int* table;
  const int* seq_lens;
  int table_stride, page_shift, page_mask, num_pages, max_len, Hkv, L, chunks;     // chunks = D / 8
  int64_t total;                                                                  // B * Hkv * L * chunks
};

__global__ void __launch_bounds__(256) gather_pages_kernel(GatherParams g) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= g.total) return;
  const int which = blockIdx.y;
  const int c = (int)(idx % g.chunks);
  int64_t rest = idx / g.chunks;
  const int j = (int)(rest % g.L);
  rest /= g.L;
  const int hk = (int)(rest % g.Hkv);
  const int b = (int)(rest / g.Hkv);
  const int len = max(0, min(g.seq_lens[b], g.max_len));
  if (j >= len) return;
  int page = b, within = j;
  if (g.table != nullptr) {
    page = max(0, min(g.table[(int64_t)b * g.table_stride + (j >> g.page_shift)], g.num_pages - 1));
    within = j & g.page_mask;
  }
  *(uint4*)(g.dst[which] + idx * 8) =
      *(const uint4*)(g.cache[which] + page * g.sp[which] + hk * g.sh[which] + within * g.st[which] + c * 8);
}

// Workspace of fl_attn_prefill_paged (byte offsets; both regions 256-byte aligned).
struct PrefillLayout {
  int64_t L;
  size_t off_k, off_v, total;
};

PrefillLayout prefill_layout(int64_t B, int64_t Hkv, int64_t D, int64_t max_len) {
  PrefillLayout L;
  L.L = std::max<int64_t>(max_len, 1);
  const size_t kv_bytes = up256((size_t)(B * Hkv * L.L * D) * 2);
  L.off_k = 0;
  L.off_v = kv_bytes;
  L.total = 2 * kv_bytes;
  return L;
}

// Workspace of fl_attn_bwd_ex (byte offsets; every region 256-byte aligned).
struct ExLayout {
  int Dc, ns, hsplit;
  bool need_o, pad_qk, pad_v;
  size_t stat, o, d_o, qpad, kpad, vpad, gq, gk, gv, sum, part, ds;   // sizes of one region each
  size_t off_lse2[2], off_delta[2], off_o[2], off_do[2], off_qpad[2], off_kpad[2], off_vpad, off_gq[2], off_gk[2], off_gv[2],
      off_sum, off_part, off_dl, off_ds, off_dw;
  size_t total;
};
ExLayout ex_layout(int64_t B, int64_t G, int64_t H, int64_t Hkv, int64_t Sq, int64_t Sk, int64_t D, int64_t Dv,
                   const fl_variant_desc* d) {
  ExLayout L;
  memset(&L, 0, sizeof(L));
  const uint32_t mask = canonical_mask(d->mask);
  L.Dc = core_dim(D, Dv);
  L.ns = d->combine == FL_DIFFERENTIAL ? 2 : 1;
  L.need_o = L.ns == 2 || (d->epilogue & FL_EPI_RMSNORM) != 0;
  L.pad_qk = D != L.Dc;
  L.pad_v = Dv != L.Dc;
  const size_t rq = (size_t)(B * G * H * Sq), rk = (size_t)(B * G * Hkv * Sk);
  L.stat = up256(rq * 4);
  L.o = L.need_o ? up256(rq * Dv * 4) : 0;
  L.d_o = up256(rq * L.Dc * 2);
  L.qpad = L.pad_qk ? up256(rq * L.Dc * 2) : 0;
  L.kpad = L.pad_qk ? up256(rk * L.Dc * 2) : 0;
  L.vpad = L.pad_v ? up256(rk * L.Dc * 2) : 0;
  L.gq = up256(rq * L.Dc * 4);
  L.gk = up256(rk * L.Dc * 4);
  L.gv = up256(rk * L.Dc * 4);
  L.sum = up256(workspace_bytes(B, Sq, Sk, mask));
  L.hsplit = choose_hsplit(B, G, H, Hkv, Sq, Sk, mask, clamp_window(d->window, Sq, Sk));
  L.part = L.hsplit > 1 ? up256((size_t)L.hsplit * rk * L.Dc * 4) : 0;
  size_t at = 0;
  auto take = [&](size_t n) { const size_t o = at; at += n; return o; };
  for (int s = 0; s < L.ns; ++s) {
    L.off_lse2[s] = take(L.stat);
    L.off_delta[s] = take(L.stat);
    L.off_o[s] = take(L.o);
    L.off_do[s] = take(L.d_o);
    L.off_qpad[s] = take(L.qpad);
    L.off_kpad[s] = take(L.kpad);
    L.off_gq[s] = take(L.gq);
    L.off_gk[s] = take(L.gk);
    L.off_gv[s] = take(L.gv);
  }
  L.off_vpad = take(L.vpad);
  L.off_sum = take(L.sum);
  L.off_part = take(2 * L.part);
  L.off_dl = take(L.ns == 2 ? L.stat : 0);
  // bias gradients: dS of every score (bf16), reduced over the broadcast axes afterwards
  L.ds = d->n_bias > 0 ? up256(rq * (size_t)Sk * 2) : 0;
  L.off_ds = take(L.ds);
  // rms_weight gradient: one partial sum per workgroup (four rows) of the epilogue-derivative kernel
  L.off_dw = take((d->epilogue & FL_EPI_RMSNORM) != 0 ? up256(((rq + 3) / 4) * (size_t)Dv * 4) : 0);
  L.total = at;
  return L;
}

// Is the variant one the plain backward entry point (no extra outputs, no padding) takes?
bool bwd_simple(const fl_variant_desc* d, int64_t D, int64_t Dv) {
  return bwd_desc_ok(d) && D == Dv && (D == 64 || D == 128);
}
// Can fl_attn_bwd_ex build the variant from the backward kernels?
bool bwd_ex_ok(const fl_variant_desc* d, int64_t D, int64_t Dv) {
  if (!((D == 32 || D == 64 || D == 128) && (Dv == 32 || Dv == 64 || Dv == 128))) return false;
  return find_bwd_entry(d, core_dim(D, Dv), (int)d->n_bias) != nullptr || bwd_jit_ok(d, core_dim(D, Dv), (int)d->n_bias);
}

fl::View dense_view(void* ptr, int64_t G, int64_t H, int64_t S, int64_t Dc) {
  fl::View v;
  v.ptr = ptr;
  v.ss = Dc;
  v.sh = S * Dc;
  v.sg = H * S * Dc;
  v.sb = G * H * S * Dc;
  return v;
}

}  // namespace

extern "C" {

uint32_t fl_version(void) { return (1u << 16) | 0u; }

const char* fl_strerror(fl_status s) {
  switch (s) {
    case FL_OK: return "ok";
    case FL_ERR_NULL: return "required pointer is NULL";
    case FL_ERR_DTYPE: return "unsupported dtype combination";
    case FL_ERR_SHAPE: return "inconsistent tensor sizes";
    case FL_ERR_STRIDE: return "unsupported stride";
    case FL_ERR_ALIGN: return "pointer or stride not 16-byte aligned";
    case FL_ERR_UNSUPPORTED: return "no compiled specialisation for this variant / head dim";
    case FL_ERR_AUX_MISSING: return "descriptor needs an aux tensor that was not given";
    case FL_ERR_WORKSPACE: return "workspace missing or too small";
    case FL_ERR_LAUNCH: return "HIP launch failed";
    case FL_ERR_DESC: return "invalid variant descriptor";
  }
  return "unknown status";
}

const char* fl_last_error_detail(void) { return g_detail; }

fl_status fl_set_tuning(const char* key, int value) {
  if (key == nullptr) return fail(FL_ERR_NULL, "key is NULL");
  if (value < 0) return fail(FL_ERR_UNSUPPORTED, "negative tuning value");
  if (!strcmp(key, "bm")) g_tuning.bm = value;
  else if (!strcmp(key, "bn")) g_tuning.bn = value;
  else if (!strcmp(key, "rb")) g_tuning.rb = value;
  else if (!strcmp(key, "nw")) g_tuning.nw = value;
  else if (!strcmp(key, "wpe")) g_tuning.wpe = value;
  else if (!strcmp(key, "ring")) g_tuning.ring = value;
  else if (!strcmp(key, "order")) g_tuning.order = value == 0 ? -1 : value - 1;
  else if (!strcmp(key, "pair")) g_tuning.pair = value == 0 ? -1 : value - 1;
  else if (!strcmp(key, "decode_splits")) g_tuning.decode_splits = value;
  else if (!strcmp(key, "prefill_pack")) g_tuning.prefill_pack = value;
  else if (!strcmp(key, "prefill_gather")) g_tuning.prefill_gather = value;
  else if (!strcmp(key, "bwd_wg_target")) g_tuning.bwd_wg_target = value;
  else return fail(FL_ERR_UNSUPPORTED, "unknown tuning key '%s'", key);
  return FL_OK;
}

int fl_variant_supported(const fl_variant_desc* desc, int dtype, int D, int Dv) {
  if (check_desc(desc) != FL_OK) return 0;
  if (dtype == FL_F32 && (D % 4 != 0 || Dv % 4 != 0 || D <= 0 || Dv <= 0)) return 0;
  if (find_entry(desc, dtype, D, Dv) != nullptr) return 1;
  return dtype == FL_BF16 && jit_dims_ok(D, Dv) ? 1 : 0;     // instantiated from the kernel template on first use
}

size_t fl_attn_fwd_workspace_size(const fl_tensor* q, const fl_tensor* k, const fl_variant_desc* desc) {
  if (q == nullptr || k == nullptr || desc == nullptr) return 0;
  return workspace_bytes(q->size[0], q->size[3], k->size[3], desc->mask);
}

// Keys and values read in place from a paged cache (fl_attn_prefill_paged): k and v of the call are then the cache
// tensors [pages, 1, Hkv, page_size, D], already validated by the caller.
struct PagedKeys {
  const int32_t* block_table;     // device, or NULL: sequence b is page b
  int table_stride, page_shift, num_pages;
  int64_t max_len;                // host-side bound of the sequence lengths: the key count the launch is sized for
};

// The forward call behind fl_attn_fwd.  kv_lens (device, [B], or NULL) gives every sequence its own number of keys and puts
// its query rows at the last Sq positions of those (fl_attn_prefill_paged); bf16 kernels without a document mask only.
static fl_status forward_call(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_variant_desc* desc,
                              const fl_aux* aux, fl_tensor* out, fl_tensor* lse, void* stream_v, const int32_t* kv_lens,
                              const PagedKeys* paged = nullptr) {
  g_detail[0] = 0;
  fl_status st = check_desc(desc);
  if (st != FL_OK) return st;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr) return fail(FL_ERR_NULL, "q, k, v or out is NULL");
  if (aux != nullptr && aux->struct_size != sizeof(fl_aux))
    return fail(FL_ERR_DESC, "aux->struct_size = %u, expected %zu", aux->struct_size, sizeof(fl_aux));

  const int dtype = q->dtype;
  if (dtype != FL_BF16 && dtype != FL_F32) return fail(FL_ERR_DTYPE, "q dtype %d not bf16/f32", dtype);
  const int64_t B = q->size[0], G = q->size[1], H = q->size[2], Sq = q->size[3], D = q->size[4];
  const int64_t Hkv = k->size[2], Sk = paged != nullptr ? paged->max_len : k->size[3], Dv = v->size[4];
  if (B < 0 || G < 0 || H < 0 || Sq < 0 || Sk < 0 || D <= 0 || Dv <= 0) return fail(FL_ERR_SHAPE, "negative size");
  if (Sq > 0x7fffff00LL || Sk > 0x7fffff00LL || B * G * H > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "size too large");
  if (Hkv <= 0 || H % (Hkv > 0 ? Hkv : 1) != 0)
    if (H != 0) return fail(FL_ERR_SHAPE, "k heads (%lld) must divide q heads (%lld)", (long long)Hkv, (long long)H);
  const bool empty = (B == 0 || G == 0 || H == 0 || Sq == 0);

  const int64_t qsz[5] = {B, G, H, Sq, D}, ksz[5] = {B, G, Hkv, Sk, D}, vsz[5] = {B, G, Hkv, Sk, Dv},
                osz[5] = {B, G, H, Sq, Dv};
  const bool diff = desc->combine == FL_DIFFERENTIAL;
  if (!empty) {
    if ((st = check_data_tensor(q, "q", dtype, qsz)) != FL_OK) return st;
    if (Sk > 0 && paged == nullptr) {
      if ((st = check_data_tensor(k, "k", dtype, ksz)) != FL_OK) return st;
      if ((st = check_data_tensor(v, "v", dtype, vsz)) != FL_OK) return st;
    }
    if (out->dtype != dtype && out->dtype != FL_F32) return fail(FL_ERR_DTYPE, "out dtype %d", out->dtype);
    if ((st = check_data_tensor(out, "out", out->dtype, osz)) != FL_OK) return st;
  }
  const uint32_t mask = canonical_mask(desc->mask);

  // ---- aux requirements
  const bool need_aux = desc->score_mod == FL_MOD_ALIBI || (mask & FL_MASK_DOC) || desc->n_bias > 0 || diff ||
                        (desc->epilogue & FL_EPI_GATE_SIGMOID);
  if (need_aux && aux == nullptr) return fail(FL_ERR_AUX_MISSING, "descriptor needs aux but aux is NULL");
  if (desc->score_mod == FL_MOD_ALIBI && aux->alibi_slopes == nullptr) return fail(FL_ERR_AUX_MISSING, "alibi_slopes");
  if ((mask & FL_MASK_DOC) && (aux->q_doc_ids == nullptr || aux->kv_doc_ids == nullptr))
    return fail(FL_ERR_AUX_MISSING, "q_doc_ids / kv_doc_ids");
  if (diff && aux->lambda == nullptr) return fail(FL_ERR_AUX_MISSING, "lambda");

  fl::FwdParams p;
  memset(&p, 0, sizeof(p));
  if (!empty) {
    if (diff && Sk > 0) {
      if ((st = check_data_tensor(&aux->q2, "q2", dtype, qsz)) != FL_OK) return st == FL_ERR_NULL ? fail(FL_ERR_AUX_MISSING, "q2") : st;
      if ((st = check_data_tensor(&aux->k2, "k2", dtype, ksz)) != FL_OK) return st == FL_ERR_NULL ? fail(FL_ERR_AUX_MISSING, "k2") : st;
      p.q2 = make_view(&aux->q2);
      p.k2 = make_view(&aux->k2);
    }
    if (desc->epilogue & FL_EPI_GATE_SIGMOID) {
      if ((st = check_data_tensor(&aux->gate, "gate", dtype, osz)) != FL_OK) return st == FL_ERR_NULL ? fail(FL_ERR_AUX_MISSING, "gate") : st;
      p.gate = make_view(&aux->gate);
    }
    for (uint32_t nb = 0; nb < desc->n_bias; ++nb) {
      const fl_tensor* bt = &aux->bias[nb];
      if (bt->ptr == nullptr) return fail(FL_ERR_AUX_MISSING, "bias[%u]", nb);
      if (bt->dtype != FL_BF16 && bt->dtype != FL_F32) return fail(FL_ERR_DTYPE, "bias[%u] dtype %d", nb, bt->dtype);
      const int64_t want[5] = {B, G, H, Sq, Sk};
      int64_t bs[5];
      for (int a = 0; a < 5; ++a) {
        if (bt->size[a] != want[a] && bt->size[a] != 1)
          return fail(FL_ERR_SHAPE, "bias[%u] size[%d] = %lld, expected %lld or 1", nb, a, (long long)bt->size[a],
                      (long long)want[a]);
        bs[a] = (bt->size[a] == 1 && want[a] != 1) ? 0 : bt->stride[a];
        if (bs[a] < 0) return fail(FL_ERR_STRIDE, "bias[%u] stride[%d] negative", nb, a);
      }
      if (Sk > 1 && bs[4] != 1 && bs[4] != 0) return fail(FL_ERR_STRIDE, "bias[%u] innermost stride must be 1 or 0", nb);
      fl::BiasView& bv = p.bias[nb];
      bv.ptr = bt->ptr;
      bv.sb = bs[0]; bv.sg = bs[1]; bv.sh = bs[2]; bv.si = bs[3]; bv.sj = Sk > 1 ? bs[4] : 0;
      bv.is_f32 = bt->dtype == FL_F32;
      if (dtype == FL_BF16 && bv.is_f32) return fail(FL_ERR_DTYPE, "bias[%u]: bf16 inputs take bf16 biases", nb);
      bv.vec4 = bs[4] == 1 && Sk > 1 && ((uintptr_t)bt->ptr) % 8 == 0 && bs[0] % 4 == 0 && bs[1] % 4 == 0 &&
                bs[2] % 4 == 0 && bs[3] % 4 == 0;
      // per-query rows that start 16-byte aligned: whole tiles go through LDS (decided below, with the LDS budget)
      bv.dma = dtype == FL_BF16 && bs[4] == 1 && bs[3] != 0 && ((uintptr_t)bt->ptr) % 16 == 0 && bs[0] % 8 == 0 &&
               bs[1] % 8 == 0 && bs[2] % 8 == 0 && bs[3] % 8 == 0;
    }
  }

  // ---- lse
  const bool want_lse = lse != nullptr && lse->ptr != nullptr;
  if (want_lse && !empty) {
    if (lse->dtype != FL_F32) return fail(FL_ERR_DTYPE, "lse must be f32");
    const int64_t lsz[5] = {B, diff ? 2 * G : G, H, Sq, 1};
    for (int a = 0; a < 5; ++a)
      if (lse->size[a] != lsz[a])
        return fail(FL_ERR_SHAPE, "lse size[%d] = %lld, expected %lld", a, (long long)lse->size[a], (long long)lsz[a]);
    if (Sq > 1 && lse->stride[3] != 1) return fail(FL_ERR_STRIDE, "lse must be contiguous along Sq");
    for (int a = 0; a < 3; ++a)
      if (lse->stride[a] < 0) return fail(FL_ERR_STRIDE, "lse stride[%d] negative", a);
    if (((uintptr_t)lse->ptr) % 4 != 0) return fail(FL_ERR_ALIGN, "lse pointer not 4-byte aligned");
  }

  // ---- specialisation lookup (before the empty-problem return so unsupported is reported)
  if (dtype == FL_F32) {
    if (D % 4 != 0 || Dv % 4 != 0) return fail(FL_ERR_UNSUPPORTED, "f32 head dims must be multiples of 4");
    if (!empty && out->dtype != FL_F32) return fail(FL_ERR_DTYPE, "f32 inputs need f32 out");
  }
  // (of the kernels that read a paged cache in place only the causal one is in the table)
  PagedShape shape = {1, false};
  if (paged != nullptr) shape = paged_shape(B * G * H, Hkv > 0 ? H / Hkv : 1, Sq);
  // Dense keys: a chunk of fewer than 128 query rows of grouped heads against 1024 keys or more (a query offset into a
  // long key sequence, typically) leaves part of the smallest tile empty; where packing fills it better by a fifth
  // (paged_shape), the kernel shapes with packed heads are instantiated on first use.
  const bool can_pack = paged == nullptr && dtype == FL_BF16 && !diff && desc->n_bias == 0 && desc->epilogue == 0 &&
                        (mask & FL_MASK_DOC) == 0 && D == Dv && Sq < 128 && Sk >= 1024 && Hkv > 0 && H / Hkv > 1 && !empty &&
                        !(g_tuning.bm || g_tuning.bn || g_tuning.rb || g_tuning.nw || g_tuning.wpe || g_tuning.ring);
  if (can_pack) {
    shape = paged_shape(B * G * H, H / Hkv, Sq);
    if (shape.pack == 1) shape.wide = false;
  }
  const bool packed = can_pack && shape.pack > 1;
  const fl::KernelEntry* ke = find_entry(desc, dtype, (int)D, (int)Dv, Sk, B * G * H, Sq, paged != nullptr ? &shape : nullptr,
                                         packed ? &shape : nullptr);
  if (ke == nullptr && dtype == FL_BF16 && jit_dims_ok(D, Dv)) {
    // not in the compiled table: the same kernel template, instantiated for this descriptor on first use
    ke = fl::jit_forward_entry(fl::JitRequest{(int)D, (int)Dv, (int)desc->score_mod, mask, (int)desc->n_bias, diff, desc->epilogue,
                                              paged != nullptr, (paged != nullptr || packed) && shape.wide, shape.pack});
    if (ke == nullptr) {
      char why[300];
      snprintf(why, sizeof(why), "%s", g_detail);
      return fail(FL_ERR_UNSUPPORTED, "run-time specialisation failed: %.290s", why);
    }
  }
  if (ke == nullptr)
    return fail(FL_ERR_UNSUPPORTED,
                "no specialisation for dtype=%d D=%lld Dv=%lld score_mod=%u mask=0x%x n_bias=%u combine=%u epilogue=0x%x",
                dtype, (long long)D, (long long)Dv, desc->score_mod, mask, desc->n_bias, desc->combine, desc->epilogue);

  const size_t ws_need = workspace_bytes(B, Sq, Sk, mask);
  if (ws_need > 0 && !empty && Sk > 0) {
    if (aux->workspace == nullptr || aux->workspace_bytes < ws_need)
      return fail(FL_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", ws_need, aux->workspace ? aux->workspace_bytes : (size_t)0);
    if (((uintptr_t)aux->workspace) % 8 != 0) return fail(FL_ERR_ALIGN, "workspace not 8-byte aligned");
  }
  if (empty) return FL_OK;

  // ---- parameter block
  p.q = make_view(q);
  p.out = make_view(out);
  if (Sk > 0) {
    p.k = make_view(k);
    p.v = make_view(v);
  }
  if (want_lse) {
    p.lse = (float*)lse->ptr;
    p.lse_sb = lse->size[0] > 1 ? lse->stride[0] : 0;
    p.lse_sg = lse->size[1] > 1 ? lse->stride[1] : 0;
    p.lse_sh = lse->size[2] > 1 ? lse->stride[2] : 0;
  }
  if (aux != nullptr) {
    p.alibi_slopes = aux->alibi_slopes;
    p.lambda = aux->lambda;
    p.rms_weight = aux->rms_weight;
    p.q_doc = aux->q_doc_ids;
    p.kv_doc = aux->kv_doc_ids;
  }
  p.B = (int)B; p.G = (int)G; p.H = (int)H; p.Hkv = (int)Hkv; p.Sq = (int)Sq; p.Sk = (int)Sk;
  p.D = (int)D; p.Dv = (int)Dv;
  p.window = clamp_window(desc->window, kv_lens != nullptr ? std::max(Sq, Sk) : Sq + desc->q_offset, Sk);
  p.prefix = desc->prefix_len;
  p.q_off = desc->q_offset;
  if ((int64_t)desc->q_offset + Sq > 0x7fffff00LL) return fail(FL_ERR_SHAPE, "q_offset + Sq too large");
  if (kv_lens != nullptr && (dtype != FL_BF16 || (mask & FL_MASK_DOC) || desc->q_offset != 0))
    return fail(FL_ERR_UNSUPPORTED, "per-sequence key counts: bf16, no document mask, no query offset");
  p.kv_lens = kv_lens;
  if (paged != nullptr) {
    if (kv_lens == nullptr || G != 1 || D != Dv || desc->n_bias != 0 || diff)
      return fail(FL_ERR_UNSUPPORTED, "paged keys: per-sequence lengths, one row axis, D == Dv, no bias, one stream");
    p.block_table = paged->block_table;
    p.table_stride = paged->table_stride;
    p.page_shift = paged->page_shift;
    p.page_mask = (1 << paged->page_shift) - 1;
    p.num_pages = paged->num_pages;
  }
  p.scale = desc->scale;
  p.softcap = desc->softcap;
  p.rms_eps = desc->rms_eps;
  p.out_f32 = out->dtype == FL_F32;
  p.mod = (int)desc->score_mod;
  p.mask = (int)mask;
  p.n_bias = (int)desc->n_bias;
  p.epi = (int)desc->epilogue;
  p.n_qtiles = (int)((Sq + ke->bm - 1) / ke->bm);
  if (dtype == FL_BF16) {
    // dynamic LDS: the K/V rings, then two staging buffers per wave and bias for the bias tiles
    // that are read through LDS
    const int64_t kv = ke->lds_bytes;
    for (int nb = ke->key.nbias; nb < 2; ++nb) p.bias[nb].dma = 0;
    const int n_stage = p.bias[1].dma ? 2 : (p.bias[0].dma ? 1 : 0);       // biases 0 .. n_stage-1 get buffers
    const int64_t per_wave = (int64_t)n_stage * 2 * (32 * ke->key.rb * ke->key.bn * 2);
    const int64_t stage = ke->key.nwaves * per_wave;
    const bool staged = n_stage > 0 && kv + stage <= (ke->max_lds > 0 ? ke->max_lds : fl::kMaxLdsBytes);
    if (!staged) p.bias[0].dma = p.bias[1].dma = 0;
    p.bias_lds_base = (int)kv;
    p.bias_lds_wave = staged ? (int)per_wave : 0;
    p.lds_bytes = (int)(kv + (staged ? stage : 0));
  }
  const int64_t nbh = B * G * H / ke->key.pack;    // (packed heads: a workgroup takes key.pack heads of one kv head)
  // bf16 kernels under a causal / prefix mask without a window: the work of a q-tile grows with
  // its index, so a workgroup takes a long and a short one -- when that still leaves every CU
  // several workgroups
  const bool tri = (mask & (FL_MASK_CAUSAL | FL_MASK_PREFIX)) != 0 && (mask & (FL_MASK_WINDOW | FL_MASK_DOC)) == 0;
  p.pair = g_tuning.pair >= 0 ? g_tuning.pair : (dtype == FL_BF16 && tri && nbh * ((p.n_qtiles + 1) / 2) >= 512);
  if (dtype != FL_BF16) p.pair = 0;
  const int64_t nblocks = nbh * (p.pair ? (p.n_qtiles + 1) / 2 : p.n_qtiles);
  if (nblocks > 0x7fffffffLL || nbh * Sq > 0x7fffffff00LL) return fail(FL_ERR_SHAPE, "too many workgroups");
  // default: XCD-aware order (whole (b, g, h) problems per XCD) whenever the problem count allows it
  int order = g_tuning.order >= 0 ? g_tuning.order : 1;
  if (order == 1 && nbh % 8 != 0) order = 0;
  p.order = order;
  p.doc_vec = (mask & FL_MASK_DOC) && Sk % 4 == 0 && ((uintptr_t)aux->kv_doc_ids) % 16 == 0;

  hipStream_t stream = (hipStream_t)stream_v;
  if (Sk == 0) {
    const int64_t total = B * G * H * Sq;
    hipLaunchKernelGGL(empty_keys_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, p.out,
                       p.out_f32, p.lse, p.lse_sb, p.lse_sg, p.lse_sh, p.G, p.H, p.Sq, p.Dv, diff ? 2 : 1, total);
    hipError_t e0 = hipGetLastError();
    if (e0 != hipSuccess) return fail(FL_ERR_LAUNCH, "empty-keys launch: %s", hipGetErrorString(e0));
    return FL_OK;
  }
  if (mask & FL_MASK_DOC) {
    const int nqs = (int)((Sq + fl::kSumBlock - 1) / fl::kSumBlock), nks = (int)((Sk + fl::kSumBlock - 1) / fl::kSumBlock);
    p.q_sum = (int2*)aux->workspace;
    p.kv_sum = p.q_sum + B * nqs;
    const int tq = (int)(B * nqs), tk = (int)(B * nks);
    launch_doc_summaries(aux->q_doc_ids, p.q_sum, (int)Sq, nqs, tq, aux->kv_doc_ids, p.kv_sum, (int)Sk, nks, tk, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FL_ERR_LAUNCH, "doc summary launch: %s", hipGetErrorString(e));
  }
  hipError_t e = ke->jit != nullptr ? fl::jit_forward_launch(*ke, p, (int)nblocks, stream) : ke->launch(p, (int)nblocks, stream);
  if (e != hipSuccess) return fail(FL_ERR_LAUNCH, "kernel launch: %s", hipGetErrorString(e));
  return FL_OK;
}

fl_status fl_attn_fwd(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_variant_desc* desc,
                      const fl_aux* aux, fl_tensor* out, fl_tensor* lse, void* stream_v) {
  return forward_call(q, k, v, desc, aux, out, lse, stream_v, nullptr);
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
static fl_status scratch_address(void** out) {
  static std::mutex mu;
  static void* ptrs[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= 64) return fail(FL_ERR_LAUNCH, "hipGetDevice: %s", hipGetErrorString(e));
  std::lock_guard<std::mutex> lock(mu);
  if (ptrs[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr)
      return fail(FL_ERR_LAUNCH, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    ptrs[dev] = ptr;
  }
  *out = ptrs[dev];
  return FL_OK;
}

fl_status fl_attn_fwd_noalloc(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_variant_desc* desc,
                              const fl_aux* aux, fl_tensor* out, fl_tensor* lse, void* stream_v) {
  g_detail[0] = 0;
  fl_status st = check_desc(desc);
  if (st != FL_OK) return st;
  if (q == nullptr || k == nullptr) return fail(FL_ERR_NULL, "q or k is NULL");
  const size_t need = workspace_bytes(q->size[0], q->size[3], k->size[3], canonical_mask(desc->mask));
  // variants without a workspace, and calls that fl_attn_fwd refuses for their aux block anyway
  if (need == 0 || aux == nullptr || aux->struct_size != sizeof(fl_aux))
    return fl_attn_fwd(q, k, v, desc, aux, out, lse, stream_v);
  if (q->size[0] < 0 || q->size[3] < 0 || k->size[3] < 0) return fail(FL_ERR_SHAPE, "negative size");
  if (need > kScratchBytes)
    return fail(FL_ERR_WORKSPACE,
                "the document-id summaries of this call need %zu bytes, the built-in scratch buffer holds %zu "
                "(B * (ceil(Sq / 32) + ceil(Sk / 32)) <= %zu); use fl_attn_fwd with a workspace",
                need, kScratchBytes, kScratchBytes / sizeof(int2));
  void* ptr = nullptr;
  if ((st = scratch_address(&ptr)) != FL_OK) return st;
  fl_aux a = *aux;
  a.workspace = ptr;
  a.workspace_bytes = kScratchBytes;
  return fl_attn_fwd(q, k, v, desc, &a, out, lse, stream_v);
}

size_t fl_attn_bwd_workspace_size(const fl_tensor* q, const fl_tensor* k, const fl_variant_desc* desc) {
  if (q == nullptr || k == nullptr || desc == nullptr) return 0;
  return bwd_workspace(q->size[0], q->size[1], q->size[2], k->size[2], q->size[3], k->size[3], q->size[4], canonical_mask(desc->mask),
                       clamp_window(desc->window, q->size[3], k->size[3])).total;
}

int fl_bwd_supported(const fl_variant_desc* desc, int dtype, int D, int Dv) {
  if (check_desc(desc) != FL_OK || dtype != FL_BF16) return 0;
  if (bwd_simple(desc, D, Dv)) return find_bwd_entry(desc, D) != nullptr || bwd_jit_ok(desc, D, 0) ? 1 : 0;
  return bwd_ex_ok(desc, D, Dv) ? 1 : 0;
}

}  // extern "C"

extern "C" {

fl_status fl_attn_bwd(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_tensor* out,
                      const fl_tensor* dout, const fl_tensor* lse, const fl_variant_desc* desc, const fl_aux* aux,
                      fl_tensor* dq, fl_tensor* dk, fl_tensor* dv, void* stream_v) {
  return fl::backward_call(q, k, v, out, dout, lse, desc, aux, dq, dk, dv, stream_v, nullptr, nullptr);
}

}  // extern "C"

fl_status fl::backward_call(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_tensor* out,
                            const fl_tensor* dout, const fl_tensor* lse, const fl_variant_desc* desc, const fl_aux* aux,
                            fl_tensor* dq, fl_tensor* dk, fl_tensor* dv, void* stream_v, const fl::BwdEntry* custom,
                            const void* const* user_aux) {
  g_detail[0] = 0;
  fl_status st = check_desc(desc);
  if (st != FL_OK) return st;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr || dout == nullptr || lse == nullptr ||
      dq == nullptr || dk == nullptr || dv == nullptr)
    return fail(FL_ERR_NULL, "a tensor descriptor is NULL");
  if (aux != nullptr && aux->struct_size != sizeof(fl_aux))
    return fail(FL_ERR_DESC, "aux->struct_size = %u, expected %zu", aux->struct_size, sizeof(fl_aux));
  if (q->dtype != FL_BF16) return fail(FL_ERR_DTYPE, "the backward pass takes bf16 inputs (q dtype %d)", q->dtype);
  if (custom == nullptr && !bwd_simple(desc, q->size[4], v->size[4]))   // biases, epilogues, second stream, other head dims: the composed pass
    return fl_attn_bwd_ex(q, k, v, out, dout, lse, desc, aux, dq, dk, dv, nullptr, stream_v);

  const int64_t B = q->size[0], G = q->size[1], H = q->size[2], Sq = q->size[3], D = q->size[4];
  const int64_t Hkv = k->size[2], Sk = k->size[3], Dv = v->size[4];
  if (B < 0 || G < 0 || H < 0 || Sq < 0 || Sk < 0 || D <= 0 || Dv <= 0) return fail(FL_ERR_SHAPE, "negative size");
  if (Sq > 0x7fffff00LL || Sk > 0x7fffff00LL || B * G * H > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "size too large");
  if (Hkv <= 0 || H % (Hkv > 0 ? Hkv : 1) != 0)
    if (H != 0) return fail(FL_ERR_SHAPE, "k heads (%lld) must divide q heads (%lld)", (long long)Hkv, (long long)H);
  const uint32_t mask = canonical_mask(desc->mask);
  const fl::BwdEntry* be = custom != nullptr ? custom : (D == Dv ? find_bwd_entry(desc, (int)D, 0, true) : nullptr);
  if (be == nullptr)
    return fail(FL_ERR_UNSUPPORTED, "no backward specialisation for D=%lld Dv=%lld score_mod=%u mask=0x%x", (long long)D,
                (long long)Dv, desc->score_mod, mask);
  const bool no_rows = (B == 0 || G == 0 || H == 0 || Sq == 0);       // dq is empty; dk, dv are all zero
  const bool no_keys = (B == 0 || G == 0 || H == 0 || Sk == 0);       // dk, dv are empty; dq is all zero

  const int64_t qsz[5] = {B, G, H, Sq, D}, ksz[5] = {B, G, Hkv, Sk, D}, osz[5] = {B, G, H, Sq, Dv};
  if (!no_rows) {
    if ((st = check_data_tensor(q, "q", FL_BF16, qsz)) != FL_OK) return st;
    if ((st = check_data_tensor(out, "out", FL_BF16, osz)) != FL_OK) return st;
    if ((st = check_data_tensor(dout, "dout", FL_BF16, osz)) != FL_OK) return st;
    if (dq->dtype != FL_BF16 && dq->dtype != FL_F32) return fail(FL_ERR_DTYPE, "dq dtype %d", dq->dtype);
    if ((st = check_data_tensor(dq, "dq", dq->dtype, qsz)) != FL_OK) return st;
    if (lse->ptr == nullptr) return fail(FL_ERR_NULL, "lse is NULL");
    if (lse->dtype != FL_F32) return fail(FL_ERR_DTYPE, "lse must be f32");
    const int64_t lsz[5] = {B, G, H, Sq, 1};
    for (int a = 0; a < 5; ++a)
      if (lse->size[a] != lsz[a])
        return fail(FL_ERR_SHAPE, "lse size[%d] = %lld, expected %lld", a, (long long)lse->size[a], (long long)lsz[a]);
    if (Sq > 1 && lse->stride[3] != 1) return fail(FL_ERR_STRIDE, "lse must be contiguous along Sq");
    for (int a = 0; a < 3; ++a)
      if (lse->stride[a] < 0) return fail(FL_ERR_STRIDE, "lse stride[%d] negative", a);
  }
  if (!no_keys) {
    if ((st = check_data_tensor(k, "k", FL_BF16, ksz)) != FL_OK) return st;
    if ((st = check_data_tensor(v, "v", FL_BF16, ksz)) != FL_OK) return st;
    if (dk->dtype != FL_BF16 && dk->dtype != FL_F32) return fail(FL_ERR_DTYPE, "dk dtype %d", dk->dtype);
    if (dv->dtype != dk->dtype) return fail(FL_ERR_DTYPE, "dk and dv must share one dtype");
    if ((st = check_data_tensor(dk, "dk", dk->dtype, ksz)) != FL_OK) return st;
    if ((st = check_data_tensor(dv, "dv", dv->dtype, ksz)) != FL_OK) return st;
  }
  const bool need_aux = desc->score_mod == FL_MOD_ALIBI || (mask & FL_MASK_DOC) || !(no_rows && no_keys);
  if (need_aux && aux == nullptr) return fail(FL_ERR_AUX_MISSING, "the backward pass needs aux (workspace)");
  if (desc->score_mod == FL_MOD_ALIBI && aux->alibi_slopes == nullptr) return fail(FL_ERR_AUX_MISSING, "alibi_slopes");
  if ((mask & FL_MASK_DOC) && (aux->q_doc_ids == nullptr || aux->kv_doc_ids == nullptr))
    return fail(FL_ERR_AUX_MISSING, "q_doc_ids / kv_doc_ids");
  if (no_rows && no_keys) return FL_OK;
  const BwdWorkspace wsz = bwd_workspace(B, G, H, Hkv, Sq, Sk, D, mask, clamp_window(desc->window, Sq, Sk));
  if (aux->workspace == nullptr || aux->workspace_bytes < wsz.total)
    return fail(FL_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", wsz.total, aux->workspace ? aux->workspace_bytes : (size_t)0);
  if (((uintptr_t)aux->workspace) % 16 != 0) return fail(FL_ERR_ALIGN, "workspace not 16-byte aligned");

  fl::BwdParams p;
  memset(&p, 0, sizeof(p));
  if (!no_rows) {
    p.q = make_view(q);
    p.o = make_view(out);
    p.dout = make_view(dout);
    p.dq = make_view(dq);
    p.lse = (const float*)lse->ptr;
    p.lse_sb = lse->size[0] > 1 ? lse->stride[0] : 0;
    p.lse_sg = lse->size[1] > 1 ? lse->stride[1] : 0;
    p.lse_sh = lse->size[2] > 1 ? lse->stride[2] : 0;
  }
  if (!no_keys) {
    p.k = make_view(k);
    p.v = make_view(v);
    p.dk = make_view(dk);
    p.dv = make_view(dv);
  }
  p.delta = (float*)aux->workspace;
  p.lse2 = (float*)((unsigned char*)aux->workspace + wsz.stat_bytes);
  p.alibi_slopes = aux->alibi_slopes;
  p.q_doc = aux->q_doc_ids;
  p.kv_doc = aux->kv_doc_ids;
  p.B = (int)B; p.G = (int)G; p.H = (int)H; p.Hkv = (int)Hkv; p.Sq = (int)Sq; p.Sk = (int)Sk;
  p.window = clamp_window(desc->window, Sq + desc->q_offset, Sk);
  p.prefix = desc->prefix_len;
  p.q_off = desc->q_offset;
  for (int n = 0; n < 4; ++n) p.user_aux[n] = user_aux != nullptr ? user_aux[n] : nullptr;
  p.scale = desc->scale;
  p.softcap = desc->softcap;
  p.dq_f32 = dq->dtype == FL_F32;
  p.dkv_f32 = dk->dtype == FL_F32;
  p.n_qtiles = (int)((Sq + be->bm - 1) / be->bm);
  p.n_ktiles = (int)((Sk + be->bm - 1) / be->bm);
  static_assert(fl::BwdCfg<64, 0, 0, 64, 2>::BM == kBwdKeysPerWg, "keys per dK/dV workgroup");
  p.hsplit = no_keys || no_rows ? 1 : wsz.hsplit;
  p.part_dk = (float*)((unsigned char*)aux->workspace + 2 * wsz.stat_bytes + wsz.sum_bytes);
  p.part_dv = (float*)((unsigned char*)p.part_dk + wsz.part_bytes);
  const int order = g_tuning.order >= 0 ? g_tuning.order : 1;
  p.order_q = order == 1 && (B * G * H) % 8 == 0;
  p.order_k = order == 1 && (B * G * Hkv * p.hsplit) % 8 == 0;
  const int64_t nb_q = B * G * H * p.n_qtiles, nb_k = B * G * Hkv * p.hsplit * p.n_ktiles;
  const int64_t rows = B * G * H * Sq;
  if (nb_q > 0x7fffffffLL || nb_k > 0x7fffffffLL || rows > 0x7fffffff00LL) return fail(FL_ERR_SHAPE, "too many workgroups");

  hipStream_t stream = (hipStream_t)stream_v;
  hipError_t e = hipSuccess;
  if ((mask & FL_MASK_DOC) && !no_rows && !no_keys) {
    const int nqs = (int)((Sq + fl::kSumBlock - 1) / fl::kSumBlock), nks = (int)((Sk + fl::kSumBlock - 1) / fl::kSumBlock);
    p.q_sum = (int2*)((unsigned char*)aux->workspace + 2 * wsz.stat_bytes);
    p.kv_sum = p.q_sum + B * nqs;
    const int tq = (int)(B * nqs), tk = (int)(B * nks);
    launch_doc_summaries(aux->q_doc_ids, p.q_sum, (int)Sq, nqs, tq, aux->kv_doc_ids, p.kv_sum, (int)Sk, nks, tk, stream);
    if ((e = hipGetLastError()) != hipSuccess) return fail(FL_ERR_LAUNCH, "doc summary launch: %s", hipGetErrorString(e));
  }
  if (!no_rows) {
    const int lanes_per_row = (int)Dv / 8;
    const int64_t nb_prep = (rows * lanes_per_row + 255) / 256;
    if ((e = be->prep(p, (int)nb_prep, stream)) != hipSuccess) return fail(FL_ERR_LAUNCH, "pre-pass launch: %s", hipGetErrorString(e));
    // Sk == 0: the key loop is empty and dq comes out as zeros
    if ((e = run_bwd_dq(be, p, (int)nb_q, stream)) != hipSuccess) return fail(FL_ERR_LAUNCH, "dq launch: %s", hipGetErrorString(e));
  }
  if (!no_keys) {
    // Sq == 0: the query loop is empty and dk, dv come out as zeros
    if ((e = run_bwd_dkdv(be, p, (int)nb_k, stream)) != hipSuccess) return fail(FL_ERR_LAUNCH, "dk/dv launch: %s", hipGetErrorString(e));
    if (p.hsplit > 1) {
      const int64_t chunks = B * G * Hkv * Sk * (D / 4);
      if ((e = be->reduce(p, (int)((chunks + 255) / 256), stream)) != hipSuccess)
        return fail(FL_ERR_LAUNCH, "dk/dv reduction launch: %s", hipGetErrorString(e));
    }
  }
  return FL_OK;
}

extern "C" {

size_t fl_attn_bwd_ex_workspace_size(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_variant_desc* desc) {
  if (q == nullptr || k == nullptr || v == nullptr || desc == nullptr) return 0;
  if (bwd_simple(desc, q->size[4], v->size[4])) return fl_attn_bwd_workspace_size(q, k, desc);
  return ex_layout(q->size[0], q->size[1], q->size[2], k->size[2], q->size[3], k->size[3], q->size[4], v->size[4], desc).total;
}

fl_status fl_attn_bwd_ex(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_tensor* out, const fl_tensor* dout,
                         const fl_tensor* lse, const fl_variant_desc* desc, const fl_aux* aux, fl_tensor* dq, fl_tensor* dk,
                         fl_tensor* dv, const fl_bwd_extra* extra, void* stream_v) {
  g_detail[0] = 0;
  fl_status st = check_desc(desc);
  if (st != FL_OK) return st;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr || dout == nullptr || lse == nullptr || dq == nullptr ||
      dk == nullptr || dv == nullptr)
    return fail(FL_ERR_NULL, "a tensor descriptor is NULL");
  if (extra != nullptr && extra->struct_size != sizeof(fl_bwd_extra))
    return fail(FL_ERR_DESC, "extra->struct_size = %u, expected %zu", extra->struct_size, sizeof(fl_bwd_extra));
  if (aux != nullptr && aux->struct_size != sizeof(fl_aux))
    return fail(FL_ERR_DESC, "aux->struct_size = %u, expected %zu", aux->struct_size, sizeof(fl_aux));
  if (q->dtype != FL_BF16) return fail(FL_ERR_DTYPE, "the backward pass takes bf16 inputs (q dtype %d)", q->dtype);
  const int64_t B = q->size[0], G = q->size[1], H = q->size[2], Sq = q->size[3], D = q->size[4];
  const int64_t Hkv = k->size[2], Sk = k->size[3], Dv = v->size[4];
  if (bwd_simple(desc, D, Dv)) return fl_attn_bwd(q, k, v, out, dout, lse, desc, aux, dq, dk, dv, stream_v);
  if (B <= 0 || G <= 0 || H <= 0 || Sq <= 0 || Sk <= 0 || Hkv <= 0 || H % Hkv != 0)
    return fail(FL_ERR_SHAPE, "the composed backward pass needs non-empty tensors and kv heads that divide the q heads");
  if (Sq > 0x7fffff00LL || Sk > 0x7fffff00LL || B * G * H > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "size too large");
  if (!bwd_ex_ok(desc, D, Dv))
    return fail(FL_ERR_UNSUPPORTED, "no backward kernels for D=%lld Dv=%lld score_mod=%u mask=0x%x n_bias=%u q_offset=%d",
                (long long)D, (long long)Dv, desc->score_mod, canonical_mask(desc->mask), desc->n_bias, desc->q_offset);
  if (aux == nullptr) return fail(FL_ERR_AUX_MISSING, "the backward pass needs aux (workspace)");
  const uint32_t mask = canonical_mask(desc->mask);
  const bool diff = desc->combine == FL_DIFFERENTIAL;
  const bool has_gate = (desc->epilogue & FL_EPI_GATE_SIGMOID) != 0, has_rms = (desc->epilogue & FL_EPI_RMSNORM) != 0;
  const ExLayout L = ex_layout(B, G, H, Hkv, Sq, Sk, D, Dv, desc);
  const int Dc = L.Dc, ns = L.ns;
  const fl::BwdEntry* be = find_bwd_entry(desc, Dc, (int)desc->n_bias, true);

  // ---- tensors
  const int64_t qsz[5] = {B, G, H, Sq, D}, ksz[5] = {B, G, Hkv, Sk, D}, vsz[5] = {B, G, Hkv, Sk, Dv}, osz[5] = {B, G, H, Sq, Dv};
  if ((st = check_data_tensor(q, "q", FL_BF16, qsz)) != FL_OK) return st;
  if ((st = check_data_tensor(k, "k", FL_BF16, ksz)) != FL_OK) return st;
  if ((st = check_data_tensor(v, "v", FL_BF16, vsz)) != FL_OK) return st;
  if ((st = check_data_tensor(out, "out", FL_BF16, osz)) != FL_OK) return st;
  if ((st = check_data_tensor(dout, "dout", FL_BF16, osz)) != FL_OK) return st;
  if (dq->dtype != FL_BF16 && dq->dtype != FL_F32) return fail(FL_ERR_DTYPE, "dq dtype %d", dq->dtype);
  if (dk->dtype != FL_BF16 && dk->dtype != FL_F32) return fail(FL_ERR_DTYPE, "dk dtype %d", dk->dtype);
  if (dv->dtype != dk->dtype) return fail(FL_ERR_DTYPE, "dk and dv must share one dtype");
  if ((st = check_data_tensor(dq, "dq", dq->dtype, qsz)) != FL_OK) return st;
  if ((st = check_data_tensor(dk, "dk", dk->dtype, ksz)) != FL_OK) return st;
  if ((st = check_data_tensor(dv, "dv", dv->dtype, vsz)) != FL_OK) return st;
  if (lse->ptr == nullptr) return fail(FL_ERR_NULL, "lse is NULL");
  if (lse->dtype != FL_F32) return fail(FL_ERR_DTYPE, "lse must be f32");
  const int64_t lsz[5] = {B, ns * G, H, Sq, 1};
  for (int a = 0; a < 5; ++a)
    if (lse->size[a] != lsz[a])
      return fail(FL_ERR_SHAPE, "lse size[%d] = %lld, expected %lld", a, (long long)lse->size[a], (long long)lsz[a]);
  if (Sq > 1 && lse->stride[3] != 1) return fail(FL_ERR_STRIDE, "lse must be contiguous along Sq");
  if (desc->score_mod == FL_MOD_ALIBI && aux->alibi_slopes == nullptr) return fail(FL_ERR_AUX_MISSING, "alibi_slopes");
  if ((mask & FL_MASK_DOC) && (aux->q_doc_ids == nullptr || aux->kv_doc_ids == nullptr))
    return fail(FL_ERR_AUX_MISSING, "q_doc_ids / kv_doc_ids");
  if (diff) {
    if (aux->lambda == nullptr) return fail(FL_ERR_AUX_MISSING, "lambda");
    if ((st = check_data_tensor(&aux->q2, "q2", FL_BF16, qsz)) != FL_OK) return st == FL_ERR_NULL ? fail(FL_ERR_AUX_MISSING, "q2") : st;
    if ((st = check_data_tensor(&aux->k2, "k2", FL_BF16, ksz)) != FL_OK) return st == FL_ERR_NULL ? fail(FL_ERR_AUX_MISSING, "k2") : st;
    if (extra == nullptr) return fail(FL_ERR_AUX_MISSING, "the differential variant writes dq2 and dk2 (extra is NULL)");
    if ((st = check_data_tensor(&extra->dq2, "dq2", dq->dtype, qsz)) != FL_OK) return st;
    if ((st = check_data_tensor(&extra->dk2, "dk2", dk->dtype, ksz)) != FL_OK) return st;
  }
  if (has_gate) {
    if ((st = check_data_tensor(&aux->gate, "gate", FL_BF16, osz)) != FL_OK) return st == FL_ERR_NULL ? fail(FL_ERR_AUX_MISSING, "gate") : st;
    if (extra != nullptr && extra->dgate.ptr != nullptr) {
      if (extra->dgate.dtype != FL_BF16 && extra->dgate.dtype != FL_F32) return fail(FL_ERR_DTYPE, "dgate dtype %d", extra->dgate.dtype);
      if ((st = check_data_tensor(&extra->dgate, "dgate", extra->dgate.dtype, osz)) != FL_OK) return st;
    }
  }
  // biases and their gradients
  fl::BiasView bias[2], dbias[2];
  memset(bias, 0, sizeof(bias));
  memset(dbias, 0, sizeof(dbias));
  const int64_t bwant[5] = {B, G, H, Sq, Sk};
  for (uint32_t nb = 0; nb < desc->n_bias; ++nb) {
    const fl_tensor* bt = &aux->bias[nb];
    if (bt->ptr == nullptr) return fail(FL_ERR_AUX_MISSING, "bias[%u]", nb);
    if (bt->dtype != FL_BF16) return fail(FL_ERR_DTYPE, "bias[%u]: bf16 inputs take bf16 biases", nb);
    int64_t bs[5];
    for (int a = 0; a < 5; ++a) {
      if (bt->size[a] != bwant[a] && bt->size[a] != 1)
        return fail(FL_ERR_SHAPE, "bias[%u] size[%d] = %lld, expected %lld or 1", nb, a, (long long)bt->size[a], (long long)bwant[a]);
      bs[a] = (bt->size[a] == 1 && bwant[a] != 1) ? 0 : bt->stride[a];
      if (bs[a] < 0) return fail(FL_ERR_STRIDE, "bias[%u] stride[%d] negative", nb, a);
    }
    bias[nb].ptr = bt->ptr;
    bias[nb].sb = bs[0]; bias[nb].sg = bs[1]; bias[nb].sh = bs[2]; bias[nb].si = bs[3]; bias[nb].sj = bs[4];
    const fl_tensor* gt = extra != nullptr ? &extra->dbias[nb] : nullptr;
    if (gt != nullptr && gt->ptr != nullptr) {
      if (gt->dtype != FL_F32) return fail(FL_ERR_DTYPE, "dbias[%u] must be f32", nb);
      if (((uintptr_t)gt->ptr) % 4 != 0) return fail(FL_ERR_ALIGN, "dbias[%u] not 4-byte aligned", nb);
      int64_t gs[5];
      for (int a = 0; a < 5; ++a) {
        if (gt->size[a] != bt->size[a])
          return fail(FL_ERR_SHAPE, "dbias[%u] size[%d] = %lld, the bias has %lld", nb, a, (long long)gt->size[a], (long long)bt->size[a]);
        gs[a] = (gt->size[a] == 1 && bwant[a] != 1) ? 0 : gt->stride[a];
        if (gs[a] < 0 || (gt->size[a] > 1 && gs[a] == 0)) return fail(FL_ERR_STRIDE, "dbias[%u] stride[%d]", nb, a);
      }
      dbias[nb].ptr = gt->ptr;
      dbias[nb].sb = gs[0]; dbias[nb].sg = gs[1]; dbias[nb].sh = gs[2]; dbias[nb].si = gs[3]; dbias[nb].sj = gs[4];
    }
  }
  if (aux->workspace == nullptr || aux->workspace_bytes < L.total)
    return fail(FL_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", L.total, aux->workspace ? aux->workspace_bytes : (size_t)0);
  if (((uintptr_t)aux->workspace) % 16 != 0) return fail(FL_ERR_ALIGN, "workspace not 16-byte aligned");
  const int64_t rows_q = B * G * H * Sq, rows_k = B * G * Hkv * Sk;
  if (rows_q * Dc > 0x7fffffff00LL || rows_k * Dc > 0x7fffffff00LL) return fail(FL_ERR_SHAPE, "too many rows");

  hipStream_t stream = (hipStream_t)stream_v;
  unsigned char* ws = (unsigned char*)aux->workspace;
  hipError_t e = hipSuccess;
  auto blocks = [](int64_t n) { return dim3((unsigned)((n + 255) / 256)); };
  const fl_tensor* qs[2] = {q, diff ? &aux->q2 : nullptr};
  const fl_tensor* ks[2] = {k, diff ? &aux->k2 : nullptr};

  // ---- 1. the streams' outputs, recomputed by the forward kernel without epilogue (fp32, dense)
  if (L.need_o) {
    fl_variant_desc d1 = *desc;
    d1.combine = FL_SINGLE;
    d1.epilogue = 0;
    fl_aux a1 = *aux;
    a1.workspace = ws + L.off_sum;
    a1.workspace_bytes = L.sum;
    for (int s = 0; s < ns; ++s) {
      fl_tensor to;
      memset(&to, 0, sizeof(to));
      to.ptr = ws + L.off_o[s];
      to.dtype = FL_F32;
      const int64_t dsz[5] = {B, G, H, Sq, Dv};
      int64_t stv = 1;
      for (int a = 4; a >= 0; --a) {
        to.size[a] = dsz[a];
        to.stride[a] = stv;
        stv *= dsz[a];
      }
      if ((st = fl_attn_fwd(qs[s], ks[s], v, &d1, &a1, &to, nullptr, stream_v)) != FL_OK) return st;
    }
  }

  // ---- 2. epilogue derivative: per-stream dO, delta, lse2; gate and lambda gradients
  EpiBwdParams ep;
  memset(&ep, 0, sizeof(ep));
  ep.dout = make_view(dout);
  ep.out = make_view(out);
  if (has_gate) {
    ep.gate = make_view(&aux->gate);
    if (extra != nullptr && extra->dgate.ptr != nullptr) {
      ep.dgate = make_view(&extra->dgate);
      ep.dgate_f32 = extra->dgate.dtype == FL_F32;
    }
  }
  ep.lse = (const float*)lse->ptr;
  ep.lse_sb = lse->size[0] > 1 ? lse->stride[0] : 0;
  ep.lse_sg = lse->size[1] > 1 ? lse->stride[1] : 0;
  ep.lse_sh = lse->size[2] > 1 ? lse->stride[2] : 0;
  for (int s = 0; s < ns; ++s) {
    ep.o[s] = L.need_o ? (const float*)(ws + L.off_o[s]) : nullptr;
    ep.d_o[s] = (uint16_t*)(ws + L.off_do[s]);
    ep.delta[s] = (float*)(ws + L.off_delta[s]);
    ep.lse2[s] = (float*)(ws + L.off_lse2[s]);
  }
  ep.lambda = aux->lambda;
  ep.rms_w = aux->rms_weight;
  ep.dl_rows = diff && extra->dlambda != nullptr ? (float*)(ws + L.off_dl) : nullptr;
  ep.dw_part = has_rms && extra != nullptr && extra->drms_weight != nullptr ? (float*)(ws + L.off_dw) : nullptr;
  ep.rms_eps = desc->rms_eps;
  ep.B = (int)B; ep.G = (int)G; ep.H = (int)H; ep.Sq = (int)Sq; ep.Dv = (int)Dv; ep.Dc = Dc;
  ep.ns = ns; ep.has_gate = has_gate; ep.has_rms = has_rms;
  // rows 16-byte aligned everywhere: several rows per wave, eight channels per lane; else one row per wave
  auto rows_aligned = [](const fl::View& v, int elem_bytes) {
    if (v.ptr == nullptr) return true;
    const int64_t m = 16 / elem_bytes;
    return ((uintptr_t)v.ptr) % 16 == 0 && v.sb % m == 0 && v.sg % m == 0 && v.sh % m == 0 && v.ss % m == 0;
  };
  const bool by_rows = rows_aligned(ep.dout, 2) && rows_aligned(ep.out, 2) && rows_aligned(ep.gate, 2) &&
                       rows_aligned(ep.dgate, ep.dgate_f32 ? 4 : 2) && ((uintptr_t)ep.rms_w) % 16 == 0;
  const int rows_per_wg = by_rows ? 4 * (64 / (Dc / 8)) : 4;
  const int64_t epi_wgs = (rows_q + rows_per_wg - 1) / rows_per_wg;
  if (epi_wgs > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "too many rows");
  if (!by_rows) hipLaunchKernelGGL(epi_bwd_kernel, dim3((unsigned)epi_wgs), dim3(256), 0, stream, ep);
  else if (Dc == 64) hipLaunchKernelGGL(epi_bwd_rows_kernel<8>, dim3((unsigned)epi_wgs), dim3(256), 0, stream, ep);
  else hipLaunchKernelGGL(epi_bwd_rows_kernel<16>, dim3((unsigned)epi_wgs), dim3(256), 0, stream, ep);
  if (ep.dw_part != nullptr)
    hipLaunchKernelGGL(reduce_drms_kernel, dim3((unsigned)Dv), dim3(256), 0, stream, (const float*)ep.dw_part, extra->drms_weight,
                       epi_wgs, (int)Dv);
  if (ep.dl_rows != nullptr)
    hipLaunchKernelGGL(reduce_dlambda_kernel, dim3((unsigned)H), dim3(256), 0, stream, (const float*)ep.dl_rows, extra->dlambda, (int)B, (int)G,
                       (int)H, (int)Sq);

  // ---- 3. zero-padded copies for head dims below the kernels' own
  for (int s = 0; s < ns && L.pad_qk; ++s) {
    hipLaunchKernelGGL(pad_rows_kernel, blocks(rows_q * (Dc / 8)), dim3(256), 0, stream, make_view(qs[s]), (uint16_t*)(ws + L.off_qpad[s]),
                       (int)G, (int)H, (int)Sq, (int)D, Dc, rows_q);
    hipLaunchKernelGGL(pad_rows_kernel, blocks(rows_k * (Dc / 8)), dim3(256), 0, stream, make_view(ks[s]), (uint16_t*)(ws + L.off_kpad[s]),
                       (int)G, (int)Hkv, (int)Sk, (int)D, Dc, rows_k);
  }
  if (L.pad_v)
    hipLaunchKernelGGL(pad_rows_kernel, blocks(rows_k * (Dc / 8)), dim3(256), 0, stream, make_view(v), (uint16_t*)(ws + L.off_vpad), (int)G,
                       (int)Hkv, (int)Sk, (int)Dv, Dc, rows_k);
  const bool want_dbias = dbias[0].ptr != nullptr || dbias[1].ptr != nullptr;
  // under a mask whole blocks are skipped by the dQ kernel: their dS is zero
  if (want_dbias && mask != 0)
    hipLaunchKernelGGL(zero_f32_kernel, blocks((int64_t)(L.ds / 4)), dim3(256), 0, stream, (float*)(ws + L.off_ds), (int64_t)(L.ds / 4));
  if ((e = hipGetLastError()) != hipSuccess) return fail(FL_ERR_LAUNCH, "backward pre-pass launch: %s", hipGetErrorString(e));

  // ---- 4. the backward kernels, once per stream, into dense fp32 gradient buffers
  fl::BwdParams p;
  memset(&p, 0, sizeof(p));
  p.alibi_slopes = aux->alibi_slopes;
  p.q_doc = aux->q_doc_ids;
  p.kv_doc = aux->kv_doc_ids;
  p.B = (int)B; p.G = (int)G; p.H = (int)H; p.Hkv = (int)Hkv; p.Sq = (int)Sq; p.Sk = (int)Sk;
  p.window = clamp_window(desc->window, Sq + desc->q_offset, Sk);
  p.prefix = desc->prefix_len;
  p.q_off = desc->q_offset;
  p.scale = desc->scale;
  p.softcap = desc->softcap;
  p.dq_f32 = 1;
  p.dkv_f32 = 1;
  p.n_qtiles = (int)((Sq + be->bm - 1) / be->bm);
  p.n_ktiles = (int)((Sk + be->bm - 1) / be->bm);
  p.hsplit = L.hsplit;
  p.part_dk = (float*)(ws + L.off_part);
  p.part_dv = (float*)(ws + L.off_part + L.part);
  const int order = g_tuning.order >= 0 ? g_tuning.order : 1;
  p.order_q = order == 1 && (B * G * H) % 8 == 0;
  p.order_k = order == 1 && (B * G * Hkv * p.hsplit) % 8 == 0;
  for (int nb = 0; nb < 2; ++nb) p.bias[nb] = bias[nb];
  p.ds_stage = want_dbias ? (uint16_t*)(ws + L.off_ds) : nullptr;
  const int64_t nb_q = B * G * H * p.n_qtiles, nb_k = B * G * Hkv * p.hsplit * p.n_ktiles;
  if (nb_q > 0x7fffffffLL || nb_k > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "too many workgroups");
  if (mask & FL_MASK_DOC) {
    const int nqs = (int)((Sq + fl::kSumBlock - 1) / fl::kSumBlock), nks = (int)((Sk + fl::kSumBlock - 1) / fl::kSumBlock);
    p.q_sum = (int2*)(ws + L.off_sum);
    p.kv_sum = p.q_sum + B * nqs;
    const int tq = (int)(B * nqs), tk = (int)(B * nks);
    launch_doc_summaries(aux->q_doc_ids, p.q_sum, (int)Sq, nqs, tq, aux->kv_doc_ids, p.kv_sum, (int)Sk, nks, tk, stream);
    if ((e = hipGetLastError()) != hipSuccess) return fail(FL_ERR_LAUNCH, "doc summary launch: %s", hipGetErrorString(e));
  }
  const fl::View vview = L.pad_v ? dense_view(ws + L.off_vpad, G, Hkv, Sk, Dc) : make_view(v);
  for (int s = 0; s < ns; ++s) {
    p.q = L.pad_qk ? dense_view(ws + L.off_qpad[s], G, H, Sq, Dc) : make_view(qs[s]);
    p.k = L.pad_qk ? dense_view(ws + L.off_kpad[s], G, Hkv, Sk, Dc) : make_view(ks[s]);
    p.v = vview;
    p.dout = dense_view(ws + L.off_do[s], G, H, Sq, Dc);
    p.dq = dense_view(ws + L.off_gq[s], G, H, Sq, Dc);
    p.dk = dense_view(ws + L.off_gk[s], G, Hkv, Sk, Dc);
    p.dv = dense_view(ws + L.off_gv[s], G, Hkv, Sk, Dc);
    p.delta = (float*)(ws + L.off_delta[s]);
    p.lse2 = (float*)(ws + L.off_lse2[s]);
    if ((e = run_bwd_dq(be, p, (int)nb_q, stream)) != hipSuccess) return fail(FL_ERR_LAUNCH, "dq launch: %s", hipGetErrorString(e));
    for (uint32_t nb = 0; nb < desc->n_bias; ++nb)
      if (dbias[nb].ptr != nullptr) {               // this stream's dS, summed over the axes the bias broadcasts along
        const fl_tensor* gt = &extra->dbias[nb];
        const int64_t total = gt->size[0] * gt->size[1] * gt->size[2] * gt->size[3] * gt->size[4];
        const fl::BiasView& bv = dbias[nb];
        const bool vec8 = gt->size[4] == Sk && Sk % 8 == 0 && bv.sj == 1 && ((uintptr_t)bv.ptr) % 16 == 0 && bv.sb % 4 == 0 &&
                          bv.sg % 4 == 0 && bv.sh % 4 == 0 && bv.si % 4 == 0;
        if (vec8)
          hipLaunchKernelGGL(reduce_dbias_vec8_kernel, blocks(total / 8), dim3(256), 0, stream, (const uint16_t*)p.ds_stage, bv, (int)B,
                             (int)G, (int)H, (int)Sq, (int)Sk, (int)gt->size[0], (int)gt->size[1], (int)gt->size[2], (int)gt->size[3],
                             total / 8, s);
        else
          hipLaunchKernelGGL(reduce_dbias_kernel, blocks(total), dim3(256), 0, stream, (const uint16_t*)p.ds_stage, bv, (int)B, (int)G,
                             (int)H, (int)Sq, (int)Sk, (int)gt->size[0], (int)gt->size[1], (int)gt->size[2], (int)gt->size[3],
                             (int)gt->size[4], total, s);
      }
    if ((e = run_bwd_dkdv(be, p, (int)nb_k, stream)) != hipSuccess) return fail(FL_ERR_LAUNCH, "dk/dv launch: %s", hipGetErrorString(e));
    if (p.hsplit > 1) {
      const int64_t chunks = rows_k * (Dc / 4);
      if ((e = be->reduce(p, (int)((chunks + 255) / 256), stream)) != hipSuccess)
        return fail(FL_ERR_LAUNCH, "dk/dv reduction launch: %s", hipGetErrorString(e));
    }
  }

  // ---- 5. into the caller's tensors: first D (Dv) channels, dv summed over the streams
  fl_tensor* dqs[2] = {dq, diff ? (fl_tensor*)&extra->dq2 : nullptr};
  fl_tensor* dks[2] = {dk, diff ? (fl_tensor*)&extra->dk2 : nullptr};
  for (int s = 0; s < ns; ++s) {
    hipLaunchKernelGGL(scatter_grad_kernel, blocks(rows_q * (D / 4)), dim3(256), 0, stream, (const float*)(ws + L.off_gq[s]),
                       (const float*)nullptr, make_view(dqs[s]), (int)(dqs[s]->dtype == FL_F32), (int)G, (int)H, (int)Sq, (int)D, Dc, rows_q);
    hipLaunchKernelGGL(scatter_grad_kernel, blocks(rows_k * (D / 4)), dim3(256), 0, stream, (const float*)(ws + L.off_gk[s]),
                       (const float*)nullptr, make_view(dks[s]), (int)(dks[s]->dtype == FL_F32), (int)G, (int)Hkv, (int)Sk, (int)D, Dc, rows_k);
  }
  hipLaunchKernelGGL(scatter_grad_kernel, blocks(rows_k * (Dv / 4)), dim3(256), 0, stream, (const float*)(ws + L.off_gv[0]),
                     ns == 2 ? (const float*)(ws + L.off_gv[1]) : (const float*)nullptr, make_view(dv), (int)(dv->dtype == FL_F32), (int)G,
                     (int)Hkv, (int)Sk, (int)Dv, Dc, rows_k);
  if ((e = hipGetLastError()) != hipSuccess) return fail(FL_ERR_LAUNCH, "gradient scatter launch: %s", hipGetErrorString(e));
  return FL_OK;
}

size_t fl_attn_decode_workspace_size(const fl_tensor* q, const fl_tensor* k_cache, const fl_paged_kv* kv) {
  if (q == nullptr || k_cache == nullptr || kv == nullptr) return 0;
  const int64_t B = q->size[0], H = q->size[2], T = q->size[3], D = q->size[4];
  const int ns = decode_splits(B, k_cache->size[2], D, kv->max_seq_len);
  return (size_t)(B * T * H * ns) * (size_t)(D + 2) * sizeof(float);
}

fl_status fl_attn_decode(const fl_tensor* q, const fl_tensor* k_cache, const fl_tensor* v_cache, const fl_paged_kv* kv,
                         const fl_variant_desc* desc, const fl_aux* aux, fl_tensor* out, fl_tensor* lse, void* stream_v) {
  g_detail[0] = 0;
  fl_status st = check_desc(desc);
  if (st != FL_OK) return st;
  if (q == nullptr || k_cache == nullptr || v_cache == nullptr || kv == nullptr || out == nullptr)
    return fail(FL_ERR_NULL, "q, k_cache, v_cache, kv or out is NULL");
  if (kv->struct_size != sizeof(fl_paged_kv))
    return fail(FL_ERR_DESC, "kv->struct_size = %u, expected %zu", kv->struct_size, sizeof(fl_paged_kv));
  if (aux != nullptr && aux->struct_size != sizeof(fl_aux))
    return fail(FL_ERR_DESC, "aux->struct_size = %u, expected %zu", aux->struct_size, sizeof(fl_aux));
  const uint32_t mask = canonical_mask(desc->mask);
  if ((mask & (FL_MASK_DOC | FL_MASK_PREFIX)) || desc->n_bias != 0 || desc->combine != FL_SINGLE || desc->epilogue != 0 ||
      desc->q_offset != 0)
    return fail(FL_ERR_UNSUPPORTED, "the decode step covers scale, score_mod and the sliding window only");
  if (q->dtype != FL_BF16) return fail(FL_ERR_DTYPE, "the decode step takes bf16 inputs (q dtype %d)", q->dtype);

  const int64_t B = q->size[0], H = q->size[2], T = q->size[3], D = q->size[4];
  const int64_t pages = k_cache->size[0], Hkv = k_cache->size[2], page_size = k_cache->size[3];
  if (B < 0 || H < 0 || T < 0 || D <= 0 || pages < 0 || page_size <= 0) return fail(FL_ERR_SHAPE, "negative size");
  if (pages > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "more pages than an int32 table entry can name");
  if (pages == 0 && kv->max_seq_len > 0) return fail(FL_ERR_SHAPE, "max_seq_len = %d with an empty cache", kv->max_seq_len);
  if (q->size[1] != 1) return fail(FL_ERR_SHAPE, "q must be [B, 1, H, T, D]");
  if (Hkv <= 0 || H % Hkv != 0 || (H / Hkv) * T > kDecodeMaxPairs)
    if (H != 0)
      return fail(FL_ERR_SHAPE, "kv heads (%lld) must divide q heads (%lld), at most %lld (query row, q head) pairs per kv head (T = %lld)",
                  (long long)Hkv, (long long)H, (long long)kDecodeMaxPairs, (long long)T);
  if (kv->page_size != page_size) return fail(FL_ERR_SHAPE, "kv->page_size = %d, cache size[3] = %lld", kv->page_size, (long long)page_size);
  if (kv->max_seq_len < 0) return fail(FL_ERR_SHAPE, "max_seq_len negative");
  int page_shift = 0;
  if (kv->block_table != nullptr) {
    if (page_size < 8 || (page_size & (page_size - 1)) != 0)
      return fail(FL_ERR_SHAPE, "with a block table the page size (%lld) must be a power of two >= 8", (long long)page_size);
    while ((1LL << page_shift) < page_size) ++page_shift;
    if (kv->table_stride < (kv->max_seq_len + page_size - 1) / page_size)
      return fail(FL_ERR_SHAPE, "table_stride %d is less than the pages of max_seq_len", kv->table_stride);
  } else {
    if (pages < B) return fail(FL_ERR_SHAPE, "without a block table the cache needs a page per sequence");
    if (kv->max_seq_len > page_size) return fail(FL_ERR_SHAPE, "max_seq_len exceeds the page size");
  }
  const fl::DecodeEntry* de = find_decode_entry((int)D, (int)desc->score_mod, H > 0 && (H / Hkv) * T > 32 ? 2 : 1);
  if (de == nullptr || v_cache->size[4] != D)
    return fail(FL_ERR_UNSUPPORTED, "no decode specialisation for D=%lld Dv=%lld score_mod=%u", (long long)D,
                (long long)v_cache->size[4], desc->score_mod);
  const bool empty = (B == 0 || H == 0 || T == 0);
  const int64_t qsz[5] = {B, 1, H, T, D}, csz[5] = {pages, 1, Hkv, page_size, D};
  if (!empty) {
    if ((st = check_data_tensor(q, "q", FL_BF16, qsz)) != FL_OK) return st;
    if (kv->max_seq_len > 0) {
      if ((st = check_data_tensor(k_cache, "k_cache", FL_BF16, csz)) != FL_OK) return st;
      if ((st = check_data_tensor(v_cache, "v_cache", FL_BF16, csz)) != FL_OK) return st;
    }
    if (out->dtype != FL_BF16 && out->dtype != FL_F32) return fail(FL_ERR_DTYPE, "out dtype %d", out->dtype);
    if ((st = check_data_tensor(out, "out", out->dtype, qsz)) != FL_OK) return st;
    if (kv->seq_lens == nullptr) return fail(FL_ERR_NULL, "seq_lens is NULL");
  }
  const bool want_lse = lse != nullptr && lse->ptr != nullptr;
  if (want_lse && !empty) {
    if (lse->dtype != FL_F32) return fail(FL_ERR_DTYPE, "lse must be f32");
    const int64_t lsz[5] = {B, 1, H, T, 1};
    for (int a = 0; a < 5; ++a)
      if (lse->size[a] != lsz[a])
        return fail(FL_ERR_SHAPE, "lse size[%d] = %lld, expected %lld", a, (long long)lse->size[a], (long long)lsz[a]);
  }
  if (empty) return FL_OK;
  if (aux == nullptr) return fail(FL_ERR_AUX_MISSING, "the decode step needs aux (workspace)");
  if (desc->score_mod == FL_MOD_ALIBI && aux->alibi_slopes == nullptr) return fail(FL_ERR_AUX_MISSING, "alibi_slopes");
  const int ns = decode_splits(B, Hkv, D, kv->max_seq_len);
  const size_t ws_need = (size_t)(B * T * H * ns) * (size_t)(D + 2) * sizeof(float);
  if (aux->workspace == nullptr || aux->workspace_bytes < ws_need)
    return fail(FL_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", ws_need, aux->workspace ? aux->workspace_bytes : (size_t)0);
  if (((uintptr_t)aux->workspace) % 16 != 0) return fail(FL_ERR_ALIGN, "workspace not 16-byte aligned");
  if (B * Hkv * ns > 0x7fffffffLL || B * T * H > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "too many workgroups");

  fl::DecodeParams p;
  memset(&p, 0, sizeof(p));
  p.q = (const uint16_t*)q->ptr;
  p.q_sb = B > 1 ? q->stride[0] : 0;
  p.q_sh = H > 1 ? q->stride[2] : 0;
  p.q_st = T > 1 ? q->stride[3] : 0;
  p.k = (const uint16_t*)k_cache->ptr;
  p.v = (const uint16_t*)v_cache->ptr;
  p.k_sp = pages > 1 ? k_cache->stride[0] : 0;
  p.k_st = page_size > 1 ? k_cache->stride[3] : 0;
  p.k_sh = Hkv > 1 ? k_cache->stride[2] : 0;
  p.v_sp = pages > 1 ? v_cache->stride[0] : 0;
  p.v_st = page_size > 1 ? v_cache->stride[3] : 0;
  p.v_sh = Hkv > 1 ? v_cache->stride[2] : 0;
  p.block_table = kv->block_table;
  p.table_stride = kv->table_stride;
  p.page_shift = page_shift;
  p.seq_lens = kv->seq_lens;
  p.out = out->ptr;
  p.o_sb = B > 1 ? out->stride[0] : 0;
  p.o_sh = H > 1 ? out->stride[2] : 0;
  p.o_st = T > 1 ? out->stride[3] : 0;
  p.out_f32 = out->dtype == FL_F32;
  if (want_lse) {
    p.lse = (float*)lse->ptr;
    p.lse_sb = B > 1 ? lse->stride[0] : 0;
    p.lse_sh = H > 1 ? lse->stride[2] : 0;
    p.lse_st = T > 1 ? lse->stride[3] : 0;
  }
  p.part_o = (float*)aux->workspace;
  p.part_ml = p.part_o + B * T * H * ns * D;
  p.alibi_slopes = aux->alibi_slopes;
  p.B = (int)B; p.H = (int)H; p.Hkv = (int)Hkv; p.nsplit = ns; p.T = (int)T;
  p.max_len = kv->max_seq_len;
  p.num_pages = (int)pages;
  p.window = (mask & FL_MASK_WINDOW) ? clamp_window(desc->window, kv->max_seq_len, kv->max_seq_len) : -1;
  p.scale = desc->scale;
  p.softcap = desc->softcap;
  hipStream_t stream = (hipStream_t)stream_v;
  hipError_t e = de->main(p, (int)(B * Hkv * ns), stream);
  if (e != hipSuccess) return fail(FL_ERR_LAUNCH, "decode launch: %s", hipGetErrorString(e));
  if (ns > 1 && (e = de->combine(p, (int)(B * T * H), stream)) != hipSuccess)   // a single split writes the result itself
    return fail(FL_ERR_LAUNCH, "decode merge launch: %s", hipGetErrorString(e));
  return FL_OK;
}

// Chunks of so few rows that all (query row, head) pairs of a kv head fit the columns of the decode kernels go
// there: the cache is then read once per kv head instead of once per query head, no MFMA row is idle, and the key
// range is split so that few or ragged sequences still fill the chip.  With more than 32 pairs (two column blocks) the
// in-place forward kernel with packed heads measured faster when it has the workgroups to fill the chip (64 sequences x
// 16 rows, 32 / 8 heads: 0.41 against 0.53 ms), so those chunks go there when it packs and launches 512 or more.
static bool prefill_as_decode(int64_t D, int64_t B, int64_t H, int64_t Hkv, int64_t Sq, bool in_place_ok) {
  if (g_tuning.prefill_gather != 0) return false;
  if (!((D == 64 || D == 128) && Hkv > 0 && H % Hkv == 0 && Sq * (H / Hkv) <= kDecodeMaxPairs)) return false;
  if (Sq * (H / Hkv) <= 32 || !in_place_ok) return true;
  const PagedShape s = paged_shape(B * H, H / Hkv, Sq);
  const int64_t rows = (s.wide ? 256 : 128) / s.pack;
  return !(s.pack > 1 && (B * H / s.pack) * ((Sq + rows - 1) / rows) >= 512);
}

// Does the forward kernel read these pages in place?  It can when every direct-load instruction of a tile (512 / D
// consecutive tokens) lies in one page.  It does for chunks of up to 1024 rows: the in-place kernel (two ring slots; four
// waves, eight from 512 rows on at head dim 128) looks up a page and forms a base per wave and tile (per load instruction
// when pages hold fewer than the wave's 8 or 16 tokens) and runs at 0.85 - 0.93 of the tuned dense kernel, while the copy costs the time of
// about 100 query rows of attention.  Measured at 32 / 8 heads, D = 128, 8192 cached tokens (ms in place / copied):
// 64 rows 0.35 (heads packed) / 1.32, 128 rows 0.355 / 0.55, 256 rows 0.32 / 0.41, 512 rows 0.55 / 0.64,
// 1024 rows 1.00 / 1.06, 2048 rows 1.82 / 1.77.
static bool prefill_in_place(int64_t D, int64_t page_size, bool has_table, int64_t Sq, int64_t page_stride) {
  if (g_tuning.prefill_gather == 1 || !(D == 32 || D == 64 || D == 128)) return false;
  if (page_stride * 2 >= (1LL << 32)) return false;   // the kernel multiplies page numbers by 32-bit byte strides
  if (has_table && page_size < 512 / D) return false;
  return g_tuning.prefill_gather == 2 || Sq <= 1024;
}

size_t fl_attn_prefill_paged_workspace_size(const fl_tensor* q, const fl_tensor* k_cache, const fl_paged_kv* kv) {
  if (q == nullptr || k_cache == nullptr || kv == nullptr) return 0;
  const bool in_place = prefill_in_place(q->size[4], k_cache->size[3], kv->block_table != nullptr, q->size[3], k_cache->stride[0]);
  if (prefill_as_decode(q->size[4], q->size[0], q->size[2], k_cache->size[2], q->size[3], in_place))
    return fl_attn_decode_workspace_size(q, k_cache, kv);
  if (in_place) return 0;
  return prefill_layout(q->size[0], k_cache->size[2], q->size[4], kv->max_seq_len).total;
}

fl_status fl_attn_prefill_paged(const fl_tensor* q, const fl_tensor* k_cache, const fl_tensor* v_cache, const fl_paged_kv* kv,
                                const fl_variant_desc* desc, const fl_aux* aux, fl_tensor* out, fl_tensor* lse, void* stream_v) {
  g_detail[0] = 0;
  fl_status st = check_desc(desc);
  if (st != FL_OK) return st;
  if (q == nullptr || k_cache == nullptr || v_cache == nullptr || kv == nullptr || out == nullptr)
    return fail(FL_ERR_NULL, "q, k_cache, v_cache, kv or out is NULL");
  if (kv->struct_size != sizeof(fl_paged_kv))
    return fail(FL_ERR_DESC, "kv->struct_size = %u, expected %zu", kv->struct_size, sizeof(fl_paged_kv));
  if (aux != nullptr && aux->struct_size != sizeof(fl_aux))
    return fail(FL_ERR_DESC, "aux->struct_size = %u, expected %zu", aux->struct_size, sizeof(fl_aux));
  const uint32_t mask = canonical_mask(desc->mask);
  if ((mask & (FL_MASK_DOC | FL_MASK_PREFIX)) || desc->n_bias != 0 || desc->combine != FL_SINGLE || desc->epilogue != 0 ||
      desc->q_offset != 0)
    return fail(FL_ERR_UNSUPPORTED, "prefill over the paged cache covers scale, score_mod and the sliding window only "
                                    "(the causal mask and the rows' positions follow from seq_lens)");
  if (q->dtype != FL_BF16) return fail(FL_ERR_DTYPE, "prefill over the paged cache takes bf16 inputs (q dtype %d)", q->dtype);

  const int64_t B = q->size[0], H = q->size[2], Sq = q->size[3], D = q->size[4];
  const int64_t pages = k_cache->size[0], Hkv = k_cache->size[2], page_size = k_cache->size[3];
  if (B < 0 || H < 0 || Sq < 0 || D <= 0 || pages < 0 || page_size <= 0) return fail(FL_ERR_SHAPE, "negative size");
  if (pages > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "more pages than an int32 table entry can name");
  if (pages == 0 && kv->max_seq_len > 0) return fail(FL_ERR_SHAPE, "max_seq_len = %d with an empty cache", kv->max_seq_len);
  if (q->size[1] != 1) return fail(FL_ERR_SHAPE, "q must be [B, 1, H, Sq, D]");
  if (Hkv <= 0 || H % Hkv != 0)
    if (H != 0) return fail(FL_ERR_SHAPE, "kv heads (%lld) must divide q heads (%lld)", (long long)Hkv, (long long)H);
  if (kv->page_size != page_size) return fail(FL_ERR_SHAPE, "kv->page_size = %d, cache size[3] = %lld", kv->page_size, (long long)page_size);
  if (kv->max_seq_len < 0) return fail(FL_ERR_SHAPE, "max_seq_len negative");
  if (D % 8 != 0 || v_cache->size[4] != D) return fail(FL_ERR_UNSUPPORTED, "D = Dv, a multiple of 8 (D=%lld Dv=%lld)", (long long)D, (long long)v_cache->size[4]);
  int page_shift = 0;
  if (kv->block_table != nullptr) {
    if (page_size < 8 || (page_size & (page_size - 1)) != 0)
      return fail(FL_ERR_SHAPE, "with a block table the page size (%lld) must be a power of two >= 8", (long long)page_size);
    while ((1LL << page_shift) < page_size) ++page_shift;
    if (kv->table_stride < (kv->max_seq_len + page_size - 1) / page_size)
      return fail(FL_ERR_SHAPE, "table_stride %d is less than the pages of max_seq_len", kv->table_stride);
  } else {
    if (pages < B) return fail(FL_ERR_SHAPE, "without a block table the cache needs a page per sequence");
    if (kv->max_seq_len > page_size) return fail(FL_ERR_SHAPE, "max_seq_len exceeds the page size");
  }
  const bool empty = (B == 0 || H == 0 || Sq == 0);
  const int64_t qsz[5] = {B, 1, H, Sq, D}, csz[5] = {pages, 1, Hkv, page_size, D};
  if (!empty) {
    if ((st = check_data_tensor(q, "q", FL_BF16, qsz)) != FL_OK) return st;
    if (kv->max_seq_len > 0) {
      if ((st = check_data_tensor(k_cache, "k_cache", FL_BF16, csz)) != FL_OK) return st;
      if ((st = check_data_tensor(v_cache, "v_cache", FL_BF16, csz)) != FL_OK) return st;
    }
    if (kv->seq_lens == nullptr) return fail(FL_ERR_NULL, "seq_lens is NULL");
  }
  if (empty) return FL_OK;

  // The inner forward call: causal, with the sequences' own key counts (and through them the positions of the query
  // rows) read on the device.  Everything it can refuse is checked here, before the first launch.
  fl_variant_desc inner = *desc;
  inner.mask = mask | FL_MASK_CAUSAL;
  fl_aux ia;
  memset(&ia, 0, sizeof(ia));
  ia.struct_size = sizeof(fl_aux);
  ia.alibi_slopes = aux != nullptr ? aux->alibi_slopes : nullptr;
  if (!fl_variant_supported(&inner, FL_BF16, (int)D, (int)D))
    return fail(FL_ERR_UNSUPPORTED, "no forward kernel for D=%lld score_mod=%u with this mask", (long long)D, desc->score_mod);
  if (desc->score_mod == FL_MOD_ALIBI && ia.alibi_slopes == nullptr) return fail(FL_ERR_AUX_MISSING, "alibi_slopes");
  if (out->dtype != FL_BF16 && out->dtype != FL_F32) return fail(FL_ERR_DTYPE, "out dtype %d", out->dtype);
  if ((st = check_data_tensor(out, "out", out->dtype, qsz)) != FL_OK) return st;
  if (lse != nullptr && lse->ptr != nullptr) {
    if (lse->dtype != FL_F32) return fail(FL_ERR_DTYPE, "lse must be f32");
    const int64_t lsz[5] = {B, 1, H, Sq, 1};
    for (int a = 0; a < 5; ++a)
      if (lse->size[a] != lsz[a])
        return fail(FL_ERR_SHAPE, "lse size[%d] = %lld, expected %lld", a, (long long)lse->size[a], (long long)lsz[a]);
  }

  // A few rows: the decode kernels, with their own checks of the same arguments.
  const bool in_place = prefill_in_place(D, page_size, kv->block_table != nullptr, Sq, k_cache->stride[0]);
  if (prefill_as_decode(D, B, H, Hkv, Sq, in_place)) return fl_attn_decode(q, k_cache, v_cache, kv, desc, aux, out, lse, stream_v);

  // In place (short chunks): the forward kernel takes the cache tensors as its keys and values and finds every tile's
  // pages through the block table itself; no copy, no workspace.
  if (in_place) {
    if (v_cache->stride[0] * 2 >= (1LL << 32)) return fail(FL_ERR_STRIDE, "v_cache page stride is not below 2^32 bytes");
    if (kv->max_seq_len == 0) {                    // nothing cached anywhere: out = 0, lse = -inf through the dense path's Sk = 0
      fl_tensor none = *k_cache;
      none.size[0] = B; none.size[3] = 0;
      return forward_call(q, &none, &none, &inner, &ia, out, lse, stream_v, kv->seq_lens);
    }
    PagedKeys pk;
    pk.block_table = kv->block_table;
    pk.table_stride = kv->table_stride;
    pk.page_shift = page_shift;
    pk.num_pages = (int)pages;
    pk.max_len = kv->max_seq_len;
    return forward_call(q, k_cache, v_cache, &inner, &ia, out, lse, stream_v, kv->seq_lens, &pk);
  }

  // Otherwise (long chunks, pages smaller than a load instruction's rows, or on request): the pages are copied into
  // dense tensors first.
  if (aux == nullptr) return fail(FL_ERR_AUX_MISSING, "prefill over this paged cache needs aux (workspace)");
  const PrefillLayout L = prefill_layout(B, Hkv, D, kv->max_seq_len);
  if (aux->workspace == nullptr || aux->workspace_bytes < L.total)
    return fail(FL_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", L.total, aux->workspace ? aux->workspace_bytes : (size_t)0);
  if (((uintptr_t)aux->workspace) % 16 != 0) return fail(FL_ERR_ALIGN, "workspace not 16-byte aligned");
  const int64_t Sk = kv->max_seq_len;
  const int64_t total = B * Hkv * Sk * (D / 8);
  if ((total + 255) / 256 > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "too many rows to gather");
  char* ws = (char*)aux->workspace;
  fl_tensor kd, vd;
  memset(&kd, 0, sizeof(kd));
  kd.dtype = FL_BF16;
  kd.size[0] = B; kd.size[1] = 1; kd.size[2] = Hkv; kd.size[3] = Sk; kd.size[4] = D;
  kd.stride[4] = 1; kd.stride[3] = D; kd.stride[2] = Sk * D; kd.stride[1] = Hkv * Sk * D; kd.stride[0] = Hkv * Sk * D;
  vd = kd;
  kd.ptr = ws + L.off_k;
  vd.ptr = ws + L.off_v;

  if (total > 0) {
    GatherParams g;
    memset(&g, 0, sizeof(g));
    const fl_tensor* caches[2] = {k_cache, v_cache};
    for (int w = 0; w < 2; ++w) {
      g.cache[w] = (const uint16_t*)caches[w]->ptr;
      g.sp[w] = pages > 1 ? caches[w]->stride[0] : 0;
      g.st[w] = page_size > 1 ? caches[w]->stride[3] : 0;
      g.sh[w] = Hkv > 1 ? caches[w]->stride[2] : 0;
    }
    g.dst[0] = (uint16_t*)kd.ptr;
    g.dst[1] = (uint16_t*)vd.ptr;
    g.table = kv->block_table;
    g.seq_lens = kv->seq_lens;
    g.table_stride = kv->table_stride;
    g.page_shift = page_shift;
    g.page_mask = (int)page_size - 1;
    g.num_pages = (int)pages;
    g.max_len = kv->max_seq_len;
    g.Hkv = (int)Hkv;
    g.L = (int)Sk;
    g.chunks = (int)(D / 8);
    g.total = total;
    hipLaunchKernelGGL(gather_pages_kernel, dim3((unsigned)((total + 255) / 256), 2), dim3(256), 0, (hipStream_t)stream_v, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FL_ERR_LAUNCH, "page gather launch: %s", hipGetErrorString(e));
  }
  return forward_call(q, &kd, &vd, &inner, &ia, out, lse, stream_v, kv->seq_lens);
}

}  // extern "C"
