// C-ABI entry points: argument validation, descriptor -> kernel-specialisation lookup, launch.
// Nothing here computes attention; every step of the path runs in the kernels.
#include <hip/hip_runtime.h>

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
const fl::KernelEntry* find_entry(const fl_variant_desc* d, int dtype, int D, int Dv, int64_t Sk = 0, int64_t heads = 0,
                                  int64_t Sq = 0) {
  const Registry& r = registry();
  const int mask = (int)canonical_mask(d->mask);
  const fl::KernelEntry* best = nullptr;
  const fl::KernelEntry* short_loop = nullptr;    // the variant's 32-key-tile shape at three or four waves per SIMD, if listed
  const fl::KernelEntry* four_waves = nullptr;    // a 4-wave, one-row-block shape of the variant (128 query rows per workgroup)
  const fl::KernelEntry* deep_ring = nullptr;     // the default shape with four-slot K / V rings (a barrier per two tiles)
  for (int t = 0; t < 5; ++t)
    for (int e = 0; e < r.n[t]; ++e) {
      const fl::KernelEntry& k = r.tab[t][e];
      if (k.key.dtype != dtype || k.key.diff != (int)d->combine) continue;
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

// Head dims the bf16 kernel template can be instantiated for at run time.
bool jit_dims_ok(int64_t D, int64_t Dv) {
  return (D == 32 || D == 64 || D == 128) && (Dv == 32 || Dv == 64 || Dv == 128);
}

size_t workspace_bytes(int64_t B, int64_t Sq, int64_t Sk, uint32_t mask) {
  if (!(mask & FL_MASK_DOC)) return 0;
  const int64_t nq = (Sq + fl::kSumBlock - 1) / fl::kSumBlock, nk = (Sk + fl::kSumBlock - 1) / fl::kSumBlock;
  return (size_t)(B * (nq + nk)) * sizeof(int2);
}

// (min, max) of the document ids of each block of 32 tokens: one wave per block.
__global__ void doc_summary_kernel(const int32_t* __restrict__ ids, int2* __restrict__ sum, int S, int nblk,
                                   int total) {
  const int w = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int lane = threadIdx.x & 63;
  if (w >= total) return;
  const int b = w / nblk, blk = w % nblk;
  const int j = blk * fl::kSumBlock + (lane & 31);
  const int jc = j < S ? j : S - 1;
  int lo = ids[(int64_t)b * S + jc], hi = lo;
#pragma unroll
  for (int o = 16; o >= 1; o >>= 1) {
    lo = min(lo, __shfl_xor(lo, o));
    hi = max(hi, __shfl_xor(hi, o));
  }
  if (lane == 0) sum[w] = make_int2(lo, hi);
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

const fl::BwdEntry* find_bwd_entry(const fl_variant_desc* d, int D) {
  static const BwdRegistry reg;                    // initialised once, also under concurrent first calls
  const fl::BwdEntry* const* tab = reg.tab;
  const int* n = reg.n;
  const int mask = (int)canonical_mask(d->mask);
  for (int t = 0; t < 2; ++t)
    for (int e = 0; e < n[t]; ++e) {
      const fl::BwdEntry& k = tab[t][e];
      if (k.key.D == D && k.key.mod == (int)d->score_mod && k.key.mask == mask) return &k;
    }
  return nullptr;
}

bool bwd_desc_ok(const fl_variant_desc* d) {
  return d->n_bias == 0 && d->combine == FL_SINGLE && d->epilogue == 0 && d->q_offset == 0;
}

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

const fl::DecodeEntry* find_decode_entry(int D, int mod) {
  int n = 0;
  const fl::DecodeEntry* tab = fl::entries_decode(&n);
  for (int e = 0; e < n; ++e)
    if (tab[e].D == D && tab[e].mod == mod) return &tab[e];
  return nullptr;
}

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

fl_status fl_attn_fwd(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_variant_desc* desc,
                      const fl_aux* aux, fl_tensor* out, fl_tensor* lse, void* stream_v) {
  g_detail[0] = 0;
  fl_status st = check_desc(desc);
  if (st != FL_OK) return st;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr) return fail(FL_ERR_NULL, "q, k, v or out is NULL");
  if (aux != nullptr && aux->struct_size != sizeof(fl_aux))
    return fail(FL_ERR_DESC, "aux->struct_size = %u, expected %zu", aux->struct_size, sizeof(fl_aux));

  const int dtype = q->dtype;
  if (dtype != FL_BF16 && dtype != FL_F32) return fail(FL_ERR_DTYPE, "q dtype %d not bf16/f32", dtype);
  const int64_t B = q->size[0], G = q->size[1], H = q->size[2], Sq = q->size[3], D = q->size[4];
  const int64_t Hkv = k->size[2], Sk = k->size[3], Dv = v->size[4];
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
    if (Sk > 0) {
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
  const fl::KernelEntry* ke = find_entry(desc, dtype, (int)D, (int)Dv, Sk, B * G * H, Sq);
  if (ke == nullptr && dtype == FL_BF16 && jit_dims_ok(D, Dv)) {
    // not in the compiled table: the same kernel template, instantiated for this descriptor on first use
    ke = fl::jit_forward_entry(fl::JitRequest{(int)D, (int)Dv, (int)desc->score_mod, mask, (int)desc->n_bias, diff, desc->epilogue});
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
  p.window = clamp_window(desc->window, Sq + desc->q_offset, Sk);
  p.prefix = desc->prefix_len;
  p.q_off = desc->q_offset;
  if ((int64_t)desc->q_offset + Sq > 0x7fffff00LL) return fail(FL_ERR_SHAPE, "q_offset + Sq too large");
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
  const int64_t nbh = B * G * H;
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
    const int64_t total = nbh * Sq;
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
    hipLaunchKernelGGL(doc_summary_kernel, dim3((tq + 3) / 4), dim3(256), 0, stream, aux->q_doc_ids, p.q_sum, (int)Sq, nqs, tq);
    hipLaunchKernelGGL(doc_summary_kernel, dim3((tk + 3) / 4), dim3(256), 0, stream, aux->kv_doc_ids, p.kv_sum, (int)Sk, nks, tk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FL_ERR_LAUNCH, "doc summary launch: %s", hipGetErrorString(e));
  }
  hipError_t e = ke->jit != nullptr ? fl::jit_forward_launch(*ke, p, (int)nblocks, stream) : ke->launch(p, (int)nblocks, stream);
  if (e != hipSuccess) return fail(FL_ERR_LAUNCH, "kernel launch: %s", hipGetErrorString(e));
  return FL_OK;
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
  if (check_desc(desc) != FL_OK || dtype != FL_BF16 || D != Dv || !bwd_desc_ok(desc)) return 0;
  return find_bwd_entry(desc, D) != nullptr ? 1 : 0;
}

fl_status fl_attn_bwd(const fl_tensor* q, const fl_tensor* k, const fl_tensor* v, const fl_tensor* out,
                      const fl_tensor* dout, const fl_tensor* lse, const fl_variant_desc* desc, const fl_aux* aux,
                      fl_tensor* dq, fl_tensor* dk, fl_tensor* dv, void* stream_v) {
  g_detail[0] = 0;
  fl_status st = check_desc(desc);
  if (st != FL_OK) return st;
  if (q == nullptr || k == nullptr || v == nullptr || out == nullptr || dout == nullptr || lse == nullptr ||
      dq == nullptr || dk == nullptr || dv == nullptr)
    return fail(FL_ERR_NULL, "a tensor descriptor is NULL");
  if (aux != nullptr && aux->struct_size != sizeof(fl_aux))
    return fail(FL_ERR_DESC, "aux->struct_size = %u, expected %zu", aux->struct_size, sizeof(fl_aux));
  if (!bwd_desc_ok(desc))
    return fail(FL_ERR_UNSUPPORTED, "the backward pass covers variants without bias, second stream, epilogue and query offset");
  if (q->dtype != FL_BF16) return fail(FL_ERR_DTYPE, "the backward pass takes bf16 inputs (q dtype %d)", q->dtype);

  const int64_t B = q->size[0], G = q->size[1], H = q->size[2], Sq = q->size[3], D = q->size[4];
  const int64_t Hkv = k->size[2], Sk = k->size[3], Dv = v->size[4];
  if (B < 0 || G < 0 || H < 0 || Sq < 0 || Sk < 0 || D <= 0 || Dv <= 0) return fail(FL_ERR_SHAPE, "negative size");
  if (Sq > 0x7fffff00LL || Sk > 0x7fffff00LL || B * G * H > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "size too large");
  if (Hkv <= 0 || H % (Hkv > 0 ? Hkv : 1) != 0)
    if (H != 0) return fail(FL_ERR_SHAPE, "k heads (%lld) must divide q heads (%lld)", (long long)Hkv, (long long)H);
  const uint32_t mask = canonical_mask(desc->mask);
  const fl::BwdEntry* be = D == Dv ? find_bwd_entry(desc, (int)D) : nullptr;
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
  p.window = clamp_window(desc->window, Sq, Sk);
  p.prefix = desc->prefix_len;
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
    hipLaunchKernelGGL(doc_summary_kernel, dim3((tq + 3) / 4), dim3(256), 0, stream, aux->q_doc_ids, p.q_sum, (int)Sq, nqs, tq);
    hipLaunchKernelGGL(doc_summary_kernel, dim3((tk + 3) / 4), dim3(256), 0, stream, aux->kv_doc_ids, p.kv_sum, (int)Sk, nks, tk);
    if ((e = hipGetLastError()) != hipSuccess) return fail(FL_ERR_LAUNCH, "doc summary launch: %s", hipGetErrorString(e));
  }
  if (!no_rows) {
    const int lanes_per_row = (int)Dv / 8;
    const int64_t nb_prep = (rows * lanes_per_row + 255) / 256;
    if ((e = be->prep(p, (int)nb_prep, stream)) != hipSuccess) return fail(FL_ERR_LAUNCH, "pre-pass launch: %s", hipGetErrorString(e));
    // Sk == 0: the key loop is empty and dq comes out as zeros
    if ((e = be->dq(p, (int)nb_q, stream)) != hipSuccess) return fail(FL_ERR_LAUNCH, "dq launch: %s", hipGetErrorString(e));
  }
  if (!no_keys) {
    // Sq == 0: the query loop is empty and dk, dv come out as zeros
    if ((e = be->dkdv(p, (int)nb_k, stream)) != hipSuccess) return fail(FL_ERR_LAUNCH, "dk/dv launch: %s", hipGetErrorString(e));
    if (p.hsplit > 1) {
      const int64_t chunks = B * G * Hkv * Sk * (D / 4);
      if ((e = be->reduce(p, (int)((chunks + 255) / 256), stream)) != hipSuccess)
        return fail(FL_ERR_LAUNCH, "dk/dv reduction launch: %s", hipGetErrorString(e));
    }
  }
  return FL_OK;
}

size_t fl_attn_decode_workspace_size(const fl_tensor* q, const fl_tensor* k_cache, const fl_paged_kv* kv) {
  if (q == nullptr || k_cache == nullptr || kv == nullptr) return 0;
  const int64_t B = q->size[0], H = q->size[2], D = q->size[4];
  const int ns = decode_splits(B, k_cache->size[2], D, kv->max_seq_len);
  return (size_t)(B * H * ns) * (size_t)(D + 2) * sizeof(float);
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

  const int64_t B = q->size[0], H = q->size[2], D = q->size[4];
  const int64_t pages = k_cache->size[0], Hkv = k_cache->size[2], page_size = k_cache->size[3];
  if (B < 0 || H < 0 || D <= 0 || pages < 0 || page_size <= 0) return fail(FL_ERR_SHAPE, "negative size");
  if (pages > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "more pages than an int32 table entry can name");
  if (pages == 0 && kv->max_seq_len > 0) return fail(FL_ERR_SHAPE, "max_seq_len = %d with an empty cache", kv->max_seq_len);
  if (q->size[1] != 1 || q->size[3] != 1) return fail(FL_ERR_SHAPE, "q must be [B, 1, H, 1, D]");
  if (Hkv <= 0 || H % Hkv != 0 || H / Hkv > 32)
    if (H != 0) return fail(FL_ERR_SHAPE, "kv heads (%lld) must divide q heads (%lld), at most 32 q heads per kv head", (long long)Hkv, (long long)H);
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
  const fl::DecodeEntry* de = find_decode_entry((int)D, (int)desc->score_mod);
  if (de == nullptr || v_cache->size[4] != D)
    return fail(FL_ERR_UNSUPPORTED, "no decode specialisation for D=%lld Dv=%lld score_mod=%u", (long long)D,
                (long long)v_cache->size[4], desc->score_mod);
  const bool empty = (B == 0 || H == 0);
  const int64_t qsz[5] = {B, 1, H, 1, D}, csz[5] = {pages, 1, Hkv, page_size, D};
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
    const int64_t lsz[5] = {B, 1, H, 1, 1};
    for (int a = 0; a < 5; ++a)
      if (lse->size[a] != lsz[a])
        return fail(FL_ERR_SHAPE, "lse size[%d] = %lld, expected %lld", a, (long long)lse->size[a], (long long)lsz[a]);
  }
  if (empty) return FL_OK;
  if (aux == nullptr) return fail(FL_ERR_AUX_MISSING, "the decode step needs aux (workspace)");
  if (desc->score_mod == FL_MOD_ALIBI && aux->alibi_slopes == nullptr) return fail(FL_ERR_AUX_MISSING, "alibi_slopes");
  const int ns = decode_splits(B, Hkv, D, kv->max_seq_len);
  const size_t ws_need = (size_t)(B * H * ns) * (size_t)(D + 2) * sizeof(float);
  if (aux->workspace == nullptr || aux->workspace_bytes < ws_need)
    return fail(FL_ERR_WORKSPACE, "workspace needs %zu bytes, got %zu", ws_need, aux->workspace ? aux->workspace_bytes : (size_t)0);
  if (((uintptr_t)aux->workspace) % 16 != 0) return fail(FL_ERR_ALIGN, "workspace not 16-byte aligned");
  if (B * Hkv * ns > 0x7fffffffLL || B * H > 0x7fffffffLL) return fail(FL_ERR_SHAPE, "too many workgroups");

  fl::DecodeParams p;
  memset(&p, 0, sizeof(p));
  p.q = (const uint16_t*)q->ptr;
  p.q_sb = B > 1 ? q->stride[0] : 0;
  p.q_sh = H > 1 ? q->stride[2] : 0;
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
  p.out_f32 = out->dtype == FL_F32;
  if (want_lse) {
    p.lse = (float*)lse->ptr;
    p.lse_sb = B > 1 ? lse->stride[0] : 0;
    p.lse_sh = H > 1 ? lse->stride[2] : 0;
  }
  p.part_o = (float*)aux->workspace;
  p.part_ml = p.part_o + B * H * ns * D;
  p.alibi_slopes = aux->alibi_slopes;
  p.B = (int)B; p.H = (int)H; p.Hkv = (int)Hkv; p.nsplit = ns;
  p.max_len = kv->max_seq_len;
  p.num_pages = (int)pages;
  p.window = (mask & FL_MASK_WINDOW) ? clamp_window(desc->window, kv->max_seq_len, kv->max_seq_len) : -1;
  p.scale = desc->scale;
  p.softcap = desc->softcap;
  hipStream_t stream = (hipStream_t)stream_v;
  hipError_t e = de->main(p, (int)(B * Hkv * ns), stream);
  if (e != hipSuccess) return fail(FL_ERR_LAUNCH, "decode launch: %s", hipGetErrorString(e));
  if (ns > 1 && (e = de->combine(p, (int)(B * H), stream)) != hipSuccess)   // a single split writes the result itself
    return fail(FL_ERR_LAUNCH, "decode merge launch: %s", hipGetErrorString(e));
  return FL_OK;
}

}  // extern "C"
