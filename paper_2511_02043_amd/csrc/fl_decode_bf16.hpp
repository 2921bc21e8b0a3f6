// Decode-step attention over a paged key/value cache for gfx950: the newest query rows of each
// sequence (the token being generated; or the few tokens a speculative step verifies, or a very
// short prompt chunk) against that sequence's cached keys and values -- the shape the serving
// experiment of the paper's Sec. 4.1 runs once per generated token.  The arithmetic is the
// forward pass (Eq. 3, score_mod of Eq. 4, online softmax of Sec. 3.4) for the T query rows at
// positions len - T .. len - 1, causal among themselves; the work is reading the cache once, so
// the kernel is built around HBM: every wave streams its own key/value tiles into a private LDS
// ring with direct global->LDS loads, several tiles ahead, and never meets another wave inside
// the loop.
//
//   * a workgroup owns one (sequence, kv head, split of the key range); its waves take the
//     tiles of that range round-robin;
//   * the (query row, query head) pairs that share the kv head are the columns of the MFMA tiles
//     (lane = pair; CB blocks of 32 columns), so a K / V tile is read once for the whole group:
//     S^T = K Q^T and O^T += V^T P^T exactly as in the forward kernel, with the running max /
//     sum per lane;
//   * a page table is followed per tile row when the direct loads are issued;
//   * waves, then splits, are merged with the rescale rule of Sec. 3.3 / 3.4 (the partial
//     (m, l, O) of each split goes through the caller's workspace to a small second kernel).
#pragma once
#include "fl_bwd_bf16.hpp"

namespace fl {

struct DecodeParams {
  const uint16_t* q;               // [B, H, T, D], strides in elements
  int64_t q_sb, q_sh, q_st;
  const uint16_t* k;               // cache: page, token in page, kv head strides in elements
  const uint16_t* v;
  int64_t k_sp, k_st, k_sh, v_sp, v_st, v_sh;
  const int32_t* block_table;      // [B, table_stride], or null: sequence b is page b
  int32_t table_stride;
  int32_t page_shift;              // log2(tokens per page) when block_table is given
  const int32_t* seq_lens;         // [B]
  void* out;                       // [B, H, T, D]
  int64_t o_sb, o_sh, o_st;
  int32_t out_f32;
  float* lse;                      // [B, H, T] or null
  int64_t lse_sb, lse_sh, lse_st;
  float* part_o;                   // workspace [B, T, H, nsplit, D]
  float* part_ml;                  // workspace [B, T, H, nsplit, 2]: running max (log2 domain), sum
  const float* alibi_slopes;       // [H]
  int32_t B, H, Hkv, nsplit;
  int32_t T;                       // query rows per sequence: the tokens at positions len - T .. len - 1
  int32_t num_pages;               // size[0] of the caches: table entries are cut to [0, num_pages)
  int32_t max_len;                 // the host-side bound of seq_lens that sized the launch, the table and the workspace
  int32_t window;                  // < 0: no window
  float scale, softcap;
};

template <int D_, int MOD_, int CB_ = 1>
struct DecodeCfg : BwdCfg<D_, MOD_, 0, 32, 1> {
  static constexpr int CB = CB_;                   // blocks of 32 (query row, head) columns per kv head
  // D = 128: five waves with 16 KiB stages, which fill the CU's 160 KiB of LDS (four, one per SIMD, moved 4 % fewer
  // bytes per second; three waves with three stages each -- more bytes in flight per wave, fewer waves -- 15 % fewer;
  // with two column blocks the register budget allows one wave per SIMD only); D = 64: eight waves (two per SIMD) with 8 KiB
  // stages -- a tile carries half the bytes there, and a second wave on the SIMD hides the first one's
  // per-tile chain of waits (load, LDS read, matrix core, exponentials); ten waves, or six with three stages, measured no better
  static constexpr int NWV = D_ == 128 ? (CB_ == 1 ? 5 : 4) : 8;    // waves per workgroup
  static constexpr int NSTG = 2;                   // ring stages per wave
  // register budget: the workgroup fills a CU's LDS, so D = 128 has one wave per SIMD anyway; two column blocks
  // there need more than 256 registers
  static constexpr int WPE = (D_ == 128 && CB_ == 2) ? 1 : 2;
  static constexpr int STAGE = 2 * BwdCfg<D_, MOD_, 0, 32, 1>::TILE;                 // K tile, V tile
  static constexpr int WAVE_LDS = NSTG * STAGE;
  static constexpr int LDS = NWV * WAVE_LDS;
  static constexpr int IPT = 2 * BwdCfg<D_, MOD_, 0, 32, 1>::TILE_INSTR;             // load instructions per tile
  static_assert((NSTG - 1) * IPT < 64, "vmcnt is a 6-bit counter");
};

template <int N>
__device__ __forceinline__ void wait_vm() {          // at most N vector-memory operations still in flight
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x0F70 | ((N >> 4) << 14));
}

template <class C>
__global__ void __launch_bounds__(C::NWV * 64) __attribute__((amdgpu_waves_per_eu(C::WPE, C::WPE)))
decode_kernel(const DecodeParams p) {
  constexpr int D = C::D, KK = C::KK, DB = C::DB, ROW = C::ROW, BN = 32, CB = C::CB;
  typedef BwdWave<C> W;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  W w;
  w.init(tid & 63);
  const int lane = w.lane;

  const int split = blockIdx.x % p.nsplit;
  const int bhk = blockIdx.x / p.nsplit;
  const int hk = bhk % p.Hkv, b = bhk / p.Hkv;
  const int group = p.H / p.Hkv;                   // query heads per kv head
  const int ncol = p.T * group;                    // (row, head) pairs of this kv head (<= 32 * CB)
  // a length outside [0, max_len] would walk past the block table: such a sequence is cut to the bound
  const int len = min(max(p.seq_lens[b], 0), p.max_len);
  // this lane's pair in each column block (clamped copies beyond the last pair): query row, head, position
  int row[CB], hq[CB], pos[CB];
  bool live[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const int c = 32 * cb + w.col;
    live[cb] = c < ncol;
    const int cc = live[cb] ? c : ncol - 1;
    row[cb] = cc / group;
    hq[cb] = hk * group + cc % group;
    pos[cb] = len - p.T + row[cb];                 // negative: a row before the sequence's first token sees no key
  }

  // key tiles of this workgroup, then of this wave: from the first key the oldest row sees to the last key
  const int first_key = p.window >= 0 ? max(0, len - p.T - p.window) : 0;
  // tiles that start before the newest row's first key, or end after the oldest row's position, hide scores
  const int first_full = p.window >= 0 ? max(0, len - 1 - p.window) : 0;
  const int t_lo = first_key / BN, t_hi = (len + BN - 1) / BN;
  const int per_split = (t_hi - t_lo + p.nsplit - 1) / p.nsplit;
  const int t_begin = t_lo + split * per_split, t_end = min(t_hi, t_begin + per_split);

  bf16x8 qf[CB][KK];
  float slope2[CB], m_run[CB], l_run[CB];          // log2-domain running max (same in both halves), per-lane partial sum
  f32x16 oacc[CB][DB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const uint16_t* qp = p.q + b * p.q_sb + hq[cb] * p.q_sh + row[cb] * p.q_st;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[cb][kk] = *(const bf16x8*)(qp + 16 * kk + 8 * w.half);
    slope2[cb] = C::MOD == kModAlibi ? p.alibi_slopes[hq[cb]] * kLog2e : 0.f;
    m_run[cb] = -INFINITY;
    l_run[cb] = 0.f;
#pragma unroll
    for (int d = 0; d < DB; ++d) oacc[cb][d] = W::zero16();
  }
  const float c_scale = p.scale * kLog2e;

  unsigned char* ring = lds_raw + wave * C::WAVE_LDS;
  // Pages of a tile: a tile of 32 keys touches at most four pages (pages hold at least 8 tokens and
  // tiles are aligned to them).  Their table entries are fetched one tile ahead of the direct loads that
  // need them, by vector loads of one address for the whole wave whose values stay untouched in
  // registers until then: the wait for them falls at the top of the next step, where the tile that
  // step computes on has to have landed anyway.  (A consumer right behind the load would wait for every
  // outstanding vector load, the tile just requested included, before the current tile's arithmetic.)
  struct Pages {
    int pg[4];                                     // table entries as loaded, the same in every lane
  };
  auto lookup = [&](int t) __attribute__((always_inline)) -> Pages {
    Pages r;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (p.block_table != nullptr) {
        // first token of the tile's u-th page, clamped into the sequence; never below token 0, although
        // only workgroups that own a tile (so len >= 1) look anything up
        const int j = max(min(t * BN + (u << p.page_shift), len - 1), 0);
        r.pg[u] = p.block_table[(int64_t)b * p.table_stride + (j >> p.page_shift)];
      } else {
        r.pg[u] = b;
      }
    }
    return r;
  };
  // ... made wave-uniform and cut to the cache (an entry outside it is wrong data, never a wild address): this
  // is where the entries are waited for
  auto resolve = [&](const Pages& raw) __attribute__((always_inline)) -> Pages {
    Pages r;
#pragma unroll
    for (int u = 0; u < 4; ++u) r.pg[u] = min(max(__builtin_amdgcn_readfirstlane(raw.pg[u]), 0), p.num_pages - 1);
    return r;
  };
  // all load instructions of tile t (32 keys of K, then of V) into ring stage `stage`; rows past
  // the sequence end repeat its last key (their scores are masked)
  auto load_tile = [&](int t, int stage, const Pages& pages) __attribute__((always_inline)) {
    unsigned char* st = ring + stage * C::STAGE;
    const int tile_page0 = (t * BN) >> p.page_shift;
#pragma unroll
    for (int inst = 0; inst < C::TILE_INSTR; ++inst) {
      const int dst_row = inst * C::RPI + lane / (D / 8);
      const int chunk = (lane % (D / 8)) ^ swz_u<D>(dst_row);
      // the rows of one instruction share a page, so its index is uniform
      const int j_first = max(min(t * BN + inst * C::RPI, len - 1), 0);
      const int j = max(min(t * BN + dst_row, len - 1), 0);
      int64_t page, off;
      if (p.block_table != nullptr) {
        const int u = (j_first >> p.page_shift) - tile_page0;                // 0..3, uniform
        page = u == 0 ? pages.pg[0] : (u == 1 ? pages.pg[1] : (u == 2 ? pages.pg[2] : pages.pg[3]));
        off = j & ((1 << p.page_shift) - 1);
      } else {
        page = b;
        off = j;
      }
      const uint16_t* kr = p.k + page * p.k_sp + off * p.k_st + hk * p.k_sh + chunk * 8;
      const uint16_t* vr = p.v + page * p.v_sp + off * p.v_st + hk * p.v_sh + chunk * 8;
      __builtin_amdgcn_global_load_lds((global_cvoid*)kr, (lds_void*)(st + inst * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((global_cvoid*)vr, (lds_void*)(st + C::TILE + inst * 1024), 16, 0, 0);
    }
  };

  // this wave's tiles: t_begin + wave, + NWV, ...; NSTG - 1 of them in flight ahead of the one in use
  int t_issue = t_begin + wave;
#pragma unroll
  for (int s = 0; s < C::NSTG - 1; ++s) {
    if (t_issue < t_end) load_tile(t_issue, s, resolve(lookup(t_issue)));
    t_issue += C::NWV;
  }
  // pages of the next tile to request (a workgroup without tiles, e.g. of an empty sequence, looks nothing up)
  Pages next_pages = {{0, 0, 0, 0}};
  if (t_begin < t_end) next_pages = lookup(t_issue < t_end ? t_issue : t_begin);
  int stage = 0;
  for (int t = t_begin + wave; t < t_end; t += C::NWV) {
    const int stage_ld = stage == 0 ? C::NSTG - 1 : stage - 1;      // the stage the previous tile used
    const Pages pages_now = resolve(next_pages);
    if (t_issue < t_end) {
      load_tile(t_issue, stage_ld, pages_now);
      wait_vm<(C::NSTG - 1) * C::IPT>();           // everything but the NSTG - 1 younger tiles has landed
    } else {
      wait_vm<0>();
    }
    t_issue += C::NWV;
    if (t_issue < t_end) next_pages = lookup(t_issue);
    const uint32_t base = (uint32_t)(wave * C::WAVE_LDS + stage * C::STAGE);
    uint32_t ra_b[KK], ta_b[DB][2];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) ra_b[kk] = w.ra[kk] + base;
#pragma unroll
    for (int d = 0; d < DB; ++d) {
      ta_b[d][0] = w.ta[d][0] + base;
      ta_b[d][1] = w.ta[d][1] + base;
    }
    const int jb = t * BN + 4 * w.half;            // key of register 0
    const bool partial = t * BN + BN > len - p.T + 1 || t * BN < first_full;     // uniform
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      // scores of the tile's 32 keys for this block's pairs: lane = pair, register r = key 8*(r/4) + 4*half + r%4
      f32x16 s = W::zero16();
      w.template row_stream_g<RowOne<0>, KK, 2>(ra_b, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[cb][decltype(fc)::value], s, 0, 0, 0);
      });
      const int lo_key = p.window >= 0 ? pos[cb] - p.window : 0;
      float x[16];
      float mx = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = jb + 8 * (r >> 2) + (r & 3);
        float a;
        if constexpr (C::MOD == kModSoftcap) {
          const float e = fast_exp2(s[r] * (2.f * c_scale / p.softcap));
          a = fmaf(fast_rcp(e + 1.f), -2.f * p.softcap * kLog2e, p.softcap * kLog2e);
        } else if constexpr (C::MOD == kModAlibi) {
          a = fmaf(s[r], c_scale, -slope2[cb] * (float)(pos[cb] - j));
        } else {
          a = s[r] * c_scale;
        }
        if (partial && (j > pos[cb] || j < lo_key)) a = -INFINITY;
        x[r] = a;
        mx = fmaxf(mx, a);
      }
      mx = half_swap_max(mx);
      // the running max only advances when the tile's max exceeds it by more than 2^8 (P stays
      // bounded by 2^8; l and the final division use the same reference, so nothing changes in real
      // arithmetic): the O rescale becomes a rare, wave-uniform branch
      const float m_new = (mx - m_run[cb] > kLazyMaxLog2) ? mx : m_run[cb];   // false for NaN (-inf - -inf)
      const float m_safe = m_new == -INFINITY ? 0.f : m_new;
      const bool moved = m_new != m_run[cb];
      const float alpha = moved ? fast_exp2(m_run[cb] - m_safe) : 1.f;  // exp2(-inf) = 0 on the first tile
      m_run[cb] = m_new;
      float psum = 0.f;
      uint32_t pw[8];
#pragma unroll
      for (int r2 = 0; r2 < 8; ++r2) {
        const float p0 = fast_exp2(x[2 * r2] - m_safe), p1 = fast_exp2(x[2 * r2 + 1] - m_safe);
        psum += p0 + p1;
        pw[r2] = pack_bf16(p0, p1);
      }
      l_run[cb] = fmaf(l_run[cb], alpha, psum);
      if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
        for (int d = 0; d < DB; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[cb][d][r] *= alpha;
      }
      w.template tr_stream_g<TrOne<C::TILE, DB, ROW>, 2 * DB, 2>(ta_b, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        constexpr int f = decltype(fc)::value, d = f % DB, ks = f / DB;
        const bf16x8 bop = __builtin_bit_cast(
            bf16x8, (i32x4){(int)pw[4 * ks], (int)pw[4 * ks + 1], (int)pw[4 * ks + 2], (int)pw[4 * ks + 3]});
        oacc[cb][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bop, oacc[cb][d], 0, 0, 0);
      });
    }
    stage = stage + 1 == C::NSTG ? 0 : stage + 1;
  }

  // ---- merge the waves (Sec. 3.3 / 3.4 rescale rule), one column block at a time: everyone parks
  // (m, l, O) in its own ring region, wave 0 folds them and writes the split's partial result
  static_assert((DB * 4 + 1) * 64 * 16 <= C::WAVE_LDS, "parking area");
  W::template wait_lds<0>();
#pragma unroll
  for (int cb = 0; cb < CB; ++cb) {
    const float l_wave = half_swap_sum(l_run[cb]);
    float4* park = (float4*)(lds_raw + wave * C::WAVE_LDS) + lane;     // [quad][lane] float4, then (m, l)
    if (cb > 0) __syncthreads();                   // wave 0 has read the previous block's parked values
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4)
        park[(d * 4 + r4) * 64] = make_float4(oacc[cb][d][4 * r4], oacc[cb][d][4 * r4 + 1], oacc[cb][d][4 * r4 + 2], oacc[cb][d][4 * r4 + 3]);
    park[DB * 4 * 64] = make_float4(m_run[cb], l_wave, 0.f, 0.f);
    __syncthreads();
    if (wave != 0) continue;
    float m_all = m_run[cb];
#pragma unroll
    for (int u = 1; u < C::NWV; ++u) {
      const float4* other = (const float4*)(lds_raw + u * C::WAVE_LDS) + lane;
      m_all = fmaxf(m_all, other[DB * 4 * 64].x);
    }
    const float m_safe = m_all == -INFINITY ? 0.f : m_all;
    float l_all = 0.f;
    f32x16 o[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d) o[d] = W::zero16();
#pragma unroll
    for (int u = 0; u < C::NWV; ++u) {
      const float4* other = (const float4*)(lds_raw + u * C::WAVE_LDS) + lane;
      const float4 ml = other[DB * 4 * 64];
      const float wgt = fast_exp2(ml.x - m_safe);                 // 0 for a wave that saw no key
      l_all = fmaf(ml.y, wgt, l_all);
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const float4 q4 = other[(d * 4 + r4) * 64];
          o[d][4 * r4] = fmaf(q4.x, wgt, o[d][4 * r4]);
          o[d][4 * r4 + 1] = fmaf(q4.y, wgt, o[d][4 * r4 + 1]);
          o[d][4 * r4 + 2] = fmaf(q4.z, wgt, o[d][4 * r4 + 2]);
          o[d][4 * r4 + 3] = fmaf(q4.w, wgt, o[d][4 * r4 + 3]);
        }
    }
    if (live[cb] && p.nsplit == 1) {
      // the only split of its sequence: this is the result, no partials and no merge kernel
      const float inv = l_all > 0.f ? 1.f / l_all : 0.f;
      const int64_t ob = b * p.o_sb + hq[cb] * p.o_sh + row[cb] * p.o_st;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int ch = 32 * d + 8 * r4 + 4 * w.half;
          const float x0 = o[d][4 * r4] * inv, x1 = o[d][4 * r4 + 1] * inv, x2 = o[d][4 * r4 + 2] * inv, x3 = o[d][4 * r4 + 3] * inv;
          if (p.out_f32) *(float4*)((float*)p.out + ob + ch) = make_float4(x0, x1, x2, x3);
          else *(uint2*)((uint16_t*)p.out + ob + ch) = make_uint2(pack_bf16(x0, x1), pack_bf16(x2, x3));
        }
      if (w.half == 0 && p.lse != nullptr)
        p.lse[b * p.lse_sb + hq[cb] * p.lse_sh + row[cb] * p.lse_st] = l_all > 0.f ? (m_all + __log2f(l_all)) * kLn2 : -INFINITY;
    } else if (live[cb]) {
      const int64_t slot = (((int64_t)b * p.T + row[cb]) * p.H + hq[cb]) * p.nsplit + split;
      float* po = p.part_o + slot * D;
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          *(float4*)(po + 32 * d + 8 * r4 + 4 * w.half) = make_float4(o[d][4 * r4], o[d][4 * r4 + 1], o[d][4 * r4 + 2], o[d][4 * r4 + 3]);
      if (w.half == 0) *(float2*)(p.part_ml + slot * 2) = make_float2(m_all, l_all);
    }
  }
}

// Merge of the splits of one (sequence, head): out = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M).
// One wave per (sequence, query row, head).  The statistics are read one split per lane (maximum and sum by
// wave reductions); the partial outputs are then accumulated with each lane on its D / 64 channels,
// the weight of split s taken from lane s, several loads in flight (a loop that waited for every
// split's load in turn cost more than the attention itself on a long single sequence).
template <int D>
__global__ void __launch_bounds__(64) decode_combine_kernel(const DecodeParams p) {
  const int bh = blockIdx.x;                       // (b * T + row) * H + h, the order of the partial results
  const int h = bh % p.H, row = (bh / p.H) % p.T, b = bh / p.H / p.T;
  const int lane = threadIdx.x;
  constexpr int CPT = D / 64;
  const float* ml = p.part_ml + (int64_t)bh * p.nsplit * 2;
  float m_all = -INFINITY;
  for (int s = lane; s < p.nsplit; s += 64) m_all = fmaxf(m_all, ml[2 * s]);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) m_all = fmaxf(m_all, __shfl_xor(m_all, o));
  const float m_safe = m_all == -INFINITY ? 0.f : m_all;
  float l_all = 0.f, acc[CPT];
#pragma unroll
  for (int e = 0; e < CPT; ++e) acc[e] = 0.f;
  for (int c = 0; c < p.nsplit; c += 64) {         // 64 splits per round, one per lane
    const int s = c + lane;
    float wgt = 0.f;
    if (s < p.nsplit) {
      wgt = fast_exp2(ml[2 * s] - m_safe);
      l_all = fmaf(ml[2 * s + 1], wgt, l_all);
    }
    const int n = min(64, p.nsplit - c);           // uniform
    const float* po = p.part_o + ((int64_t)bh * p.nsplit + c) * D + lane * CPT;
    for (int u0 = 0; u0 < n; u0 += 8) {            // eight loads in flight; past n: the last split again, weight 0
      float x[8][CPT];
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const int u = min(u0 + k, n - 1);
#pragma unroll
        for (int e = 0; e < CPT; ++e) x[k][e] = po[(int64_t)u * D + e];
      }
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const float wu = __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(wgt), u0 + k));
#pragma unroll
        for (int e = 0; e < CPT; ++e) acc[e] = fmaf(x[k][e], wu, acc[e]);
      }
    }
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) l_all += __shfl_xor(l_all, o);
  const float inv = l_all > 0.f ? 1.f / l_all : 0.f;
  const int64_t o = b * p.o_sb + h * p.o_sh + row * p.o_st + lane * CPT;
#pragma unroll
  for (int e = 0; e < CPT; ++e) {
    if (p.out_f32) ((float*)p.out)[o + e] = acc[e] * inv;
    else ((uint16_t*)p.out)[o + e] = (uint16_t)(pack_bf16(acc[e] * inv, 0.f) & 0xFFFFu);
  }
  if (lane == 0 && p.lse != nullptr)
    p.lse[b * p.lse_sb + h * p.lse_sh + row * p.lse_st] = l_all > 0.f ? (m_all + __log2f(l_all)) * kLn2 : -INFINITY;
}

}  // namespace fl
