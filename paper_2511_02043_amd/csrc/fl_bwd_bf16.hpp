// bf16 backward kernels of the attention variants for gfx950: gradients of the fused forward
// pass (Eq. 3 with the score_mod of Eq. 4 and the masks of the attention listing) with respect
// to Q, K and V, from the saved log-sum-exp -- the training extension the paper's conclusion
// leaves open.  Like the forward pass, nothing of size [Sq, Sk] ever reaches device memory: each
// score tile is recomputed on the matrix cores, turned into probabilities with the saved
// row statistics and consumed at once.
//
//     P  = exp(s - lse)                 s: the transformed, masked score of the forward pass
//     dP = dO V^T
//     dS = P * (dP - delta)             delta_i = sum_c dO_ic O_ic  (= rowsum(P * dP))
//     dZ = dS * (1 - tanh^2)            soft-cap only
//     dV = P^T dO,   dK = scale * dZ^T Q,   dQ = scale * dZ K
//
// Two passes, both without atomics (bitwise reproducible results):
//   * bwd_dq_kernel: a workgroup owns 128 query rows (one per lane, as in the forward kernel)
//     and walks the key tiles; per tile S^T = K Q^T and dP^T = V dO^T land in the 32x32
//     accumulator layout with the query in the lane, dS^T rounded to bf16 is the B operand of
//     dQ^T += K^T dS^T, whose A operand is the same K tile read through the transposing LDS load.
//   * dK / dV: a workgroup owns 128 keys (one per lane) and walks the query tiles of the query
//     heads of its group; S = Q K^T and dP = dO V^T have the key in the lane and the query row in
//     the register index, so P and dS are the B operands of dV^T += dO^T P and dK^T += Q^T dS with
//     dO^T / Q^T read transposed from LDS.  bwd_dkdv_kernel (D = 64) does all of it in every wave,
//     software-pipelined over 32-row blocks; bwd_dkdv_ws_kernel (D = 128, where one wave's
//     accumulators fill a SIMD's registers) splits it over two specialised waves per SIMD.
//     With grouped heads and few workgroups, the group's heads are cut over several workgroups
//     whose fp32 partials bwd_reduce_kv_kernel adds in a fixed order.
// A small pre-pass writes delta and the log2-scaled lse (+inf for rows without a visible key, so
// that their probabilities come out as exactly 0).
//
// LDS tiles are row-major [rows][D] bf16 with one 16-byte-chunk swizzle that serves both access
// patterns without bank conflicts: the row read (32 consecutive rows, one chunk per lane) and
// the transposing read (4 rows x 4 chunks per 32 lanes).
#pragma once
#include "fl_kernel_bf16.hpp"

namespace fl {

struct BwdParams {
  View q, k, v, o, dout;           // inputs  [B, G, H | Hkv, S, D]
  View dq, dk, dv;                 // outputs (ptr is written)
  const float* lse;                // [B, G, H, Sq] from the forward pass
  int64_t lse_sb, lse_sg, lse_sh;
  float* delta;                    // workspace [B, G, H, Sq]: rowsum(dO * O)
  float* lse2;                     // workspace [B, G, H, Sq]: lse * log2(e), +inf for dead rows
  const float* alibi_slopes;
  const int32_t* q_doc;            // [B, Sq]
  const int32_t* kv_doc;           // [B, Sk]
  int2* q_sum;                     // (min, max) document id per block of 32 rows / keys
  int2* kv_sum;
  int32_t B, G, H, Hkv, Sq, Sk;
  int32_t window, prefix;
  float scale, softcap;
  int32_t dq_f32, dkv_f32;         // 1: that output is float, 0: bf16
  int32_t n_qtiles, n_ktiles;      // workgroups per (b, g, h) of the dQ kernel / per (b, g, hkv) of the dK/dV kernel
  int32_t order_q, order_k;        // 1: XCD-aware workgroup order (whole (b, g, h) problems per XCD) in that kernel
  int32_t hsplit;                  // dK/dV kernel: the query heads of a group are cut into hsplit subsets, one workgroup each
  float* part_dk;                  // hsplit > 1: fp32 partial sums [hsplit][B, G, Hkv, Sk, D], summed by bwd_reduce_kv_kernel
  float* part_dv;
  BiasView bias[2];                // the forward pass's additive biases (kernels built with NBIAS > 0), bf16
  int32_t q_off;                   // query row i sits at sequence position i + q_off (positional masks, ALiBi); >= 0
  const void* user_aux[4];         // run-time compiled variants: the caller's device arrays that the expressions read
  uint16_t* ds_stage;              // bias gradients wanted: dS of every score, bf16 dense [B, G, H, Sq, Sk]; the host sums it
                                   // over the axes each bias broadcasts along afterwards (null: not wanted)
};

// chunk swizzle of a tile row (see the header comment): an XOR on the 16-byte chunk index that
// depends on row % 16 only.
template <int D>
__device__ __forceinline__ int swz_u(int r) {
  if constexpr (D == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
  else return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
}

// Query rows [lo, hi) that can see any key in [j_lo, j_hi] under the positional masks.
__device__ __forceinline__ void query_range(const uint32_t MASK, int j_lo, int j_hi, int Sq, int window, int prefix,
                                            int& lo, int& hi) {
  lo = 0;
  hi = Sq;
  if ((MASK & kMaskPrefix) != 0) {
    if (j_lo >= prefix) lo = j_lo;
  } else if ((MASK & (kMaskCausal | kMaskWindow)) != 0) {
    lo = j_lo;
  }
  if ((MASK & kMaskWindow) != 0) hi = min(Sq, j_hi + window + 1);
  lo = min(lo, hi);
}

template <int D_, int MOD_, uint32_t MASK_, int BN_, int WPE_, int NBIAS_ = 0>
struct BwdCfg {
  static constexpr int D = D_, MOD = MOD_, BN = BN_, WPE = WPE_, NBIAS = NBIAS_;
  static constexpr uint32_t MASK = MASK_;
  static constexpr int NW = 4, NT = NW * 64;
  static constexpr int BM = NW * 32;               // rows (dQ kernel) or keys (dK/dV kernel) per workgroup
  static constexpr int NB = BN / 32;               // 32-row blocks of a streamed tile
  static constexpr int KK = D / 16;                // k-steps over the head dim
  static constexpr int DB = D / 32;                // 32-channel blocks of the head dim
  static constexpr int ROW = D * 2;                // bytes of a tile row
  static constexpr int TILE = BN * ROW;            // bytes of one streamed tile
  static constexpr int STAT = BN * 4;              // bytes of one per-row statistic of a tile (dK/dV kernel)
  static constexpr int STAGE_DQ = 2 * TILE;        // K, V
  static constexpr int STAGE_KV = 2 * TILE + 2 * STAT;   // Q, dO, lse2, delta
  static constexpr int TILE_INSTR = TILE / 1024;   // 64-lane x 16-byte direct loads per tile
  static constexpr int RPI = 1024 / ROW;           // tile rows per load instruction
  static constexpr int GR = WPE == 1 ? 4 : 2;      // dK/dV pipeline: row fragments read ahead (a lone wave per SIMD hides LDS latency itself)
  static constexpr int GT = WPE == 1 ? 4 : 2;      // dK/dV pipeline: transposed fragments read ahead
  static_assert(D == 64 || D == 128, "head dims of the backward kernels");
  static_assert(TILE_INSTR % NW == 0, "every wave issues the same number of loads");
  static_assert((NW * RPI) % 16 == 0, "a lane's destination row keeps its residue mod 16");
};

// Fragment -> LDS offset maps of the pipelined loops.  RowPair: KK row fragments of the block at
// OFF0, then KK of the block at OFF1.  TrQuad: DB transposed fragments each of (block at OFF0,
// rows 0..15), (block at OFF1, rows 0..15), (OFF0, rows 16..31), (OFF1, rows 16..31).
template <int OFF0, int OFF1, int KK>
struct RowPair {
  static constexpr int off(int f) { return f < KK ? OFF0 : OFF1; }
};
template <int OFF0, int OFF1, int DB, int ROW>
struct TrQuad {
  static constexpr int off(int f) { return (((f / DB) % 2) == 0 ? OFF0 : OFF1) + ((f / DB) / 2) * 16 * ROW; }
};

template <int OFF>
struct RowOne {                                    // KK row fragments of the block at OFF
  static constexpr int off(int) { return OFF; }
};
template <int OFF, int DB, int ROW>
struct TrOne {                                     // DB transposed fragments of rows 0..15, then DB of rows 16..31
  static constexpr int off(int f) { return OFF + (f / DB) * 16 * ROW; }
};

template <class C>
struct BwdWave {
  static constexpr int D = C::D, KK = C::KK, DB = C::DB, ROW = C::ROW;
  static constexpr uint32_t MASK = C::MASK;

  int lane, half, col;
  uint32_t ra[C::KK];              // per-lane byte offset of the row-read fragment of k-step kk (row block 0)
  uint32_t ta[C::DB][2];           // per-lane byte offsets of the transposing read of channel block d (rows +0 / +8)

  __device__ __forceinline__ void init(int lane_) {
    lane = lane_;
    half = lane >> 5;
    col = lane & 31;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) ra[kk] = col * ROW + ((2 * kk + half) ^ swz_u<D>(col)) * 16;
    const int s16 = lane & 15;
    const int r0 = 4 * half + (s16 >> 2);          // row this lane addresses in the transposing read
#pragma unroll
    for (int d = 0; d < DB; ++d) {
      const int ch = 32 * d + 16 * ((lane >> 4) & 1) + 4 * (s16 & 3);   // first of its 4 channels
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int r = r0 + 8 * u;
        ta[d][u] = r * ROW + ((ch >> 3) ^ swz_u<D>(r)) * 16 + (ch & 7) * 2;
      }
    }
  }

  static __device__ __forceinline__ f32x16 zero16() {
    return f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  }

  // LDS reads are issued by hand with explicit lgkmcnt waits (LDS returns in order): the compiler
  // then sees no LDS read in the loop and cannot tie one to the direct global->LDS loads of the
  // next tile that are in flight.
  template <int OFF>
  static __device__ __forceinline__ void read_b128(i32x4& dst, uint32_t addr) {
    if constexpr (OFF <= 65535) {
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
    } else {
      const uint32_t a = addr + (uint32_t)OFF;
      asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(a) : "memory");
    }
  }
  template <int OFF>
  static __device__ __forceinline__ void read_tr(i32x2& dst, uint32_t addr) {
    if constexpr (OFF <= 65535) {
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
    } else {
      const uint32_t a = addr + (uint32_t)OFF;
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(dst) : "v"(a) : "memory");
    }
  }
  template <int OFF>
  static __device__ __forceinline__ void write_b128(uint32_t addr, i32x4 v) {
    asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFF) : "memory");
  }
  template <int N>
  static __device__ __forceinline__ void wait_lds() {
    static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(N) : "memory");
    __builtin_amdgcn_sched_barrier(0);
  }

  // KK row-read fragments (A operand, 32 tile rows x 16 channels each) of the 32-row block at
  // LDS byte offset OFF, read two ahead; body(kk, fragment).
  template <int OFF, class Body>
  __device__ __forceinline__ void row_stream(Body&& body) const {
    constexpr int G = 2, NG = KK / G;
    i32x4 fr[KK];
    static_for<0, G>([&](auto f) __attribute__((always_inline)) { read_b128<OFF>(fr[f], ra[f]); });
    static_for<0, NG>([&](auto gc) __attribute__((always_inline)) {
      constexpr int g = gc;
      if constexpr (g + 1 < NG)
        static_for<(g + 1) * G, (g + 2) * G>([&](auto f) __attribute__((always_inline)) { read_b128<OFF>(fr[f], ra[f]); });
      wait_lds<(g + 1 < NG) ? G : 0>();
      static_for<g * G, (g + 1) * G>([&](auto f) __attribute__((always_inline)) { body(f, __builtin_bit_cast(bf16x8, fr[f])); });
    });
  }
  // 2 * DB transposed fragments (A operand, 32 channels x 16 tile rows each) of the 32-row block
  // at OFF: fragment f = ks * DB + d covers rows 16 * ks .. + 15 and channels 32 * d .. + 31, with
  // the contraction index order of the accumulator registers (element e <-> row 8*(e/4) + 4*half + e%4).
  template <int OFF, class Body>
  __device__ __forceinline__ void tr_stream(Body&& body) const {
    constexpr int NF = 2 * DB, G = 2, NG = NF / G;
    i32x2 lo[NF], hi[NF];
    static_for<0, G>([&](auto f) __attribute__((always_inline)) {
      read_tr<OFF + (f / DB) * 16 * ROW>(lo[f], ta[f % DB][0]);
      read_tr<OFF + (f / DB) * 16 * ROW>(hi[f], ta[f % DB][1]);
    });
    static_for<0, NG>([&](auto gc) __attribute__((always_inline)) {
      constexpr int g = gc;
      if constexpr (g + 1 < NG)
        static_for<(g + 1) * G, (g + 2) * G>([&](auto f) __attribute__((always_inline)) {
          read_tr<OFF + (f / DB) * 16 * ROW>(lo[f], ta[f % DB][0]);
          read_tr<OFF + (f / DB) * 16 * ROW>(hi[f], ta[f % DB][1]);
        });
      wait_lds<(g + 1 < NG) ? 2 * G : 0>();
      static_for<g * G, (g + 1) * G>([&](auto f) __attribute__((always_inline)) {
        body(f, __builtin_bit_cast(bf16x8, (i32x4){lo[f][0], lo[f][1], hi[f][0], hi[f][1]}));
      });
    });
  }

  // Generic forms for the software-pipelined loops: O::off(f) is the LDS byte offset of fragment
  // f (a compile-time function), fragments are read G ahead, body(f, fragment) runs in order.
  template <class O, int NF, int G, class Body>
  __device__ __forceinline__ void row_stream_g(const uint32_t (&ra)[C::KK], Body&& body) const {
    constexpr int NG = NF / G;
    static_assert(NF % G == 0 && G <= 15, "fragment groups");
    i32x4 fr[NF];
    static_for<0, G>([&](auto f) __attribute__((always_inline)) { read_b128<O::off(f)>(fr[f], ra[f % KK]); });
    static_for<0, NG>([&](auto gc) __attribute__((always_inline)) {
      constexpr int g = gc;
      if constexpr (g + 1 < NG)
        static_for<(g + 1) * G, (g + 2) * G>([&](auto f) __attribute__((always_inline)) { read_b128<O::off(f)>(fr[f], ra[f % KK]); });
      wait_lds<(g + 1 < NG) ? G : 0>();
      static_for<g * G, (g + 1) * G>([&](auto f) __attribute__((always_inline)) { body(f, __builtin_bit_cast(bf16x8, fr[f])); });
    });
  }
  template <class O, int NF, int G, class Body>
  __device__ __forceinline__ void tr_stream_g(const uint32_t (&ta)[C::DB][2], Body&& body) const {
    constexpr int NG = NF / G;
    static_assert(NF % G == 0 && 2 * G <= 15, "fragment groups");
    i32x2 lo[NF], hi[NF];
    static_for<0, G>([&](auto f) __attribute__((always_inline)) {
      read_tr<O::off(f)>(lo[f], ta[f % DB][0]);
      read_tr<O::off(f)>(hi[f], ta[f % DB][1]);
    });
    static_for<0, NG>([&](auto gc) __attribute__((always_inline)) {
      constexpr int g = gc;
      if constexpr (g + 1 < NG)
        static_for<(g + 1) * G, (g + 2) * G>([&](auto f) __attribute__((always_inline)) {
          read_tr<O::off(f)>(lo[f], ta[f % DB][0]);
          read_tr<O::off(f)>(hi[f], ta[f % DB][1]);
        });
      wait_lds<(g + 1 < NG) ? 2 * G : 0>();
      static_for<g * G, (g + 1) * G>([&](auto f) __attribute__((always_inline)) {
        body(f, __builtin_bit_cast(bf16x8, (i32x4){lo[f][0], lo[f][1], hi[f][0], hi[f][1]}));
      });
    });
  }
};

// One 64-lane x 16-byte direct load instruction `inst` of a [rows][D] tile whose row 0 is at
// `base` (row stride `row_bytes`); rows at or past n_valid are replaced by row n_valid - 1.
template <class C>
__device__ __forceinline__ void tile_load_instr(const unsigned char* base, int64_t row_bytes, int n_valid, int inst,
                                                int lane, unsigned char* lds_tile) {
  const int dst_row = inst * C::RPI + lane / (C::D / 8);
  const int chunk = (lane % (C::D / 8)) ^ swz_u<C::D>(dst_row);
  const int row = dst_row < n_valid ? dst_row : n_valid - 1;
  lds_void* dst = (lds_void*)(lds_tile + inst * 1024);
  __builtin_amdgcn_global_load_lds((global_cvoid*)(base + (int64_t)row * row_bytes + chunk * 16), dst, 16, 0, 0);
}

// The score pipeline of the forward pass replayed on one raw dot product x = <q_i, k_j>:
// returns the log2-domain exponent argument a (P = exp2(a)) and the soft-cap derivative factor.
//   rel = i - j;  slope2 = slope * log2(e);  lse2 = lse * log2(e).
template <int MOD>
__device__ __forceinline__ float replay_score(float x, float c_scale, float lse2, float softcap, float slope2,
                                              float rel, float& fac) {
  fac = 1.f;
  if constexpr (MOD == kModSoftcap) {
    const float e = fast_exp2(x * (2.f * c_scale / softcap));     // exp(2 z / cap)
    const float t = fmaf(fast_rcp(e + 1.f), -2.f, 1.f);           // tanh(z / cap)
    fac = fmaf(-t, t, 1.f);
    return fmaf(t, softcap * kLog2e, -lse2);
  } else if constexpr (MOD == kModAlibi) {
    return fmaf(x, c_scale, -lse2) - slope2 * fabsf(rel);
  } else {
    return fmaf(x, c_scale, -lse2);
  }
}

template <uint32_t MASK>
__device__ __forceinline__ bool hidden(int i, int j, int Sq, int Sk, int q_off, int window, int prefix, int qdoc, int kdoc) {
  return i >= Sq || j >= Sk || is_masked(MASK, i + q_off, j, window, prefix, qdoc, kdoc);
}

// Run-time compiled variants (kModCustom / kMaskCustom): the caller's expressions see the sizes of the call and their
// captured arrays through the forward pass's parameter block; this is the part of it they read.
__device__ __forceinline__ FwdParams user_context(const BwdParams& p) {
  FwdParams u;
  u.B = p.B; u.G = p.G; u.H = p.H; u.Sq = p.Sq; u.Sk = p.Sk;
#pragma unroll
  for (int n = 0; n < 4; ++n) u.user_aux[n] = p.user_aux[n];
  return u;
}
// The score pipeline of a compiled score_mod replayed on the raw dot product x of (i, j) (valid indices): exponent
// argument and derivative factor, as replay_score.
template <int MOD>
__device__ __forceinline__ float replay_user(float x, const BwdParams& p, const FwdParams& u, float lse2, int b, int g, int h,
                                             int i, int j, float& fac) {
  const int ic = i < p.Sq ? i : p.Sq - 1, jc = j < p.Sk ? j : p.Sk - 1;
  const float s = x * p.scale;
  fac = fl_user_score_mod_grad(s, b, g, h, ic + p.q_off, jc, u);
  return fmaf(fl_user_score_mod(s, b, g, h, ic + p.q_off, jc, u), kLog2e, -lse2);
}
// hidden() with the compiled mask expression on top (evaluated on valid indices only)
template <uint32_t MASK>
__device__ __forceinline__ bool hidden_user(int i, int j, const BwdParams& p, const FwdParams& u, int b, int g, int h, int qdoc,
                                            int kdoc) {
  if (hidden<MASK>(i, j, p.Sq, p.Sk, p.q_off, p.window, p.prefix, qdoc, kdoc)) return true;
  if constexpr ((MASK & kMaskCustom) != 0) return fl_user_mask(b, g, h, i + p.q_off, j, u);
  return false;
}

// Offsets of the (b, g, h) slice of each bias / bias gradient (elements).
template <int NBIAS>
struct BiasHead {
  int64_t off[NBIAS > 0 ? NBIAS : 1];
  __device__ __forceinline__ void set(const BwdParams& p, int b, int g, int h) {
#pragma unroll
    for (int n = 0; n < NBIAS; ++n) off[n] = b * p.bias[n].sb + g * p.bias[n].sg + h * p.bias[n].sh;
  }
  // can four consecutive keys of a row be fetched with one 8-byte load?  (uniform)
  __device__ __forceinline__ bool rows_vec4(const BwdParams& p) const {
    bool ok = true;
#pragma unroll
    for (int n = 0; n < NBIAS; ++n) {
      const BiasView& v = p.bias[n];
      ok = ok && v.sj == 1 && ((uint64_t)v.ptr) % 8 == 0 && ((v.sb | v.sg | v.sh | v.si) & 3) == 0;
    }
    return ok;
  }
  // the four bf16 values of keys j .. j + 3 of row i of bias n, as loaded (j a multiple of 4, rows_vec4())
  __device__ __forceinline__ uint2 raw4(const BwdParams& p, int n, int i, int j) const {
    return *(const uint2*)((const uint16_t*)p.bias[n].ptr + off[n] + (int64_t)i * p.bias[n].si + j);
  }
  __device__ __forceinline__ uint16_t raw1(const BwdParams& p, int n, int i, int j) const {
    return ((const uint16_t*)p.bias[n].ptr)[off[n] + (int64_t)i * p.bias[n].si + (int64_t)j * p.bias[n].sj];
  }
  // sum of the biases of score (i, j) in log2 units; i, j are valid indices
  __device__ __forceinline__ float value(const BwdParams& p, int i, int j) const {
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < NBIAS; ++n)
      s += bf16_to_f32(((const uint16_t*)p.bias[n].ptr)[off[n] + (int64_t)i * p.bias[n].si + (int64_t)j * p.bias[n].sj]);
    return s * kLog2e;
  }
};

// Four consecutive channels of a dK or dV row: to the output tensor, or (grouped-query heads cut
// over several workgroups) to this workgroup's fp32 partial.
__device__ __forceinline__ void store_kv_grad(const BwdParams& p, const View& out, float* part, int split, int b, int g,
                                              int hk, int j, int ch, int D, float x0, float x1, float x2, float x3) {
  if (p.hsplit > 1) {
    const int64_t row = ((((int64_t)split * p.B + b) * p.G + g) * p.Hkv + hk) * p.Sk + j;
    *(float4*)(part + row * D + ch) = make_float4(x0, x1, x2, x3);
  } else {
    const int64_t row = b * out.sb + g * out.sg + hk * out.sh + (int64_t)j * out.ss;
    if (p.dkv_f32) *(float4*)((float*)out.ptr + row + ch) = make_float4(x0, x1, x2, x3);
    else *(uint2*)((uint16_t*)out.ptr + row + ch) = make_uint2(pack_bf16(x0, x1), pack_bf16(x2, x3));
  }
}

// Sum of the hsplit partials of dK and dV, in a fixed order (reproducible), written in the output dtype.
template <int D>
__global__ void __launch_bounds__(256) bwd_reduce_kv_kernel(const BwdParams p) {
  constexpr int cpr = D / 4;                       // float4 chunks per row
  const int64_t rows = (int64_t)p.B * p.G * p.Hkv * p.Sk;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * cpr) return;
  const int64_t row = idx / cpr;
  const int ch = (int)(idx % cpr) * 4;
  const int j = (int)(row % p.Sk);
  const int hk = (int)((row / p.Sk) % p.Hkv);
  const int g = (int)((row / ((int64_t)p.Sk * p.Hkv)) % p.G);
  const int b = (int)(row / ((int64_t)p.Sk * p.Hkv * p.G));
  float4 k = make_float4(0.f, 0.f, 0.f, 0.f), v = k;
  for (int s = 0; s < p.hsplit; ++s) {
    const float4 a = *(const float4*)(p.part_dk + ((int64_t)s * rows + row) * D + ch);
    const float4 c = *(const float4*)(p.part_dv + ((int64_t)s * rows + row) * D + ch);
    k.x += a.x; k.y += a.y; k.z += a.z; k.w += a.w;
    v.x += c.x; v.y += c.y; v.z += c.z; v.w += c.w;
  }
  const int64_t krow = b * p.dk.sb + g * p.dk.sg + hk * p.dk.sh + (int64_t)j * p.dk.ss;
  const int64_t vrow = b * p.dv.sb + g * p.dv.sg + hk * p.dv.sh + (int64_t)j * p.dv.ss;
  if (p.dkv_f32) {
    *(float4*)((float*)p.dk.ptr + krow + ch) = k;
    *(float4*)((float*)p.dv.ptr + vrow + ch) = v;
  } else {
    *(uint2*)((uint16_t*)p.dk.ptr + krow + ch) = make_uint2(pack_bf16(k.x, k.y), pack_bf16(k.z, k.w));
    *(uint2*)((uint16_t*)p.dv.ptr + vrow + ch) = make_uint2(pack_bf16(v.x, v.y), pack_bf16(v.z, v.w));
  }
}

// ------------------------------------------------------------------------------------------------
// pre-pass: delta = rowsum(dO * O), lse2 = lse * log2(e) (+inf where lse = -inf)
// ------------------------------------------------------------------------------------------------
template <int DV>
__global__ void __launch_bounds__(256) bwd_prep_kernel(const BwdParams p) {
  constexpr int LPR = DV / 8;                      // lanes per row, 16 bytes each
  const int64_t rows = (int64_t)p.B * p.G * p.H * p.Sq;
  const int64_t row = ((int64_t)blockIdx.x * 256 + threadIdx.x) / LPR;
  const int part = threadIdx.x % LPR;
  const int64_t rc = row < rows ? row : rows - 1;
  const int i = (int)(rc % p.Sq);
  const int h = (int)((rc / p.Sq) % p.H);
  const int g = (int)((rc / ((int64_t)p.Sq * p.H)) % p.G);
  const int b = (int)(rc / ((int64_t)p.Sq * p.H * p.G));
  const uint16_t* op = (const uint16_t*)p.o.ptr + b * p.o.sb + g * p.o.sg + h * p.o.sh + (int64_t)i * p.o.ss + 8 * part;
  const uint16_t* dp = (const uint16_t*)p.dout.ptr + b * p.dout.sb + g * p.dout.sg + h * p.dout.sh + (int64_t)i * p.dout.ss + 8 * part;
  const uint4 ov = *(const uint4*)op, dv = *(const uint4*)dp;
  const uint32_t ow[4] = {ov.x, ov.y, ov.z, ov.w}, dw[4] = {dv.x, dv.y, dv.z, dv.w};
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    s = fmaf(__uint_as_float(ow[e] << 16), __uint_as_float(dw[e] << 16), s);
    s = fmaf(__uint_as_float(ow[e] & 0xFFFF0000u), __uint_as_float(dw[e] & 0xFFFF0000u), s);
  }
#pragma unroll
  for (int o = LPR / 2; o >= 1; o >>= 1) s += __shfl_xor(s, o);
  if (part == 0 && row < rows) {
    p.delta[row] = s;
    const float l = p.lse[b * p.lse_sb + g * p.lse_sg + h * p.lse_sh + i];
    p.lse2[row] = l == -INFINITY ? INFINITY : l * kLog2e;
  }
}

// ------------------------------------------------------------------------------------------------
// dQ
// ------------------------------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT) __attribute__((amdgpu_waves_per_eu(C::WPE, C::WPE)))
bwd_dq_kernel(const BwdParams p) {
  constexpr int D = C::D, BN = C::BN, NB = C::NB, KK = C::KK, DB = C::DB, ROW = C::ROW;
  constexpr uint32_t MASK = C::MASK;
  constexpr uint32_t POS = MASK & ~kMaskDoc;
  typedef BwdWave<C> W;
#ifdef FL_LDS_STATIC   // instantiated at run time: the size is part of the code object (a launch through the module API
                       // cannot ask for more than 64 KiB of dynamic LDS)
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[2 * C::STAGE_DQ];
#else
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
#endif

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  W w;
  w.init(tid & 63);
  const int lane = w.lane;

  // grid decode: longest q-tiles (under a causal mask) first
  const int nq = p.n_qtiles;
  int qt, bh;
  if (p.order_q == 1) {
    // consecutive workgroup ids go round-robin to the 8 XCDs: give each XCD whole heads, so that a
    // head's K / V tiles stay in one L2 (the host checks that the head count is a multiple of 8)
    const int idx = blockIdx.x >> 3;
    bh = (idx / nq) * 8 + (blockIdx.x & 7);
    qt = nq - 1 - idx % nq;
  } else {
    qt = nq - 1 - (int)(blockIdx.x % nq);
    bh = blockIdx.x / nq;
  }
  const int h = bh % p.H, g = (bh / p.H) % p.G, b = bh / (p.H * p.G);
  const int hk = h / (p.H / p.Hkv);
  const FwdParams uctx = user_context(p);          // what a compiled variant's expressions read (unused otherwise)
  const int i0 = qt * C::BM, iw = i0 + 32 * wave;
  const int i = iw + w.col, ic = i < p.Sq ? i : p.Sq - 1;
  const int64_t srow = ((int64_t)(b * p.G + g) * p.H + h) * p.Sq + ic;

  // per-lane operands: Q and dO rows as B fragments, row statistics
  bf16x8 qf[KK], dof[KK];
  {
    const uint16_t* qp = (const uint16_t*)p.q.ptr + b * p.q.sb + g * p.q.sg + h * p.q.sh + (int64_t)ic * p.q.ss;
    const uint16_t* dp = (const uint16_t*)p.dout.ptr + b * p.dout.sb + g * p.dout.sg + h * p.dout.sh + (int64_t)ic * p.dout.ss;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qf[kk] = *(const bf16x8*)(qp + 16 * kk + 8 * w.half);
      dof[kk] = *(const bf16x8*)(dp + 16 * kk + 8 * w.half);
    }
  }
  const float lse2 = p.lse2[srow], delta = p.delta[srow];
  const float c_scale = p.scale * kLog2e;
  const float slope2 = C::MOD == kModAlibi ? p.alibi_slopes[h] * kLog2e : 0.f;
  int qdoc = 0;
  if constexpr ((MASK & kMaskDoc) != 0) qdoc = p.q_doc[(int64_t)b * p.Sq + ic];
  BiasHead<C::NBIAS> bh_;
  bh_.set(p, b, g, h);
  const bool bias_vec4 = C::NBIAS > 0 && bh_.rows_vec4(p);

  f32x16 acc[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) acc[d] = W::zero16();

  // visible key range and tile skipping
  const int i_last = (i0 + C::BM < p.Sq ? i0 + C::BM : p.Sq) - 1;
  int k_lo, k_hi;
  key_range(MASK, i0 + p.q_off, i_last + p.q_off, p.Sk, p.window, p.prefix, k_lo, k_hi);   // rows by their positions
  const int t_lo = k_lo / BN, t_hi = (k_hi + BN - 1) / BN;
  const int nks = (p.Sk + kSumBlock - 1) / kSumBlock;
  int2 qs_wg = make_int2(0, 0);
  if constexpr ((MASK & kMaskDoc) != 0) {
    const int nqs = (p.Sq + kSumBlock - 1) / kSumBlock;
    const int2* qsum = p.q_sum + (int64_t)b * nqs;
    qs_wg = qsum[i0 / kSumBlock];
    for (int u = 1; u < C::BM / kSumBlock; ++u)
      if (i0 / kSumBlock + u < nqs) {
        const int2 t = qsum[i0 / kSumBlock + u];
        qs_wg.x = min(qs_wg.x, t.x);
        qs_wg.y = max(qs_wg.y, t.y);
      }
  }
  // does key tile t hold anything visible to the workgroup's rows?  (document-id summaries)
  auto tile_visible = [&](int t) __attribute__((always_inline)) -> bool {
    const int2* ksum = p.kv_sum + (int64_t)b * nks;
    int2 ks = ksum[min(t * NB, nks - 1)];
    for (int u = 1; u < NB; ++u)
      if (t * NB + u < nks) {
        const int2 x = ksum[t * NB + u];
        ks.x = min(ks.x, x.x);
        ks.y = max(ks.y, x.y);
      }
    return classify_block(MASK, i0 + p.q_off, i_last + p.q_off, t * BN, t * BN + BN - 1, p.Sk, p.window, p.prefix, qs_wg, ks) != kSkip;
  };
  auto next_tile = [&](int t) __attribute__((always_inline)) -> int {
    if constexpr ((MASK & kMaskDoc) != 0) {
      if (t < t_hi && !tile_visible(t)) {            // a run of hidden tiles: 64 per round, one per lane
        ++t;
        while (t < t_hi) {
          const int tt = t + lane;
          const unsigned long long found = __builtin_amdgcn_ballot_w64(tt < t_hi && tile_visible(tt));
          if (found != 0) {
            t += __builtin_ctzll(found);
            break;
          }
          t += 64;
        }
        t = __builtin_amdgcn_readfirstlane(t < t_hi ? t : t_hi);
      }
    }
    return t;
  };

  const unsigned char* kbase = (const unsigned char*)((const uint16_t*)p.k.ptr + b * p.k.sb + g * p.k.sg + hk * p.k.sh);
  const unsigned char* vbase = (const unsigned char*)((const uint16_t*)p.v.ptr + b * p.v.sb + g * p.v.sg + hk * p.v.sh);
  const int64_t kss = p.k.ss * 2, vss = p.v.ss * 2;
  auto load_tile = [&](int t, int stage) __attribute__((always_inline)) {
    const int nvalid = min(BN, p.Sk - t * BN);
    unsigned char* st = lds_raw + stage * C::STAGE_DQ;
#pragma unroll
    for (int u = 0; u < C::TILE_INSTR / C::NW; ++u) {
      tile_load_instr<C>(kbase + (int64_t)(t * BN) * kss, kss, nvalid, wave + u * C::NW, lane, st);
      tile_load_instr<C>(vbase + (int64_t)(t * BN) * vss, vss, nvalid, wave + u * C::NW, lane, st + C::TILE);
    }
  };

  // (tn: the tile to request into the other stage while this one is worked on; with biases its loads are issued behind
  // the first block's bias loads, so that waiting for those -- vector loads return in order -- leaves them in flight)
  auto compute = [&](auto stage_c, int t, int tn) __attribute__((always_inline)) {
    constexpr int ST = decltype(stage_c)::value * C::STAGE_DQ;
    if constexpr (C::NBIAS == 0) load_tile(tn, 1 - decltype(stage_c)::value);
    const int j0 = t * BN;
    static_for<0, NB>([&](auto nbc) __attribute__((always_inline)) {
      constexpr int nb = decltype(nbc)::value;
      // the wave's 32 rows against this block's 32 keys under the positional masks (uniform)
      const int cls = classify_block(POS, iw + p.q_off, iw + 31 + p.q_off, j0 + 32 * nb, j0 + 32 * nb + 31, p.Sk, p.window, p.prefix,
                                     make_int2(0, 0), make_int2(0, 0));
      if (cls == kSkip) {                          // nothing visible: dS = 0
        if constexpr (C::NBIAS > 0 && nb == 0) load_tile(tn, 1 - decltype(stage_c)::value);
        return;
      }
      const bool need_mask = (MASK & (kMaskDoc | kMaskCustom)) != 0 || iw + 31 >= p.Sq || cls != kFull;
      // This lane's bias values of the block: requested before the matrix work and left untouched until after it (a
      // conversion right here would put the wait for them, and for the tile loads issued before them, in front of the
      // MFMAs); four keys per load where the rows allow it.
      constexpr int NBR = C::NBIAS > 0 ? C::NBIAS : 1;
      uint2 bq[NBR][4];
      uint16_t b1[NBR][16];
      const bool bvec = C::NBIAS > 0 && bias_vec4 && j0 + 32 * nb + 32 <= p.Sk;   // uniform
      if constexpr (C::NBIAS > 0) {
        if (bvec) {
#pragma unroll
          for (int n = 0; n < C::NBIAS; ++n)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) bq[n][q4] = bh_.raw4(p, n, ic, j0 + 32 * nb + 4 * w.half + 8 * q4);
        } else {
#pragma unroll
          for (int n = 0; n < C::NBIAS; ++n)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int jj = j0 + 32 * nb + 4 * w.half + 8 * (r >> 2) + (r & 3);
              b1[n][r] = bh_.raw1(p, n, ic, jj < p.Sk ? jj : p.Sk - 1);
            }
        }
      }
      if constexpr (C::NBIAS > 0 && nb == 0) load_tile(tn, 1 - decltype(stage_c)::value);
      f32x16 s = W::zero16(), dp = W::zero16();
      w.template row_stream<ST + nb * 32 * ROW>([&](auto kk, bf16x8 a) __attribute__((always_inline)) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], s, 0, 0, 0);
      });
      w.template row_stream<ST + C::TILE + nb * 32 * ROW>([&](auto kk, bf16x8 a) __attribute__((always_inline)) {
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dof[kk], dp, 0, 0, 0);
      });
      const int jb = j0 + 32 * nb + 4 * w.half;    // key of register 0
      float bl[C::NBIAS > 0 ? 16 : 1];             // sum of the biases of each score, log2 units
      if constexpr (C::NBIAS > 0) {
        // the first block's values are older than the next tile's loads: all but those have to have landed
        if constexpr (nb == 0) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * (C::TILE_INSTR / C::NW)));
        if (bvec) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float sum = 0.f;
#pragma unroll
            for (int n = 0; n < C::NBIAS; ++n) {
              const uint32_t wd = (r & 2) ? bq[n][r >> 2].y : bq[n][r >> 2].x;
              sum += __uint_as_float((r & 1) ? (wd & 0xFFFF0000u) : (wd << 16));
            }
            bl[r] = sum * kLog2e;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float sum = 0.f;
#pragma unroll
            for (int n = 0; n < C::NBIAS; ++n) sum += bf16_to_f32(b1[n][r]);
            bl[r] = sum * kLog2e;
          }
        }
      }
      int kd[16];
      if constexpr ((MASK & kMaskDoc) != 0) {
        const int32_t* kdoc = p.kv_doc + (int64_t)b * p.Sk;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = jb + 8 * (r >> 2) + (r & 3);
          kd[r] = kdoc[j < p.Sk ? j : p.Sk - 1];
        }
      }
      // dsw: the gradient of the raw scaled score (what dQ contracts with K); dbw: the gradient of the score after the
      // score_mod, which is the bias gradient (biases follow the score_mod) -- the two differ by the soft-cap derivative
      constexpr bool kSplit = C::NBIAS > 0 && C::MOD == kModSoftcap;
      uint32_t dsw[8], dbw[8];                   // (dbw is only written and read when the two differ)
#pragma unroll
      for (int r2 = 0; r2 < 8; ++r2) {
        float dsv[2], dbv[2], pr[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int r = 2 * r2 + e;
          const int j = jb + 8 * (r >> 2) + (r & 3);
          float fac;
          float a;
          if constexpr (C::MOD == kModCustom) a = replay_user<C::MOD>(s[r], p, uctx, lse2, b, g, h, i, j, fac);
          else a = replay_score<C::MOD>(s[r], c_scale, lse2, p.softcap, slope2, (float)(i + p.q_off - j), fac);
          if constexpr (C::NBIAS > 0) a += bl[r];
          pr[e] = fast_exp2(a);
          dbv[e] = dp[r] - delta;
          dsv[e] = (C::MOD == kModSoftcap || C::MOD == kModCustom) ? dbv[e] * fac : dbv[e];
        }
        if (need_mask) {                           // uniform; kept a branch: most tiles need no mask
          asm volatile("");
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int r = 2 * r2 + e;
            const int j = jb + 8 * (r >> 2) + (r & 3);
            if (hidden_user<MASK>(i, j, p, uctx, b, g, h, qdoc, (MASK & kMaskDoc) ? kd[r] : 0)) pr[e] = 0.f;
          }
        }
        dsv[0] *= pr[0];
        dsv[1] *= pr[1];
        dsw[r2] = pack_bf16(dsv[0], dsv[1]);
        if constexpr (kSplit) dbw[r2] = pack_bf16(dbv[0] * pr[0], dbv[1] * pr[1]);
      }
      if constexpr (C::NBIAS > 0) {                // staged for the host's reduction over the axes each bias broadcasts
        // along; registers 4q .. 4q + 3 are the four consecutive keys jb + 8q ..
        auto staged = [&](int n) __attribute__((always_inline)) { return kSplit ? dbw[n] : dsw[n]; };
        if (p.ds_stage != nullptr && i < p.Sq) {
          uint16_t* row = p.ds_stage + (((int64_t)(b * p.G + g) * p.H + h) * p.Sq + i) * p.Sk;
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int j = jb + 8 * q4;
            if ((p.Sk & 3) == 0 && j + 3 < p.Sk) {
              *(uint2*)(row + j) = make_uint2(staged(2 * q4), staged(2 * q4 + 1));
            } else {
#pragma unroll
              for (int u = 0; u < 4; ++u)
                if (j + u < p.Sk) row[j + u] = (uint16_t)(staged(2 * q4 + (u >> 1)) >> (16 * (u & 1)));
            }
          }
        }
      }
      w.template tr_stream<ST + nb * 32 * ROW>([&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        constexpr int f = decltype(fc)::value, d = f % DB, ks = f / DB;
        const bf16x8 bop = __builtin_bit_cast(
            bf16x8, (i32x4){(int)dsw[4 * ks], (int)dsw[4 * ks + 1], (int)dsw[4 * ks + 2], (int)dsw[4 * ks + 3]});
        acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bop, acc[d], 0, 0, 0);
      });
    });
  };

  int t = next_tile(t_lo);
  if (t < t_hi) {
    load_tile(t, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)
    __syncthreads();
    while (true) {
      bool done = false;
      static_for<0, 2>([&](auto sc) __attribute__((always_inline)) {
        if (!done) {
          const int tn = next_tile(t + 1);
          compute(sc, t, tn < t_hi ? tn : t);      // (past the last tile: the current one again, into the stage nobody reads)
          __builtin_amdgcn_s_waitcnt(0x0F70);
          __syncthreads();
          t = tn;
          done = t >= t_hi;
        }
      });
      if (done) break;
    }
  }

  if (i < p.Sq) {
    const int64_t orow = b * p.dq.sb + g * p.dq.sg + h * p.dq.sh + (int64_t)i * p.dq.ss;
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int ch = 32 * d + 8 * r4 + 4 * w.half;
        const float x0 = acc[d][4 * r4] * p.scale, x1 = acc[d][4 * r4 + 1] * p.scale;
        const float x2 = acc[d][4 * r4 + 2] * p.scale, x3 = acc[d][4 * r4 + 3] * p.scale;
        if (p.dq_f32) *(float4*)((float*)p.dq.ptr + orow + ch) = make_float4(x0, x1, x2, x3);
        else *(uint2*)((uint16_t*)p.dq.ptr + orow + ch) = make_uint2(pack_bf16(x0, x1), pack_bf16(x2, x3));
      }
  }
}

// ------------------------------------------------------------------------------------------------
// dK, dV
// ------------------------------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(C::NT) __attribute__((amdgpu_waves_per_eu(C::WPE, C::WPE)))
bwd_dkdv_kernel(const BwdParams p) {
  constexpr int D = C::D, BN = C::BN, NB = C::NB, KK = C::KK, DB = C::DB, ROW = C::ROW;
  constexpr uint32_t MASK = C::MASK;
  constexpr uint32_t POS = MASK & ~kMaskDoc;
  typedef BwdWave<C> W;
#ifdef FL_LDS_STATIC   // instantiated at run time: the size is part of the code object (a launch through the module API
                       // cannot ask for more than 64 KiB of dynamic LDS)
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[3 * C::STAGE_KV];
#else
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
#endif

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  W w;
  w.init(tid & 63);
  const int lane = w.lane;

  // grid decode: key tiles in increasing order (under a causal mask the first ones see the most rows)
  const int nk = p.n_ktiles;
  int kt, bh;
  if (p.order_k == 1) {                            // whole key/value heads per XCD: their Q / dO tiles stay in one L2
    const int idx = blockIdx.x >> 3;
    bh = (idx / nk) * 8 + (blockIdx.x & 7);
    kt = idx % nk;
  } else {
    kt = blockIdx.x % nk;
    bh = blockIdx.x / nk;
  }
  // bh counts (b, g, kv head, subset of the group's query heads)
  const int split = bh % p.hsplit, bhk = bh / p.hsplit;
  const int hk = bhk % p.Hkv, g = (bhk / p.Hkv) % p.G, b = bhk / (p.Hkv * p.G);
  const int group = p.H / p.Hkv / p.hsplit;        // query heads this workgroup sums over
  const int h_first = hk * (p.H / p.Hkv) + split * group;
  const int j0 = kt * C::BM, jw = j0 + 32 * wave;
  const int j = jw + w.col, jc = j < p.Sk ? j : p.Sk - 1;
  const FwdParams uctx = user_context(p);          // what a compiled variant's expressions read (unused otherwise)

  bf16x8 kf[KK], vf[KK];
  {
    const uint16_t* kp = (const uint16_t*)p.k.ptr + b * p.k.sb + g * p.k.sg + hk * p.k.sh + (int64_t)jc * p.k.ss;
    const uint16_t* vp = (const uint16_t*)p.v.ptr + b * p.v.sb + g * p.v.sg + hk * p.v.sh + (int64_t)jc * p.v.ss;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      kf[kk] = *(const bf16x8*)(kp + 16 * kk + 8 * w.half);
      vf[kk] = *(const bf16x8*)(vp + 16 * kk + 8 * w.half);
    }
  }
  const float c_scale = p.scale * kLog2e;
  int kdoc = 0;
  if constexpr ((MASK & kMaskDoc) != 0) kdoc = p.kv_doc[(int64_t)b * p.Sk + jc];

  f32x16 dk[DB], dv[DB];
#pragma unroll
  for (int d = 0; d < DB; ++d) {
    dk[d] = W::zero16();
    dv[d] = W::zero16();
  }

  // query rows that can see the workgroup's keys; q-tile skipping for document masks
  const int j_last = (j0 + C::BM < p.Sk ? j0 + C::BM : p.Sk) - 1;
  int q_lo, q_hi;
  query_range(MASK, j0, j_last, p.Sq + p.q_off, p.window, p.prefix, q_lo, q_hi);   // as positions; row = position - q_off
  q_lo = max(q_lo - p.q_off, 0);
  q_hi = max(q_hi - p.q_off, 0);
  const int t_lo = q_lo / BN, t_hi = (q_hi + BN - 1) / BN;
  const int nt = t_hi - t_lo;                      // q-tiles per head
  const int n_items = nt > 0 ? nt * group : 0;     // (head of the group, q-tile), head-major
  const int nqs = (p.Sq + kSumBlock - 1) / kSumBlock;
  int2 ks_wg = make_int2(0, 0);
  if constexpr ((MASK & kMaskDoc) != 0) {
    const int nks = (p.Sk + kSumBlock - 1) / kSumBlock;
    const int2* ksum = p.kv_sum + (int64_t)b * nks;
    ks_wg = ksum[j0 / kSumBlock];
    for (int u = 1; u < C::BM / kSumBlock; ++u)
      if (j0 / kSumBlock + u < nks) {
        const int2 x = ksum[j0 / kSumBlock + u];
        ks_wg.x = min(ks_wg.x, x.x);
        ks_wg.y = max(ks_wg.y, x.y);
      }
  }
  // does the q-tile of item `it` hold a row that sees any of the workgroup's keys?  (document-id summaries)
  auto item_visible = [&](int it) __attribute__((always_inline)) -> bool {
    const int2* qsum = p.q_sum + (int64_t)b * nqs;
    const int t = t_lo + it % nt;
    int2 qs = qsum[min(t * NB, nqs - 1)];
    for (int u = 1; u < NB; ++u)
      if (t * NB + u < nqs) {
        const int2 x = qsum[t * NB + u];
        qs.x = min(qs.x, x.x);
        qs.y = max(qs.y, x.y);
      }
    const int q_last = (t * BN + BN < p.Sq ? t * BN + BN : p.Sq) - 1;
    return classify_block(MASK, t * BN + p.q_off, q_last + p.q_off, j0, j0 + C::BM - 1, p.Sk, p.window, p.prefix, qs, ks_wg) != kSkip;
  };
  auto next_item = [&](int it) __attribute__((always_inline)) -> int {
    if constexpr ((MASK & kMaskDoc) != 0) {
      if (it < n_items && !item_visible(it)) {       // a run of hidden q-tiles: 64 per round, one per lane
        ++it;
        while (it < n_items) {
          const int ii = it + lane;
          const unsigned long long found = __builtin_amdgcn_ballot_w64(ii < n_items && item_visible(ii));
          if (found != 0) {
            it += __builtin_ctzll(found);
            break;
          }
          it += 64;
        }
        it = __builtin_amdgcn_readfirstlane(it < n_items ? it : n_items);
      }
    }
    return it;
  };

  auto load_item = [&](int it, int stage) __attribute__((always_inline)) {
    const int t = t_lo + it % nt, h = h_first + it / nt;
    const int nvalid = min(BN, p.Sq - t * BN);
    unsigned char* st = lds_raw + stage * C::STAGE_KV;
    const unsigned char* qb = (const unsigned char*)((const uint16_t*)p.q.ptr + b * p.q.sb + g * p.q.sg + h * p.q.sh + (int64_t)(t * BN) * p.q.ss);
    const unsigned char* db = (const unsigned char*)((const uint16_t*)p.dout.ptr + b * p.dout.sb + g * p.dout.sg + h * p.dout.sh + (int64_t)(t * BN) * p.dout.ss);
#pragma unroll
    for (int u = 0; u < C::TILE_INSTR / C::NW; ++u) {
      tile_load_instr<C>(qb, p.q.ss * 2, nvalid, wave + u * C::NW, lane, st);
      tile_load_instr<C>(db, p.dout.ss * 2, nvalid, wave + u * C::NW, lane, st + C::TILE);
    }
    // row statistics: 64 rows per instruction, 4 bytes per lane
    const int64_t srow = ((int64_t)(b * p.G + g) * p.H + h) * p.Sq;
    for (int u = wave; u < 2 * (BN / 64 > 0 ? BN / 64 : 1); u += C::NW) {
      const int which = u % 2, blk = u / 2;        // 0: lse2, 1: delta
      const int r = blk * 64 + lane;
      const int row = t * BN + (r < nvalid ? r : nvalid - 1);
      const float* src = (which == 0 ? p.lse2 : p.delta) + srow + row;
      if (BN >= 64 || lane < BN) {
        lds_void* dst = (lds_void*)(st + 2 * C::TILE + which * C::STAT + blk * 256);
        __builtin_amdgcn_global_load_lds((global_cvoid*)src, dst, 4, 0, 0);
      }
    }
  };

  // ---- software pipeline over 32-row query blocks.  Step n owns block n (scores and dP in
  // registers) and its successor:
  //   phase A:  S, dP of block n + 1 on the matrix core   ||   P, dS of the first 16 rows of block n
  //   phase B:  dV += dO^T P, dK += Q^T dS of block n, rows 0..15 first   ||   P, dS of rows 16..31
  // so the matrix core and the vector ALU of a wave have independent work at the same time.  The
  // Q / dO tiles cycle through a ring of three LDS stages: the tile after next is requested when
  // every wave has left the tile before the current one.
  struct Blk {
    f32x16 s, dp;
  };
  constexpr int NSTAGE = 3;
  // one step: block QB of the tile in the LDS stage at byte offset base_c is current, block QN of
  // the tile at base_n is next (the same tile, or row block 0 of the following one)
  auto step = [&](auto qb_c, auto qn_c, uint32_t base_c, uint32_t base_n, int it, bool first, Blk& cur, Blk& nxt) __attribute__((always_inline)) {
    constexpr int QB = decltype(qb_c)::value, QN = decltype(qn_c)::value;
    const int t = t_lo + it % nt, h = h_first + it / nt;
    const int ib = t * BN + 32 * QB;
    const float slope2 = C::MOD == kModAlibi ? p.alibi_slopes[h] * kLog2e : 0.f;
    const int cls = classify_block(POS, ib + p.q_off, ib + 31 + p.q_off, jw, jw + 31, p.Sk, p.window, p.prefix, make_int2(0, 0), make_int2(0, 0));
    const bool need_mask = (MASK & (kMaskDoc | kMaskCustom)) != 0 || ib + 31 >= p.Sq || cls != kFull;
    uint32_t ra_n[KK], ta_c[DB][2];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) ra_n[kk] = w.ra[kk] + base_n;
#pragma unroll
    for (int d = 0; d < DB; ++d) {
      ta_c[d][0] = w.ta[d][0] + base_c;
      ta_c[d][1] = w.ta[d][1] + base_c;
    }
    // row statistics of the current block's 16 rows of this half: quads of lse2 and of delta, read
    // shortly before the element pairs that use them
    const uint32_t stat_addr = (uint32_t)(4 * w.half) * 4 + base_c;
    i32x4 st_l[4], st_d[4];
    auto read_stats = [&](auto q_lo, auto q_hi) __attribute__((always_inline)) {   // quads [q_lo, q_hi): rows 8*q .. 8*q + 3 (+ 4*half)
      static_for<decltype(q_lo)::value, decltype(q_hi)::value>([&](auto qc) __attribute__((always_inline)) {
        constexpr int q4 = decltype(qc)::value;
        W::template read_b128<2 * C::TILE + (32 * QB + 8 * q4) * 4>(st_l[q4], stat_addr);
        W::template read_b128<2 * C::TILE + C::STAT + (32 * QB + 8 * q4) * 4>(st_d[q4], stat_addr);
      });
    };
    if (first) {                                   // the very first block: its scores are not there yet
      uint32_t ra_c[KK];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) ra_c[kk] = w.ra[kk] + base_c;
      cur.s = W::zero16();
      cur.dp = W::zero16();
      w.template row_stream_g<RowPair<QB * 32 * ROW, C::TILE + QB * 32 * ROW, KK>, 2 * KK, 2>(
          ra_c, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
            constexpr int f = decltype(fc)::value;
            if constexpr (f < KK) cur.s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[f], cur.s, 0, 0, 0);
            else cur.dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, vf[f - KK], cur.dp, 0, 0, 0);
          });
    }
    read_stats(std::integral_constant<int, 0>(), std::integral_constant<int, 2>());   // for the pairs of phase A
    const int irow = ib + 4 * w.half;              // query row of register 0
    int qd[16];
    if constexpr ((MASK & kMaskDoc) != 0) {
      const int32_t* qdoc = p.q_doc + (int64_t)b * p.Sq;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = irow + 8 * (r >> 2) + (r & 3);
        qd[r] = qdoc[i < p.Sq ? i : p.Sq - 1];
      }
    }
    float bl[C::NBIAS > 0 ? 16 : 1];               // bias values of the current block's scores of this lane
    if constexpr (C::NBIAS > 0) {
      BiasHead<C::NBIAS> bh_;
      bh_.set(p, b, g, h);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int i = irow + 8 * (r >> 2) + (r & 3);
        bl[r] = bh_.value(p, i < p.Sq ? i : p.Sq - 1, jc);
      }
    }
    uint32_t pw[8], dsw[8];
    auto ew_pair = [&](int r2) __attribute__((always_inline)) {      // P and dS of registers 2*r2, 2*r2 + 1
      float pv[2], dsv[2];
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const int r = 2 * r2 + e;
        const int i = irow + 8 * (r >> 2) + (r & 3);
        const float lse2 = __int_as_float(st_l[r >> 2][r & 3]), delta = __int_as_float(st_d[r >> 2][r & 3]);
        float fac;
        float a;
        if constexpr (C::MOD == kModCustom) a = replay_user<C::MOD>(cur.s[r], p, uctx, lse2, b, g, h, i, j, fac);
        else a = replay_score<C::MOD>(cur.s[r], c_scale, lse2, p.softcap, slope2, (float)(i + p.q_off - j), fac);
        if constexpr (C::NBIAS > 0) a += bl[r];
        pv[e] = fast_exp2(a);
        dsv[e] = cur.dp[r] - delta;
        if constexpr (C::MOD == kModSoftcap || C::MOD == kModCustom) dsv[e] *= fac;
      }
      if (need_mask) {                             // uniform; kept a branch: most blocks need no mask
        asm volatile("");
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int r = 2 * r2 + e;
          const int i = irow + 8 * (r >> 2) + (r & 3);
          if (hidden_user<MASK>(i, j, p, uctx, b, g, h, (MASK & kMaskDoc) ? qd[r] : 0, kdoc)) pv[e] = 0.f;
        }
      }
      dsv[0] *= pv[0];
      dsv[1] *= pv[1];
      pw[r2] = pack_bf16(pv[0], pv[1]);
      dsw[r2] = pack_bf16(dsv[0], dsv[1]);
      asm volatile("" : "+v"(pw[r2]), "+v"(dsw[r2]));               // stays where it is scheduled
    };
    // phase A
    nxt.s = W::zero16();
    nxt.dp = W::zero16();
    w.template row_stream_g<RowPair<QN * 32 * ROW, C::TILE + QN * 32 * ROW, KK>, 2 * KK, C::GR>(
        ra_n, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
          constexpr int f = decltype(fc)::value;
          if constexpr (f < KK) nxt.s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[f], nxt.s, 0, 0, 0);
          else nxt.dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, vf[f - KK], nxt.dp, 0, 0, 0);
          constexpr int per = (2 * KK) / 4;        // MFMAs per element pair (pairs 0..3 in this phase)
          if constexpr (f % per == per - 1) ew_pair(f / per);
          __builtin_amdgcn_sched_barrier(0);
        });
    // phase B
    read_stats(std::integral_constant<int, 2>(), std::integral_constant<int, 4>());   // covered by the first wait below
    w.template tr_stream_g<TrQuad<C::TILE + QB * 32 * ROW, QB * 32 * ROW, DB, ROW>, 4 * DB, C::GT>(
        ta_c, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
          constexpr int f = decltype(fc)::value, d = f % DB, grp = f / DB, ks = grp / 2;
          if constexpr (grp % 2 == 0) {
            const bf16x8 bop = __builtin_bit_cast(
                bf16x8, (i32x4){(int)pw[4 * ks], (int)pw[4 * ks + 1], (int)pw[4 * ks + 2], (int)pw[4 * ks + 3]});
            dv[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bop, dv[d], 0, 0, 0);
          } else {
            const bf16x8 bop = __builtin_bit_cast(
                bf16x8, (i32x4){(int)dsw[4 * ks], (int)dsw[4 * ks + 1], (int)dsw[4 * ks + 2], (int)dsw[4 * ks + 3]});
            dk[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bop, dk[d], 0, 0, 0);
          }
          constexpr int per = (2 * DB) / 4;        // MFMAs per element pair (pairs 4..7 during the rows-0..15 half)
          if constexpr (f < 2 * DB && f % per == per - 1) ew_pair(4 + f / per);
          __builtin_amdgcn_sched_barrier(0);
        });
  };
  static_assert(NB == 2, "a tile is two row blocks: the two score register sets swap roles twice per tile");

  int it0 = next_item(0);
  if (it0 < n_items) {
    int it1 = next_item(it0 + 1);
    int it2 = it1 < n_items ? next_item(it1 + 1) : n_items;
    load_item(it0, 0);
    if (it1 < n_items) load_item(it1, 1);
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)
    __syncthreads();
    if (it2 < n_items) load_item(it2, 2);
    Blk ba, bb;
    int stage = 0;                                 // ring stage of the current tile
    bool first = true;
    while (it0 < n_items) {
      const int stage_n = stage + 1 == NSTAGE ? 0 : stage + 1;
      const uint32_t base_c = stage * C::STAGE_KV, base_n = stage_n * C::STAGE_KV;
      step(std::integral_constant<int, 0>(), std::integral_constant<int, 1>(), base_c, base_c, it0, first, ba, bb);
      step(std::integral_constant<int, 1>(), std::integral_constant<int, 0>(), base_c, base_n, it0, false, bb, ba);
      first = false;
      __builtin_amdgcn_s_waitcnt(0x0F70);          // the tile after next has landed ...
      __syncthreads();                             // ... for everyone, and everyone has left this tile
      it0 = it1;
      it1 = it2;
      it2 = it2 < n_items ? next_item(it2 + 1) : n_items;
      if (it2 < n_items) load_item(it2, stage);
      stage = stage_n;
    }
  }

  if (j < p.Sk) {
#pragma unroll
    for (int d = 0; d < DB; ++d)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int ch = 32 * d + 8 * r4 + 4 * w.half;
        store_kv_grad(p, p.dk, p.part_dk, split, b, g, hk, j, ch, D, dk[d][4 * r4] * p.scale, dk[d][4 * r4 + 1] * p.scale,
                      dk[d][4 * r4 + 2] * p.scale, dk[d][4 * r4 + 3] * p.scale);
        store_kv_grad(p, p.dv, p.part_dv, split, b, g, hk, j, ch, D, dv[d][4 * r4], dv[d][4 * r4 + 1], dv[d][4 * r4 + 2],
                      dv[d][4 * r4 + 3]);
      }
  }
}

// ------------------------------------------------------------------------------------------------
// dK, dV with specialised waves: the same contractions as bwd_dkdv_kernel, for head dims whose
// accumulators (32 keys x D channels x two gradients in fp32) leave no room for a second wave on
// the SIMD.  Eight waves per workgroup; waves w and w + 4 own the same 32 keys and share a SIMD:
//   wave w     ("P wave"):   S = Q K^T, P = exp2(..), dV += dO^T P one block later; hands P (times
//                            the soft-cap derivative) to its partner through LDS, fp32
//   wave w + 4 ("dS wave"):  dP = dO V^T, dS = P * (dP - delta) one block later, dK += Q^T dS
// Each does half of the matrix work of a block and holds one accumulator set, so both fit the
// register budget of two waves per SIMD and fill each other's stalls.  One workgroup barrier per
// 32-row block hands the P blocks over (two exchange buffers per wave pair).
// ------------------------------------------------------------------------------------------------
template <class C>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
bwd_dkdv_ws_kernel(const BwdParams p) {
  constexpr int D = C::D, BN = C::BN, NB = C::NB, KK = C::KK, DB = C::DB, ROW = C::ROW;
  constexpr uint32_t MASK = C::MASK;
  constexpr uint32_t POS = MASK & ~kMaskDoc;
  static_assert(C::MOD != kModCustom && (MASK & kMaskCustom) == 0, "compiled variants run the plain dK/dV kernel");
  constexpr int NWS = 8;                           // waves of the workgroup
  constexpr int NSTAGE = 3;
  constexpr int XBUF = 64 * 16 * 4;                // one exchange buffer: 16 floats per lane, [quad][lane][4]
  constexpr int XCH = NSTAGE * C::STAGE_KV;        // exchange buffers [key group][2] follow the tile ring
  constexpr int PPM = 8 / KK;                      // element pairs per MFMA of phase 1
  static_assert(NB == 2 && BN == 64, "two row blocks per tile");
  static_assert(C::TILE_INSTR % NWS == 0, "every wave issues the same number of loads");
  typedef BwdWave<C> W;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int role = wave >> 2, kg = wave & 3;       // 0: P wave, 1: dS wave; key group
  W w;
  w.init(tid & 63);
  const int lane = w.lane;

  const int nk = p.n_ktiles;
  int kt, bh;
  if (p.order_k == 1) {                            // whole key/value heads per XCD: their Q / dO tiles stay in one L2
    const int idx = blockIdx.x >> 3;
    bh = (idx / nk) * 8 + (blockIdx.x & 7);
    kt = idx % nk;
  } else {
    kt = blockIdx.x % nk;
    bh = blockIdx.x / nk;
  }
  // bh counts (b, g, kv head, subset of the group's query heads)
  const int split = bh % p.hsplit, bhk = bh / p.hsplit;
  const int hk = bhk % p.Hkv, g = (bhk / p.Hkv) % p.G, b = bhk / (p.Hkv * p.G);
  const int group = p.H / p.Hkv / p.hsplit;        // query heads this workgroup sums over
  const int h_first = hk * (p.H / p.Hkv) + split * group;
  const int j0 = kt * C::BM, jw = j0 + 32 * kg;
  const int j = jw + w.col, jc = j < p.Sk ? j : p.Sk - 1;
  const float c_scale = p.scale * kLog2e;

  // query rows that can see the workgroup's keys; q-tile skipping for document masks
  const int j_last = (j0 + C::BM < p.Sk ? j0 + C::BM : p.Sk) - 1;
  int q_lo, q_hi;
  query_range(MASK, j0, j_last, p.Sq + p.q_off, p.window, p.prefix, q_lo, q_hi);   // as positions; row = position - q_off
  q_lo = max(q_lo - p.q_off, 0);
  q_hi = max(q_hi - p.q_off, 0);
  const int t_lo = q_lo / BN, t_hi = (q_hi + BN - 1) / BN;
  const int nt = t_hi - t_lo;                      // q-tiles per head
  const int n_items = nt > 0 ? nt * group : 0;     // (head of the group, q-tile), head-major
  const int nqs = (p.Sq + kSumBlock - 1) / kSumBlock;
  int2 ks_wg = make_int2(0, 0);
  if constexpr ((MASK & kMaskDoc) != 0) {
    const int nks = (p.Sk + kSumBlock - 1) / kSumBlock;
    const int2* ksum = p.kv_sum + (int64_t)b * nks;
    ks_wg = ksum[j0 / kSumBlock];
    for (int u = 1; u < C::BM / kSumBlock; ++u)
      if (j0 / kSumBlock + u < nks) {
        const int2 x = ksum[j0 / kSumBlock + u];
        ks_wg.x = min(ks_wg.x, x.x);
        ks_wg.y = max(ks_wg.y, x.y);
      }
  }
  // does the q-tile of item `it` hold a row that sees any of the workgroup's keys?  (document-id summaries)
  auto item_visible = [&](int it) __attribute__((always_inline)) -> bool {
    const int2* qsum = p.q_sum + (int64_t)b * nqs;
    const int t = t_lo + it % nt;
    int2 qs = qsum[min(t * NB, nqs - 1)];
    for (int u = 1; u < NB; ++u)
      if (t * NB + u < nqs) {
        const int2 x = qsum[t * NB + u];
        qs.x = min(qs.x, x.x);
        qs.y = max(qs.y, x.y);
      }
    const int q_last = (t * BN + BN < p.Sq ? t * BN + BN : p.Sq) - 1;
    return classify_block(MASK, t * BN + p.q_off, q_last + p.q_off, j0, j0 + C::BM - 1, p.Sk, p.window, p.prefix, qs, ks_wg) != kSkip;
  };
  auto next_item = [&](int it) __attribute__((always_inline)) -> int {
    if constexpr ((MASK & kMaskDoc) != 0) {
      if (it < n_items && !item_visible(it)) {       // a run of hidden q-tiles: 64 per round, one per lane
        ++it;
        while (it < n_items) {
          const int ii = it + lane;
          const unsigned long long found = __builtin_amdgcn_ballot_w64(ii < n_items && item_visible(ii));
          if (found != 0) {
            it += __builtin_ctzll(found);
            break;
          }
          it += 64;
        }
        it = __builtin_amdgcn_readfirstlane(it < n_items ? it : n_items);
      }
    }
    return it;
  };
  auto load_item = [&](int it, int stage) __attribute__((always_inline)) {
    const int t = t_lo + it % nt, h = h_first + it / nt;
    const int nvalid = min(BN, p.Sq - t * BN);
    unsigned char* st = lds_raw + stage * C::STAGE_KV;
    const unsigned char* qb = (const unsigned char*)((const uint16_t*)p.q.ptr + b * p.q.sb + g * p.q.sg + h * p.q.sh + (int64_t)(t * BN) * p.q.ss);
    const unsigned char* db = (const unsigned char*)((const uint16_t*)p.dout.ptr + b * p.dout.sb + g * p.dout.sg + h * p.dout.sh + (int64_t)(t * BN) * p.dout.ss);
#pragma unroll
    for (int u = 0; u < C::TILE_INSTR / NWS; ++u) {
      tile_load_instr<C>(qb, p.q.ss * 2, nvalid, wave + u * NWS, lane, st);
      tile_load_instr<C>(db, p.dout.ss * 2, nvalid, wave + u * NWS, lane, st + C::TILE);
    }
    if (wave < 2) {                                // row statistics, 4 bytes per lane: wave 0 lse2, wave 1 delta
      const int64_t srow = ((int64_t)(b * p.G + g) * p.H + h) * p.Sq;
      const int row = t * BN + (lane < nvalid ? lane : nvalid - 1);
      const float* src = (wave == 0 ? p.lse2 : p.delta) + srow + row;
      lds_void* dst = (lds_void*)(st + 2 * C::TILE + wave * C::STAT);
      __builtin_amdgcn_global_load_lds((global_cvoid*)src, dst, 4, 0, 0);
    }
  };
  // end of an iteration: this wave's LDS traffic (and, when `loads`, its tile loads) is complete, then
  // the workgroup barrier.  No fence beyond that: every LDS access of the loop is issued by hand.
  auto iteration_end = [&](bool loads) __attribute__((always_inline)) {
    if (loads) __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0)
    asm volatile("" ::: "memory");                   // no memory access moves across the barrier at compile time
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  // window of the tile list: items at list positions P - 1, P, P + 1, P + 2 (n_items = none)
  int itm1 = n_items, it0 = next_item(0);
  int itp1 = it0 < n_items ? next_item(it0 + 1) : n_items;
  int itp2 = itp1 < n_items ? next_item(itp1 + 1) : n_items;
  if (it0 < n_items) load_item(it0, 0);
  if (itp1 < n_items) load_item(itp1, 1);
  if (itp2 < n_items) load_item(itp2, 2);
  iteration_end(true);
  int s0 = 0;                                      // ring stage of position P
  const uint32_t xaddr = XCH + kg * (2 * XBUF) + lane * 16;   // this lane's slot in exchange buffer 0 of its wave pair
  const uint32_t stat_addr = (uint32_t)(4 * w.half) * 4;

  if (role == 0) {
    // ================= P wave =================
    bf16x8 kf[KK];
    {
      const uint16_t* kp = (const uint16_t*)p.k.ptr + b * p.k.sb + g * p.k.sg + hk * p.k.sh + (int64_t)jc * p.k.ss;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kf[kk] = *(const bf16x8*)(kp + 16 * kk + 8 * w.half);
    }
    int kdoc = 0;
    if constexpr ((MASK & kMaskDoc) != 0) kdoc = p.kv_doc[(int64_t)b * p.Sk + jc];
    f32x16 dv[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d) dv[d] = W::zero16();
    f32x16 sa = W::zero16(), sb = W::zero16();
    uint32_t pw[8] = {0, 0, 0, 0, 0, 0, 0, 0};     // bf16 pairs of the last block's P, consumed one iteration later
    auto scores = [&](auto off_c, uint32_t base, f32x16& dst) __attribute__((always_inline)) {   // S of one block, no overlap
      uint32_t ra_b[KK];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) ra_b[kk] = w.ra[kk] + base;
      dst = W::zero16();
      w.template row_stream_g<RowOne<decltype(off_c)::value>, KK, 2>(ra_b, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        dst = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[decltype(fc)::value], dst, 0, 0, 0);
      });
    };
    // block QB of item `it` (stage offset base_c) is current (scores in cur); the scores of block QN at
    // base_n go to nxt; P of the current block goes to exchange buffer XB
    auto p_iter = [&](auto qb_c, auto qn_c, auto xb_c, uint32_t base_c, uint32_t base_n, int it, f32x16& cur, f32x16& nxt) __attribute__((always_inline)) {
      constexpr int QB = decltype(qb_c)::value, QN = decltype(qn_c)::value, XB = decltype(xb_c)::value;
      const int t = t_lo + it % nt, h = h_first + it / nt;
      const int ib = t * BN + 32 * QB;
      const float slope2 = C::MOD == kModAlibi ? p.alibi_slopes[h] * kLog2e : 0.f;
      const int cls = classify_block(POS, ib + p.q_off, ib + 31 + p.q_off, jw, jw + 31, p.Sk, p.window, p.prefix, make_int2(0, 0), make_int2(0, 0));
      const bool need_mask = (MASK & kMaskDoc) != 0 || ib + 31 >= p.Sq || cls != kFull;
      uint32_t ra_n[KK];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) ra_n[kk] = w.ra[kk] + base_n;
      i32x4 st_l[4];                               // lse2 of the block's 16 rows of this half
      static_for<0, 4>([&](auto qc) __attribute__((always_inline)) {
        W::template read_b128<2 * C::TILE + (32 * QB + 8 * decltype(qc)::value) * 4>(st_l[decltype(qc)::value], stat_addr + base_c);
      });
      const int irow = ib + 4 * w.half;            // query row of register 0
      int qd[16];
      if constexpr ((MASK & kMaskDoc) != 0) {
        const int32_t* qdoc = p.q_doc + (int64_t)b * p.Sq;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = irow + 8 * (r >> 2) + (r & 3);
          qd[r] = qdoc[i < p.Sq ? i : p.Sq - 1];
        }
      }
      float bl[C::NBIAS > 0 ? 16 : 1];             // bias values of the current block's scores of this lane
      if constexpr (C::NBIAS > 0) {
        BiasHead<C::NBIAS> bh_;
        bh_.set(p, b, g, h);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int i = irow + 8 * (r >> 2) + (r & 3);
          bl[r] = bh_.value(p, i < p.Sq ? i : p.Sq - 1, jc);
        }
      }
      float pf[4];
      auto ew_pair = [&](auto r2c) __attribute__((always_inline)) {
        constexpr int r2 = decltype(r2c)::value;
        float pv[2], fc2[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int r = 2 * r2 + e;
          const int i = irow + 8 * (r >> 2) + (r & 3);
          const float lse2 = __int_as_float(st_l[r >> 2][r & 3]);
          float a = replay_score<C::MOD>(cur[r], c_scale, lse2, p.softcap, slope2, (float)(i + p.q_off - j), fc2[e]);
          if constexpr (C::NBIAS > 0) a += bl[r];
          pv[e] = fast_exp2(a);
        }
        if (need_mask) {                           // uniform; kept a branch: most blocks need no mask
          asm volatile("");
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int r = 2 * r2 + e;
            const int i = irow + 8 * (r >> 2) + (r & 3);
            if (hidden<MASK>(i, j, p.Sq, p.Sk, p.q_off, p.window, p.prefix, (MASK & kMaskDoc) ? qd[r] : 0, kdoc)) pv[e] = 0.f;
          }
        }
        pw[r2] = pack_bf16(pv[0], pv[1]);
        asm volatile("" : "+v"(pw[r2]));
        pf[2 * (r2 & 1)] = C::MOD == kModSoftcap ? pv[0] * fc2[0] : pv[0];
        pf[2 * (r2 & 1) + 1] = C::MOD == kModSoftcap ? pv[1] * fc2[1] : pv[1];
        if constexpr (r2 % 2 == 1)                 // registers 4q .. 4q + 3 are complete: quad q = r2 / 2
          W::template write_b128<XB * XBUF + (r2 / 2) * 1024>(
              xaddr, (i32x4){__float_as_int(pf[0]), __float_as_int(pf[1]), __float_as_int(pf[2]), __float_as_int(pf[3])});
      };
      // phase 1: scores of the next block  ||  P of the current block
      nxt = W::zero16();
      w.template row_stream_g<RowOne<QN * 32 * ROW>, KK, 2>(ra_n, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        constexpr int f = decltype(fc)::value;
        nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[f], nxt, 0, 0, 0);
        static_for<f * PPM, (f + 1) * PPM>([&](auto r2c) __attribute__((always_inline)) { ew_pair(r2c); });
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    // dV += dO^T P for the block whose P (bf16 pairs in pw) the previous iteration formed: it runs
    // first in an iteration, while the partner wave is in its mixed phase, and the mixed phase above
    // runs while the partner is in its pure matrix phase
    auto dv_phase = [&](auto qb_c, uint32_t base_c) __attribute__((always_inline)) {
      constexpr int QB = decltype(qb_c)::value;
      uint32_t ta_c[DB][2];
#pragma unroll
      for (int d = 0; d < DB; ++d) {
        ta_c[d][0] = w.ta[d][0] + base_c;
        ta_c[d][1] = w.ta[d][1] + base_c;
      }
      w.template tr_stream_g<TrOne<C::TILE + QB * 32 * ROW, DB, ROW>, 2 * DB, 2>(ta_c, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        constexpr int f = decltype(fc)::value, d = f % DB, ks = f / DB;
        const bf16x8 bop = __builtin_bit_cast(
            bf16x8, (i32x4){(int)pw[4 * ks], (int)pw[4 * ks + 1], (int)pw[4 * ks + 2], (int)pw[4 * ks + 3]});
        dv[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bop, dv[d], 0, 0, 0);
      });
    };
    if (it0 < n_items) scores(std::integral_constant<int, 0>(), 0u, sa);
    while (true) {
      const bool vp = it0 < n_items, vm = itm1 < n_items;
      if (!vp && !vm) break;
      const uint32_t b0 = s0 * C::STAGE_KV, b1 = (s0 + 1 == NSTAGE ? 0 : s0 + 1) * C::STAGE_KV;
      const int s2 = s0 + 2 >= NSTAGE ? s0 + 2 - NSTAGE : s0 + 2;
      // even iteration: dV of block (P - 1, 1); block (P, 0) current, (P, 1) next
      if (vm) dv_phase(std::integral_constant<int, 1>(), (uint32_t)(s2 * C::STAGE_KV));
      if (vp) p_iter(std::integral_constant<int, 0>(), std::integral_constant<int, 1>(), std::integral_constant<int, 0>(), b0, b0, it0, sa, sb);
      iteration_end(true);
      if (!vp) break;
      // odd iteration: dV of block (P, 0); block (P, 1) current, (P + 1, 0) next; the tile at P + 2
      // replaces the one at P - 1
      if (vm && itp2 < n_items) load_item(itp2, s2);
      dv_phase(std::integral_constant<int, 0>(), b0);
      p_iter(std::integral_constant<int, 1>(), std::integral_constant<int, 0>(), std::integral_constant<int, 1>(), b0, b1, it0, sb, sa);
      iteration_end(false);
      itm1 = it0;
      it0 = itp1;
      itp1 = itp2;
      itp2 = itp2 < n_items ? next_item(itp2 + 1) : n_items;
      s0 = s0 + 1 == NSTAGE ? 0 : s0 + 1;
    }
    if (j < p.Sk) {
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          store_kv_grad(p, p.dv, p.part_dv, split, b, g, hk, j, 32 * d + 8 * r4 + 4 * w.half, D, dv[d][4 * r4],
                        dv[d][4 * r4 + 1], dv[d][4 * r4 + 2], dv[d][4 * r4 + 3]);
    }
  } else {
    // ================= dS wave =================
    bf16x8 vf[KK];
    {
      const uint16_t* vp = (const uint16_t*)p.v.ptr + b * p.v.sb + g * p.v.sg + hk * p.v.sh + (int64_t)jc * p.v.ss;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) vf[kk] = *(const bf16x8*)(vp + 16 * kk + 8 * w.half);
    }
    f32x16 dk[DB];
#pragma unroll
    for (int d = 0; d < DB; ++d) dk[d] = W::zero16();
    f32x16 da = W::zero16(), db = W::zero16();
    auto dscores = [&](auto off_c, uint32_t base, f32x16& dst) __attribute__((always_inline)) {  // dP of one block, no overlap
      uint32_t ra_b[KK];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) ra_b[kk] = w.ra[kk] + base;
      dst = W::zero16();
      w.template row_stream_g<RowOne<decltype(off_c)::value>, KK, 2>(ra_b, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        dst = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, vf[decltype(fc)::value], dst, 0, 0, 0);
      });
    };
    // block QP at stage offset base_p was handed over in exchange buffer XB (its dP in cur); the dP of
    // block QN at base_n goes to nxt
    auto ds_iter = [&](auto qp_c, auto qn_c, auto xb_c, uint32_t base_p, uint32_t base_n, f32x16& cur, f32x16& nxt) __attribute__((always_inline)) {
      constexpr int QP = decltype(qp_c)::value, QN = decltype(qn_c)::value, XB = decltype(xb_c)::value;
      uint32_t ra_n[KK], ta_p[DB][2];
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) ra_n[kk] = w.ra[kk] + base_n;
#pragma unroll
      for (int d = 0; d < DB; ++d) {
        ta_p[d][0] = w.ta[d][0] + base_p;
        ta_p[d][1] = w.ta[d][1] + base_p;
      }
      i32x4 pq[4], st_d[4];                        // P of the block (fp32) and delta of its rows, by register quad
      static_for<0, 4>([&](auto qc) __attribute__((always_inline)) {
        constexpr int q4 = decltype(qc)::value;
        W::template read_b128<XB * XBUF + q4 * 1024>(pq[q4], xaddr);
        W::template read_b128<2 * C::TILE + C::STAT + (32 * QP + 8 * q4) * 4>(st_d[q4], stat_addr + base_p);
      });
      uint32_t dsw[8];
      auto ew_pair = [&](auto r2c) __attribute__((always_inline)) {
        constexpr int r2 = decltype(r2c)::value;
        float dsv[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int r = 2 * r2 + e;
          dsv[e] = __int_as_float(pq[r >> 2][r & 3]) * (cur[r] - __int_as_float(st_d[r >> 2][r & 3]));
        }
        dsw[r2] = pack_bf16(dsv[0], dsv[1]);
        asm volatile("" : "+v"(dsw[r2]));
      };
      // phase 1: dP of the next block  ||  dS of the handed-over block
      nxt = W::zero16();
      w.template row_stream_g<RowOne<C::TILE + QN * 32 * ROW>, KK, 2>(ra_n, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        constexpr int f = decltype(fc)::value;
        nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, vf[f], nxt, 0, 0, 0);
        static_for<f * PPM, (f + 1) * PPM>([&](auto r2c) __attribute__((always_inline)) { ew_pair(r2c); });
        __builtin_amdgcn_sched_barrier(0);
      });
      // phase 2: dK += Q^T dS
      w.template tr_stream_g<TrOne<QP * 32 * ROW, DB, ROW>, 2 * DB, 2>(ta_p, [&](auto fc, bf16x8 a) __attribute__((always_inline)) {
        constexpr int f = decltype(fc)::value, d = f % DB, ks = f / DB;
        const bf16x8 bop = __builtin_bit_cast(
            bf16x8, (i32x4){(int)dsw[4 * ks], (int)dsw[4 * ks + 1], (int)dsw[4 * ks + 2], (int)dsw[4 * ks + 3]});
        dk[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bop, dk[d], 0, 0, 0);
      });
    };
    if (it0 < n_items) dscores(std::integral_constant<int, C::TILE>(), 0u, da);
    while (true) {
      const bool vp = it0 < n_items, vm = itm1 < n_items;
      if (!vp && !vm) break;
      const uint32_t b0 = s0 * C::STAGE_KV;
      const int s2 = s0 + 2 >= NSTAGE ? s0 + 2 - NSTAGE : s0 + 2;
      const uint32_t b2 = s2 * C::STAGE_KV;        // stage of position P - 1
      // even iteration: block (P - 1, 1) was handed over in buffer 1; dP of block (P, 0) is next
      if (vm) ds_iter(std::integral_constant<int, 1>(), std::integral_constant<int, 0>(), std::integral_constant<int, 1>(), b2, b0, db, da);
      iteration_end(true);
      if (!vp) break;
      // odd iteration: block (P, 0) was handed over in buffer 0; dP of block (P, 1) is next
      if (vm && itp2 < n_items) load_item(itp2, s2);
      ds_iter(std::integral_constant<int, 0>(), std::integral_constant<int, 1>(), std::integral_constant<int, 0>(), b0, b0, da, db);
      iteration_end(false);
      itm1 = it0;
      it0 = itp1;
      itp1 = itp2;
      itp2 = itp2 < n_items ? next_item(itp2 + 1) : n_items;
      s0 = s0 + 1 == NSTAGE ? 0 : s0 + 1;
    }
    if (j < p.Sk) {
#pragma unroll
      for (int d = 0; d < DB; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4)
          store_kv_grad(p, p.dk, p.part_dk, split, b, g, hk, j, 32 * d + 8 * r4 + 4 * w.half, D, dk[d][4 * r4] * p.scale,
                        dk[d][4 * r4 + 1] * p.scale, dk[d][4 * r4 + 2] * p.scale, dk[d][4 * r4 + 3] * p.scale);
    }
  }
}

}  // namespace fl
