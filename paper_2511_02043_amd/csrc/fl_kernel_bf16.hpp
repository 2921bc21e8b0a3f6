// bf16 attention-variant forward kernel for gfx950: both contractions on bf16 MFMA with fp32
// accumulation, scores and softmax state in registers, K/V tiles ring-buffered in LDS and
// filled by direct global->LDS loads.
//
// Structure (Sec. 3 of the paper names the fused pass this realises: one score tile at a time,
// folded into a running row maximum / row sum with the accumulator rescaled as needed, then
// multiplied by the matching V tile;
// Sec. 3.2: the key axis is a sequential loop inside the workgroup that owns a query tile;
// Sec. 3.4: running max / running sum with the exp(m_old - m_new) correction; Sec. 3.5: D and
// Dv each fit one tile, so the twin matmul needs no loop over them; Sec. 3.6: 1-D launch whose
// index is decoded in the kernel).
//
// Orientation.  Each wave owns RB blocks of 32 query rows and computes TRANSPOSED score blocks
//     S^T[key n][query m] = sum_d K[n][d] Q[m][d]          (v_mfma_f32_32x32x16_bf16)
// with K as the A operand (one 16-byte LDS read per lane) and Q as the B operand (kept in
// registers for the whole kernel).  In the 32x32 accumulator layout lane L then holds, for the
// single query m = L % 32, sixteen keys n = 8*(r/4) + 4*(L/32) + r%4 (r = 0..15).  So
//   * a softmax row lives in two lanes (L and L^32): row max / row sum are in-lane reductions
//     plus one half-swap,
//   * the probabilities, rounded to bf16 pairwise, ARE the B operand of the second contraction
//     O^T[dv][m] = sum_n V^T[dv][n] P^T[n][m] without any shuffle, and
//   * V^T as the A operand comes from row-major V in LDS through ds_read_b64_tr_b16.
// Within one 16-key MFMA step the contraction index order is (half, element) -> key
// 16*ks + 8*(e/4) + 4*half + e%4 for both operands.
// Every K or V fragment read from LDS feeds the MFMAs of all RB row blocks of the wave (RB = 2
// halves the LDS traffic per FLOP but needs a whole SIMD's registers for one wave; RB = 1 with two
// waves per SIMD measured faster and is the default).
//
// Software pipeline.  Iteration n owns tile t0 (scores in registers,
// transformed, row max folded into m) and its successor t1:
//     phase A:  S1 = K(t1) Q^T on the matrix core   ||   P0 = exp2(S0 - m), first half, then the
//               transform / row max of the first key block of S1
//     phase B:  O += V(t0)^T P0 on the matrix core  ||   P0, second half (needed by the second
//               half of the MFMAs), then transform / row max of the rest of S1 and the m update
// so the matrix core and the vector ALU of one wave have independent work at the same time, and
// the two waves that share a SIMD fill each other's gaps.  What was measured on gfx950 and shaped
// this loop: a SIMD issues one instruction per 4 clocks whatever its kind (exp2 and the 32x32x16
// MFMA take two such slots), so the loop is built from as few instructions as possible -- one
// LDS wait per fragment group, no idle-cycle padding, tile bookkeeping in a handful of scalar
// instructions.  The running max is only advanced when a row's new maximum exceeds the old one by
// more than 2^8 (the exponent of P stays bounded by 8), which makes the O rescale a rare,
// wave-uniform branch; l and the final normalisation use the same reference, so the result is
// unchanged in real arithmetic.
#pragma once
#include "fl_params.hpp"

// Run-time compiled expressions are handed row and key indices inside the call's sizes when they may index a captured
// array with them (1, the default); a variant without captured arrays is compiled with 0.
#ifndef FL_USER_CLAMP
#define FL_USER_CLAMP 1
#endif

namespace fl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_cvoid;

constexpr float kLazyMaxLog2 = 8.f;   // advance the running max only past this gap (log2 units)

__device__ __forceinline__ float half_swap_max(float x) {
  // {x.lo, x.lo}, {x.hi, x.hi} -> max of lanes L and L^32 in every lane
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 v = {a, b};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t u) { return __uint_as_float((uint32_t)u << 16); }

// 16-byte chunk swizzles of the LDS tiles (row r, chunk c of a row of ROW_ELEMS bf16); both are
// XORs, hence their own inverses, and both depend on r only through bits that are the same for
// every row a given lane ever touches.  K is read one 16-byte chunk per lane with 32 consecutive
// rows per instruction; V is read by the transposing load as 4 rows x 64 bytes per 32 lanes.
// Both layouts spread those accesses over all 64 banks (measured: zero bank-conflict cycles).
template <int ROW_ELEMS>
__device__ __forceinline__ int swz_k(int r, int c) {
  constexpr int CH = ROW_ELEMS / 8;
  constexpr int RPL = CH >= 16 ? 1 : 16 / CH;      // rows per 256-byte bank line
  return c ^ ((r / RPL) % CH);
}
template <int ROW_ELEMS>
__device__ __forceinline__ int swz_v(int r, int c) {
  if constexpr (ROW_ELEMS == 128) return c ^ ((r & 3) << 2);
  else if constexpr (ROW_ELEMS == 64) return c ^ (((r >> 1) & 1) << 2);
  else return c;
}

template <int D_, int DV_, int NWAVES_, int RB_, int BN_, int WPE_, int MOD_, uint32_t MASK_, int NBIAS_,
          bool DIFF_, uint32_t EPI_, int RING_ = 2, bool PAGED_ = false, int PACK_ = 1>
struct Bf16Cfg {
  static constexpr int D = D_, DV = DV_, NWAVES = NWAVES_, RB = RB_, BN = BN_, MOD = MOD_, NBIAS = NBIAS_;
  static constexpr uint32_t MASK = MASK_, EPI = EPI_;
  static constexpr bool DIFF = DIFF_;
  // Differential + RMSNorm divides a nearly cancelling difference by its own rms, which
  // amplifies the bf16 rounding of the probabilities; there P is split into a bf16 high part
  // and a bf16 remainder and the second contraction runs on both.
  static constexpr bool PSPLIT = DIFF_ && (EPI_ & kEpiRms) != 0;
  static constexpr int WPE = WPE_;                 // waves per SIMD the register budget is set for
  static constexpr int GK = 2;                     // K fragments per LDS wait (read one group ahead)
  static constexpr int GV = 2;                     // V^T fragments (two reads each) per LDS wait
  static constexpr int NT = NWAVES * 64;
  static constexpr int WROWS = 32 * RB;            // query rows per wave
  static constexpr int NS = DIFF ? 2 : 1;          // softmax streams
  // Differential: the two streams of a row block run in two different waves (wave w and wave
  // w + NWAVES / 2, which share a SIMD), so that each keeps the register footprint of ordinary
  // attention and two waves fit a SIMD; they share the V tiles and meet in the epilogue.
  static constexpr int NROWG = NWAVES / NS;        // waves per stream = row groups of the workgroup
  static constexpr int BM = NROWG * WROWS;         // query rows per workgroup
  static constexpr int NB = BN / 32;               // 32-key blocks per tile
  static constexpr int KK = D / 16;                // MFMA k-steps of the first contraction
  static constexpr int DVB = DV / 32;              // 32-channel blocks of the output
  static constexpr int K_BYTES = BN * D * 2;
  static constexpr int V_BYTES = BN * DV * 2;
  // Slots of the K ring and of the V ring.  The workgroup meets at a barrier once per RING / 2 tiles:
  // a step reads K of the next tile and V of the current one while it streams K of the tile
  // RING / 2 + 1 ahead and V of the tile RING / 2 ahead into slots that nobody reads before the next barrier.
  static constexpr int RING = RING_;
  static constexpr int SPB = RING / 2;             // pipeline steps (tiles) per barrier
  static_assert(RING_ == 2 || RING_ == 4, "ring depth");
  static_assert(RING_ == 2 || (NBIAS_ == 0 && !DIFF_), "bias staging and the two-stream loop wait for their loads every step");
  static constexpr int K_RING = 0;                 // LDS layout: K ring [RING][NS][K_BYTES], V ring [RING][V_BYTES]
  static constexpr int V_RING = RING * NS * K_BYTES;
  static constexpr int RING_BYTES = V_RING + RING * V_BYTES;
  static constexpr int XCH_BYTES = DIFF ? NROWG * 64 * DVB * 16 * 4 : 0;   // epilogue exchange of the differential variant
  static constexpr int LDS_BYTES = RING_BYTES > XCH_BYTES ? RING_BYTES : XCH_BYTES;
  static constexpr int K_INSTR = K_BYTES / 1024;   // 64-lane x 16-byte direct loads per K tile
  static constexpr int V_INSTR = V_BYTES / 1024;
  static constexpr int K_ROWS_PI = 64 / (D / 8);   // tile rows covered by one direct-load instruction
  static constexpr int V_ROWS_PI = 64 / (DV / 8);
  static_assert(NWAVES % 4 == 0, "the direct-load lane offsets assume NWAVES % 4 == 0");
  static_assert(!(DIFF_ && RB_ != 1), "the two-stream path keeps one row block per wave");
  // Keys and values read in place from a paged cache (a chunk of query rows per sequence, Sec. 4.1 serving): every
  // direct-load instruction of a tile covers K_ROWS_PI consecutive tokens, which lie in one page (pages hold a power of two
  // >= K_ROWS_PI tokens), so per instruction only a uniform base address changes; the page numbers come from the
  // sequence's block table, fetched a step ahead.
  static constexpr bool PAGED = PAGED_;
  static_assert(!PAGED_ || (!DIFF_ && NBIAS_ == 0 && RING_ == 2 && D_ == DV_ && (MASK_ & (kMaskDoc | kMaskCustom)) == 0),
                "paged keys: one stream, no bias, two ring slots, D == Dv, positional masks");
  // Grouped-query heads packed into one workgroup (short chunks of query rows against long key sequences): the workgroup's BM
  // rows are BM / PACK rows of each of PACK consecutive query heads that share a kv head, so that K / V tiles are read
  // once for all of them and a chunk shorter than BM rows still fills the MFMA rows.  A wave's rows belong to one head.
  static constexpr int PACK = PACK_;
  static constexpr int HEAD_ROWS = BM / PACK_;     // query rows per head and workgroup
  static_assert(PACK_ == 1 || (!DIFF_ && NBIAS_ == 0 && EPI_ == 0 && (MASK_ & (kMaskDoc | kMaskCustom)) == 0 && MOD_ != kModCustom &&
                               BM % PACK_ == 0 && HEAD_ROWS % WROWS == 0),
                "packed heads: one stream, no bias, no epilogue, positional masks, whole waves per head");
};

enum TileClass : int { kTileSkip = 0, kTileFull = 1, kTilePartial = 2 };

template <class C>
struct Wave {
  static constexpr int D = C::D, DV = C::DV, NB = C::NB, KK = C::KK, DVB = C::DVB, NS = C::NS, RB = C::RB;
  static constexpr bool kPlain = (C::MOD == kModNone && C::NBIAS == 0);
  typedef f32x16 Scores[C::RB][C::NB];
  // Raw bias values of one tile for this lane: for bias n, row block rb, key block nb and
  // register group r4, the four bf16 values of keys jb + 8*r4 .. +3 (loaded ahead of their use).
  struct BiasRegs {
    uint2 v[C::NBIAS > 0 ? C::NBIAS : 1][C::RB][C::NB][4];
  };

  const FwdParams& p;
  const uint16_t* brow[C::NBIAS > 0 ? C::NBIAS : 1][C::RB];   // this lane's bias rows (bias, row block)
  // Bias tiles staged through LDS (BiasView::dma): a lane holds one query row, so reading its
  // bias values straight from global memory touches one cache line per lane for 8 useful bytes.
  // Instead each wave copies the [32 x BN] tile of its rows into a private LDS buffer with
  // coalesced direct loads, one key tile ahead, and every lane picks its values up from there.
  static constexpr int BROW_BYTES = C::BN * 2;                 // bytes of one staged bias row
  static constexpr int BCH = BROW_BYTES / 16;                  // 16-byte chunks per row
  static constexpr int BNI = 32 * BROW_BYTES / 1024;           // direct-load instructions per row block
  static constexpr int BSTAGE = 32 * C::RB * BROW_BYTES;       // bytes of one staging buffer
  const uint16_t* bsrc[C::NBIAS > 0 ? C::NBIAS : 1][C::RB][BNI];   // per-lane source of each load instruction (key 0)
  uint32_t brd[C::RB];          // per-lane LDS address of its row in staging buffer 0 of bias 0
  uint32_t bsw;                 // chunk swizzle of this lane's row
  uint32_t bstage;              // LDS byte offset of this wave's staging area (uniform)
  unsigned char* lds;           // the workgroup's LDS
  int lane, half, col;
  int b, g, h;
  int i[C::RB], ic[C::RB];      // this lane's query rows (unclamped / clamped), one per row block
  int qdoc[C::RB];
  float c_scale, slope_l2;
  float alibi_c[16];            // ALiBi, uniform: slope * key offset of score register r inside its 32-key block
  uint32_t ka[C::KK];           // per-lane byte offset of the K fragment of k-step kk (block 0)
  uint32_t va[C::DVB];          // per-lane byte offset of the V^T fragment of channel block d (key block 0)
  bf16x8 qf[C::RB][C::KK];      // Q fragments of the wave's rows (of its own stream, differential variant)
  f32x16 oacc[C::RB][C::DVB];
  float m_run[C::RB], l_run[C::RB];                // log2-domain running max; per-lane partial sum

  __device__ __forceinline__ Wave(const FwdParams& p_) : p(p_) {}

  static __device__ __forceinline__ f32x16 zero16() {
    return f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  }

  // The LDS fragment reads are issued by hand a few MFMAs ahead, with explicit lgkmcnt waits
  // (LDS returns in order).  The compiler then sees no LDS read in the loop: it cannot tie one
  // to the in-flight direct global->LDS loads of the next tile (it would wait for them), and the
  // number of live fragments is fixed.  "memory" keeps compiler-tracked memory accesses from
  // slipping between a read and its wait.
  template <int OFF>
  __device__ __forceinline__ void read_k(i32x4& dst, uint32_t addr) const {
    if constexpr (OFF <= 65535) {
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
    } else {
      const uint32_t a = addr + (uint32_t)OFF;
      asm volatile("ds_read_b128 %0, %1" : "=v"(dst) : "v"(a) : "memory");
    }
  }
  template <int OFF>
  __device__ __forceinline__ void read_vt(i32x2& lo, i32x2& hi, uint32_t addr) const {
    if constexpr (OFF + 8 * DV * 2 <= 65535) {
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(OFF) : "memory");
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(OFF + 8 * DV * 2) : "memory");
    } else {
      const uint32_t a = addr + (uint32_t)OFF;
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(a) : "memory");
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a), "n"(8 * DV * 2) : "memory");
    }
  }
  // Wait until at most N younger LDS operations are in flight.  The scheduling barrier keeps the
  // consumer of the fragment below the wait; no register operand ties the two together, because
  // the hazard checker treats every register an asm statement writes as freshly written by an
  // unknown instruction and pads the following MFMA with idle cycles.
  template <int N>
  static __device__ __forceinline__ void wait_lds() {
    static_assert(N >= 0 && N <= 15, "lgkmcnt is a 4-bit counter");
    asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(N) : "memory");
    __builtin_amdgcn_sched_barrier(0);
  }

  // ---- fragment streams.  A wave issues at most one instruction every few cycles whatever its
  // kind, so the loop is built to need few of them: fragments are read from LDS one group ahead
  // and one wait covers a whole group.  body(f, fragment) is called in fragment order.
  template <int KOFF, class Body>
  __device__ __forceinline__ void k_stream(Body&& body) const {
    constexpr int NF = NB * KK, G = C::GK < NF ? C::GK : NF, NG = NF / G;   // fragments (nb, kk)
    static_assert(NF % G == 0, "K fragment groups");
    i32x4 kf[NF];
    static_for<0, G>([&](auto f) __attribute__((always_inline)) { read_k<KOFF + (f / KK) * (32 * D * 2)>(kf[f], ka[f % KK]); });
    static_for<0, NG>([&](auto gc) __attribute__((always_inline)) {
      constexpr int g = gc;
      if constexpr (g + 1 < NG)
        static_for<(g + 1) * G, (g + 2) * G>([&](auto f) __attribute__((always_inline)) {
          read_k<KOFF + (f / KK) * (32 * D * 2)>(kf[f], ka[f % KK]);
        });
      wait_lds<(g + 1 < NG) ? G : 0>();
      static_for<g * G, (g + 1) * G>([&](auto f) __attribute__((always_inline)) { body(f, __builtin_bit_cast(bf16x8, kf[f])); });
    });
  }
  template <int VOFF, class Body>
  __device__ __forceinline__ void v_stream(Body&& body) const {
    constexpr int NF = NB * 2 * DVB, G = C::GV < NF ? C::GV : NF, NG = NF / G;   // fragments (nb, ks, d)
    static_assert(NF % G == 0, "V fragment groups");
    i32x2 lo[NF], hi[NF];
    static_for<0, G>([&](auto f) __attribute__((always_inline)) {
      read_vt<VOFF + (32 * (f / (2 * DVB)) + 16 * ((f / DVB) % 2)) * (DV * 2)>(lo[f], hi[f], va[f % DVB]);
    });
    static_for<0, NG>([&](auto gc) __attribute__((always_inline)) {
      constexpr int g = gc;
      if constexpr (g + 1 < NG)
        static_for<(g + 1) * G, (g + 2) * G>([&](auto f) __attribute__((always_inline)) {
          read_vt<VOFF + (32 * (f / (2 * DVB)) + 16 * ((f / DVB) % 2)) * (DV * 2)>(lo[f], hi[f], va[f % DVB]);
        });
      wait_lds<(g + 1 < NG) ? 2 * G : 0>();
      static_for<g * G, (g + 1) * G>([&](auto f) __attribute__((always_inline)) {
        body(f, __builtin_bit_cast(bf16x8, (i32x4){lo[f][0], lo[f][1], hi[f][0], hi[f][1]}));
      });
    });
  }

  // ---- first contraction: S^T = K Q^T for all row blocks, K tile at LDS offset KOFF
  template <int KOFF>
  __device__ __forceinline__ void qk(Scores& sc) const {
    f32x16 acc[RB];
    k_stream<KOFF>([&](auto fc, bf16x8 a) __attribute__((always_inline)) {
      constexpr int f = fc, kk = f % KK, nb = f / KK;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        if (kk == 0) acc[rb] = zero16();
        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][kk], acc[rb], 0, 0, 0);
        if (kk == KK - 1) sc[rb][nb] = acc[rb];
      }
    });
  }

  // ---- variant transform (Eq. 4 score_mod, additive biases) of one score register.
  // Leaves the score in the domain exp_only() expects: raw for the plain variants (the scale is
  // folded into the exponent's FMA), log2-scaled otherwise.  j0 is the tile's first key.
  __device__ __forceinline__ float transform_one(float x, int j0, int rb, int nb, int r, const BiasRegs& br) const {
    if constexpr (kPlain) {
      return x;
    } else {
      const int j = j0 + 32 * nb + 4 * half + 8 * (r >> 2) + (r & 3);   // key of register r
      if constexpr (C::MOD == kModSoftcap) {
        // cap*tanh(x*scale/cap) in the log2 domain; tanh(y) = 1 - 2/(exp(2y)+1)
        const float e = fast_exp2(x * (2.f * c_scale / p.softcap));
        const float cl = p.softcap * kLog2e;
        x = fmaf(fast_rcp(e + 1.f), -2.f * cl, cl);
      } else if constexpr (C::MOD == kModAlibi) {
        // slope * |i - j| with j = (j0 + 32*nb + 4*half) + c, c the register's compile-time key
        // offset: one per-lane term per key block minus a uniform constant per register, then one FMA
        // (all the integers involved are far below 2^24, so the float arithmetic is exact up
        // to the final rounding of the products)
        const float d = slope_l2 * (float)(i[rb] + p.q_off - j0 - 32 * nb - 4 * half);
        x = fmaf(x, c_scale, -fabsf(d - alibi_c[r]));
      } else if constexpr (C::MOD == kModCustom) {
        // (rows past Sq and keys past Sk are computed like the last valid ones and never used: an expression that
        // indexes a captured array by i or j must not be handed an index outside the call's sizes)
        // (FL_USER_CLAMP 0: the expressions capture no array, so any index is as good as another and the minimum per
        // score is saved)
        x = fl_user_score_mod(x * p.scale, b, g, h, ic[rb] + p.q_off, FL_USER_CLAMP && j >= p.Sk ? p.Sk - 1 : j, p) * kLog2e;
      } else {
        x *= c_scale;
      }
#pragma unroll
      for (int nbias = 0; nbias < C::NBIAS; ++nbias) {
        const uint2 q4 = br.v[nbias][rb][nb][r >> 2];
        const uint32_t wd = (r & 2) ? q4.y : q4.x;
        const float bb = __uint_as_float((r & 1) ? (wd & 0xFFFF0000u) : (wd << 16));
        x = fmaf(bb, kLog2e, x);
      }
      return x;
    }
  }
  __device__ __forceinline__ void transform(Scores& sc, int j0, const BiasRegs& br) const {
    if constexpr (!kPlain) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int r = 0; r < 16; ++r) sc[rb][nb][r] = transform_one(sc[rb][nb][r], j0, rb, nb, r, br);
    }
  }

  // ---- bias values of tile j0 for this lane, issued early so that their latency hides behind
  // the matrix work of the step.  Rows whose layout allows it are read four keys per load.
  // chunk swizzle of staged row r: spreads the rows that share LDS banks over different chunks
  static __device__ __forceinline__ uint32_t bias_swz(int r) { return (uint32_t)(BCH == 4 ? (r >> 2) : (r >> 1)) & (BCH - 1); }

  // start the copy of the bias tiles of key tile j0 into staging buffer BUF (full tiles only)
  template <int BUF>
  __device__ __forceinline__ void bias_dma(int j0) const {
#pragma unroll
    for (int nbias = 0; nbias < C::NBIAS; ++nbias) {
      if (p.bias[nbias].dma == 0 || j0 + C::BN > p.Sk) continue;   // uniform
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int u = 0; u < BNI; ++u) {
          lds_void* dst = (lds_void*)(lds + bstage + (nbias * 2 + BUF) * BSTAGE + rb * (32 * BROW_BYTES) + u * 1024);
          __builtin_amdgcn_global_load_lds((global_cvoid*)(bsrc[nbias][rb][u] + j0), dst, 16, 0, 0);
        }
    }
  }

  // bias values of tile j0 for this lane: from staging buffer BUF where the tile was staged, else
  // straight from global memory (issued early so that the latency hides behind the matrix work)
  template <int BUF>
  __device__ __forceinline__ void load_bias(BiasRegs& br, int j0) const {
#pragma unroll
    for (int nbias = 0; nbias < C::NBIAS; ++nbias) {
      const BiasView& bv = p.bias[nbias];
      if (bv.dma != 0 && j0 + C::BN <= p.Sk) {     // uniform
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
              const uint32_t a = brd[rb] + (((uint32_t)(4 * nb + r4) ^ bsw) << 4);
              i32x2 v;
              asm volatile("ds_read_b64 %0, %1 offset:%2" : "=v"(v) : "v"(a), "n"((nbias * 2 + BUF) * BSTAGE) : "memory");
              br.v[nbias][rb][nb][r4] = make_uint2((uint32_t)v[0], (uint32_t)v[1]);
            }
        continue;
      }
      const bool vec = bv.vec4 != 0 && j0 + C::BN <= p.Sk;       // uniform
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const int j = j0 + 32 * nb + 4 * half + 8 * r4;
            if (vec) {
              br.v[nbias][rb][nb][r4] = *(const uint2*)(brow[nbias][rb] + j);
            } else {
              uint32_t e[4];
#pragma unroll
              for (int u = 0; u < 4; ++u) e[u] = brow[nbias][rb][(int64_t)(j + u < p.Sk ? j + u : p.Sk - 1) * bv.sj];
              br.v[nbias][rb][nb][r4] = make_uint2(e[0] | (e[1] << 16), e[2] | (e[3] << 16));
            }
          }
    }
  }

  // ---- masks of a partially visible tile: hidden scores become -inf (attention listing).
  // A lane holds one query row per row block, and register r of key block nb holds key
  // j0 + 4*half + c with the compile-time offset c = 32*nb + 8*(r/4) + r%4.  The positional masks
  // and the end of the key range are therefore two per-lane bounds on c: hidden iff c > d_hi
  // (causal: j > i; PrefixLM: j > max(i, prefix - 1); always: j > Sk - 1) or c < d_lo (window:
  // i - j > window) -- one or two compares per score instead of evaluating every mask on (i, j).
  // `word` (mask expressions with a precomputed map only): bit 16*nb + r set = this lane's score register r of key block
  // nb is hidden; then nothing is evaluated here.
  __device__ __forceinline__ void mask(Scores& sc, int j0, uint32_t word = 0) const {
    constexpr uint32_t MASK = C::MASK;
    if constexpr ((MASK & kMaskCustom) != 0) {
      if (p.block_bits != nullptr) {               // uniform
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if ((word >> (16 * nb + r)) & 1u) sc[rb][nb][r] = -INFINITY;
        return;
      }
    }
    const int jl = j0 + 4 * half;
    int d_hi[RB], d_lo[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const int ip = i[rb] + p.q_off;              // the row's sequence position
      int last = p.Sk - 1;                         // last visible key of the row
      if constexpr ((MASK & kMaskPrefix) != 0) last = min(last, max(ip, p.prefix - 1));
      else if constexpr ((MASK & (kMaskCausal | kMaskWindow)) != 0) last = min(last, ip);
      d_hi[rb] = last - jl;
      d_lo[rb] = (MASK & kMaskWindow) != 0 ? ip - p.window - jl : 0;
    }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      int kd[16];
      if constexpr ((MASK & kMaskDoc) != 0) {
        const int32_t* kdoc = p.kv_doc + (int64_t)b * p.Sk;
        const int jb = jl + 32 * nb;
        if (p.doc_vec && j0 + C::BN <= p.Sk) {     // uniform: four ids per load
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const int4 q4 = *(const int4*)(kdoc + jb + 8 * r4);
            kd[4 * r4] = q4.x; kd[4 * r4 + 1] = q4.y; kd[4 * r4 + 2] = q4.z; kd[4 * r4 + 3] = q4.w;
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = jb + 8 * (r >> 2) + (r & 3);
            kd[r] = kdoc[j < p.Sk ? j : p.Sk - 1];
          }
        }
      }
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = 32 * nb + 8 * (r >> 2) + (r & 3);
          bool hide = c > d_hi[rb];
          if constexpr ((MASK & kMaskWindow) != 0) hide = hide || c < d_lo[rb];
          if constexpr ((MASK & kMaskDoc) != 0) hide = hide || kd[r] != qdoc[rb];
          if constexpr ((MASK & kMaskCustom) != 0)  // (valid indices only, as for the score_mod; a key past Sk is hidden already)
            hide = hide || fl_user_mask(b, g, h, ic[rb] + p.q_off, FL_USER_CLAMP && jl + c >= p.Sk ? p.Sk - 1 : jl + c, p);
          if (hide) sc[rb][nb][r] = -INFINITY;
        }
    }
  }

  // ---- row max of the tile in log2 units, one per row block
  __device__ __forceinline__ void rowmax(const Scores& sc, float (&mx)[C::RB]) const {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float m = -INFINITY;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) m = fmaxf(m, sc[rb][nb][r]);
      m = half_swap_max(m);
      if constexpr (kPlain) m *= c_scale;          // scale > 0 (checked on the host)
      mx[rb] = m;
    }
  }

  // ---- running-max update with the next tile's row maxima (Alg. 2 / Sec. 3.4) and
  // the rescale of l and O that goes with it.  The max of a row only advances when it grows by
  // more than 2^kLazyMaxLog2, so the O rescale is a rare, wave-uniform branch.
  __device__ __forceinline__ void advance_max(const float (&mx)[C::RB]) {
    float alpha[RB];
    bool any = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const float m_old = m_run[rb];
      const float m_new = (mx[rb] - m_old > kLazyMaxLog2) ? mx[rb] : m_old;   // false for NaN (-inf - -inf)
      const bool moved = m_new != m_old;
      alpha[rb] = moved ? fast_exp2(m_old - (m_new == -INFINITY ? 0.f : m_new)) : 1.f;
      m_run[rb] = m_new;
      l_run[rb] *= alpha[rb];
      any = any || moved;
    }
    if (__builtin_amdgcn_ballot_w64(any) != 0) {
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int d = 0; d < DVB; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[rb][d][r] *= alpha[rb];
    }
  }

  // ---- one probability pair: p = exp2(s - m); then running row sum and bf16 pair (and remainder)
  __device__ __forceinline__ void exp_only(float s0, float s1, float m_safe, float& p0, float& p1) const {
    if constexpr (kPlain) {
      p0 = fast_exp2(fmaf(s0, c_scale, -m_safe));
      p1 = fast_exp2(fmaf(s1, c_scale, -m_safe));
    } else {
      p0 = fast_exp2(s0 - m_safe);
      p1 = fast_exp2(s1 - m_safe);
    }
  }
  __device__ __forceinline__ void sum_pack(float p0, float p1, float& psum, uint32_t& w, uint32_t& wl) const {
    psum += p0 + p1;
    w = pack_bf16(p0, p1);
    if constexpr (C::PSPLIT) wl = pack_bf16(p0 - __uint_as_float(w << 16), p1 - __uint_as_float(w & 0xFFFF0000u));
  }

  // ---- software pipeline.  A wave issues at most one vector or
  // matrix instruction every few cycles, so what bounds a step is the number of instructions of
  // each phase; the softmax work of a tile is therefore cut in two halves of equal length:
  //   phase A:  QK MFMAs of the next tile  +  exponentials of the first half of the current tile
  //             (the half the second contraction consumes first), then the transform / row max
  //             of the next tile's first key block, which is complete by then;
  //   phase B:  PV MFMAs of the current tile  +  exponentials of its second half during the
  //             MFMAs that consume the first, then the transform / row max of the next tile's
  //             last key block and the running-max update (Alg. 2 / Sec. 3.4).
  // The sum / bf16 conversion of a pair follows one pair after its exponentials (a
  // transcendental result cannot be consumed by the very next instruction without an idle
  // cycle).  Scheduling barriers pin the order; the empty asm statement keeps the sum and the
  // conversion from being sunk out of the loop body.
  struct Pipe {
    uint32_t w[C::RB][C::NB][8];   // bf16 pairs of the current tile's probabilities
    uint32_t wl[C::PSPLIT ? C::NB : 1][8];   // their bf16 remainders (PSPLIT implies RB == 1)
    float e0, e1;                  // the pair of exponentials whose sum / conversion is still due
    float psum[C::RB], m_safe[C::RB];
    float mx[C::RB];               // row maxima of the next tile so far
  };
  static constexpr int NPAIR = C::RB * C::NB * 8;  // probability pairs of a tile per lane
  static_assert(NB == 1 || NB == 2, "the pipeline splits a tile into at most two key blocks");

  // pair q in the order the second contraction needs them: (key block, k-step) major, then row block
  __device__ __forceinline__ void exp_step(const Scores& cur, Pipe& ps, int q, int q_first) {
    const int h = q / (4 * RB), rb = (q / 4) % RB, nb = h / 2, r2 = (h % 2) * 4 + q % 4;
    float n0, n1;
    exp_only(cur[rb][nb][2 * r2], cur[rb][nb][2 * r2 + 1], ps.m_safe[rb], n0, n1);
    if (q > q_first) finish_pair(ps, q - 1);
    ps.e0 = n0;
    ps.e1 = n1;
  }
  __device__ __forceinline__ void finish_pair(Pipe& ps, int q) {
    const int h = q / (4 * RB), rb = (q / 4) % RB, nb = h / 2, r2 = (h % 2) * 4 + q % 4;
    if constexpr (C::PSPLIT) {
      sum_pack(ps.e0, ps.e1, ps.psum[rb], ps.w[rb][nb][r2], ps.wl[nb][r2]);
      asm volatile("" : "+v"(ps.w[rb][nb][r2]), "+v"(ps.wl[nb][r2]), "+v"(ps.psum[rb]));
    } else {
      uint32_t unused = 0;
      sum_pack(ps.e0, ps.e1, ps.psum[rb], ps.w[rb][nb][r2], unused);
      asm volatile("" : "+v"(ps.w[rb][nb][r2]), "+v"(ps.psum[rb]));
    }
  }
  // two scores of key block nb of the next tile: variant transform in place, row max
  __device__ __forceinline__ void max_step(Scores& nxt, Pipe& ps, int nb, int L, int j1, const BiasRegs& br) {
    const int rb = L / 16, r = L % 16;
    const float x0 = transform_one(nxt[rb][nb][r], j1, rb, nb, r, br);
    const float x1 = transform_one(nxt[rb][nb][r + 1], j1, rb, nb, r + 1, br);
    nxt[rb][nb][r] = x0;
    nxt[rb][nb][r + 1] = x1;
    ps.mx[rb] = fmaxf(fmaxf(ps.mx[rb], x0), x1);
  }

  // hook(f) runs after the work of fragment f: the caller's tile loads.
  template <int KOFF, class Hook>
  __device__ __forceinline__ void phase_a(Scores& nxt, const Scores& cur, Pipe& ps, int j1, const BiasRegs& br,
                                          Hook&& hook) {
    constexpr int NF = NB * KK;
    constexpr int SE = (NB == 2 ? KK : NF) * RB;   // slots (fragment, row block) that carry exponentials
    constexpr int PA = NPAIR / 2;                  // pairs of the first half
    constexpr int SM = NF * RB - SE;               // slots that carry the max of key block 0 (NB == 2)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      ps.m_safe[rb] = m_run[rb] == -INFINITY ? 0.f : m_run[rb];
      ps.psum[rb] = 0.f;
      ps.mx[rb] = -INFINITY;
    }
    f32x16 acc[RB];
    k_stream<KOFF>([&](auto fc, bf16x8 a) __attribute__((always_inline)) {
      constexpr int f = fc, kk = f % KK, nb = f / KK;
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        if (kk == 0) acc[rb] = zero16();
        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][kk], acc[rb], 0, 0, 0);
        if (kk == KK - 1) nxt[rb][nb] = acc[rb];
        const int slot = f * RB + rb;
        if (slot < SE) {
#pragma unroll
          for (int q = slot * PA / SE; q < (slot + 1) * PA / SE; ++q) exp_step(cur, ps, q, 0);
        } else {
          const int sm = slot - SE;                // pairs of scores of key block 0, all row blocks
#pragma unroll
          for (int u = sm * (8 * RB) / (SM > 0 ? SM : 1); u < (sm + 1) * (8 * RB) / (SM > 0 ? SM : 1); ++u)
            max_step(nxt, ps, 0, 2 * u, j1, br);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      hook(fc);
      __builtin_amdgcn_sched_barrier(0);
    });
    finish_pair(ps, PA - 1);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) asm volatile("" : "+v"(ps.mx[rb]));   // block 0's maxima stay in this phase
  }

  // `advance` (uniform) is false when the next tile still needs its mask: then the running-max
  // update is left to the start of the next step.  The O rescale is a rare branch at the end.
  template <int VOFF>
  __device__ __forceinline__ void phase_b(Pipe& ps, const Scores& cur, Scores& nxt, int j1, const BiasRegs& br,
                                          bool advance) {
    constexpr int NF = NB * 2 * DVB, HALF = NF / 2;
    constexpr int SE = HALF * RB, SM = NF * RB - SE, PA = NPAIR / 2;
    static_assert(NF % 2 == 0, "chunking");
    v_stream<VOFF>([&](auto fc, bf16x8 a) __attribute__((always_inline)) {
      constexpr int f = fc, d = f % DVB, ks = (f / DVB) % 2, nb = f / (2 * DVB);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const int slot = f * RB + rb;
        if (slot == SE) finish_pair(ps, NPAIR - 1);
        const bf16x8 pb = __builtin_bit_cast(bf16x8, (i32x4){(int)ps.w[rb][nb][4 * ks], (int)ps.w[rb][nb][4 * ks + 1],
                                                             (int)ps.w[rb][nb][4 * ks + 2], (int)ps.w[rb][nb][4 * ks + 3]});
        oacc[rb][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, oacc[rb][d], 0, 0, 0);
        if constexpr (C::PSPLIT) {
          const bf16x8 pl = __builtin_bit_cast(bf16x8, (i32x4){(int)ps.wl[nb][4 * ks], (int)ps.wl[nb][4 * ks + 1],
                                                               (int)ps.wl[nb][4 * ks + 2], (int)ps.wl[nb][4 * ks + 3]});
          oacc[rb][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pl, oacc[rb][d], 0, 0, 0);
        }
        if (slot < SE) {
#pragma unroll
          for (int q = PA + slot * PA / SE; q < PA + (slot + 1) * PA / SE; ++q) exp_step(cur, ps, q, PA);
        } else {
          const int sm = slot - SE;                // pairs of scores of the last key block
#pragma unroll
          for (int u = sm * (8 * RB) / SM; u < (sm + 1) * (8 * RB) / SM; ++u) max_step(nxt, ps, NB - 1, 2 * u, j1, br);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    });
    // the tile's row sums are complete; fold the next tile's row maxima into the running state
    float alpha[RB];
    bool any = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      l_run[rb] += ps.psum[rb];
      float mxs = half_swap_max(ps.mx[rb]);
      if constexpr (kPlain) mxs *= c_scale;        // scale > 0 (checked on the host)
      const float m_old = m_run[rb];
      float m_new = (mxs - m_old > kLazyMaxLog2) ? mxs : m_old;   // false for NaN (-inf - -inf)
      m_new = advance ? m_new : m_old;
      const bool moved = m_new != m_old;
      alpha[rb] = moved ? fast_exp2(m_old - (m_new == -INFINITY ? 0.f : m_new)) : 1.f;
      m_run[rb] = m_new;
      l_run[rb] *= alpha[rb];
      any = any || moved;
    }
    if (__builtin_amdgcn_ballot_w64(any) != 0) {   // rare and wave-uniform
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int d = 0; d < DVB; ++d)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[rb][d][r] *= alpha[rb];
    }
  }
};

template <class C>
__global__ void __launch_bounds__(C::NT) __attribute__((amdgpu_waves_per_eu(C::WPE, C::WPE)))
fwd_bf16_kernel(const FwdParams call) {
  constexpr int D = C::D, DV = C::DV, BN = C::BN, NB = C::NB, KK = C::KK, DVB = C::DVB, NS = C::NS, RB = C::RB;
  constexpr uint32_t MASK = C::MASK;
  typedef Wave<C> W;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];

  const int tid = threadIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

  // ---- logical grid decode (Sec. 3.6): 1-D launch -> (b, g, h, q-tile or pair of q-tiles).
  // With p.pair a workgroup takes q-tile nq - 1 - pi and then q-tile pi: under a causal mask the
  // two together see the same number of key tiles for every pi, so all workgroups carry the same
  // load and the launch has no tail of long stragglers.  Without it, q-tiles go out longest first.
  const int nq = call.n_qtiles, npairs = call.pair ? (nq + 1) / 2 : nq;
  int bid = blockIdx.x;
  int pi, bh;
  if (call.order == 1) {
    // XCD-aware: consecutive workgroup ids go round-robin to the 8 XCDs; give each XCD whole
    // (b, g, h) problems so that a head's K/V stay in one L2 (host checks (B*G*H) % 8 == 0).
    const int xcd = bid & 7;
    const int idx = bid >> 3;
    bh = (idx / npairs) * 8 + xcd;
    pi = idx % npairs;
  } else {
    pi = bid % npairs;
    bh = bid / npairs;
  }
  // The problem as this workgroup sees it.  With per-sequence key counts (a chunk of new query rows against each
  // sequence's cached keys, Sec. 4.1 serving) sequence b has kv_lens[b] keys, cut to [0, Sk], and its query rows are the
  // last Sq positions of those: row i sits at position kv_lens[b] - Sq + i (rows at negative positions see nothing).
  // (packed heads: bh counts groups of PACK heads)
  const int heads_wg = call.H / C::PACK;
  FwdParams p = call;
  if (call.kv_lens != nullptr) {
    const int len = max(0, min(call.kv_lens[bh / (heads_wg * call.G)], call.Sk));
    p.Sk = len;
    p.q_off = len - call.Sq;
  }
  W w(p);
#pragma nounroll
  for (int pass = 0; pass < 2; ++pass) {
  const int qt = pass == 0 ? nq - 1 - pi : pi;
  if (pass == 1 && (!p.pair || qt == nq - 1 - pi)) break;   // odd tile count: the middle tile has no partner
  if (pass == 1) __syncthreads();                  // LDS is reused by the second tile
  // Everything per-lane is derived again for each tile from this opaque copy of the lane id:
  // otherwise the loop-invariant part of it is hoisted out of the tile loop and stays live in
  // registers that the main loop needs.
  int lane = tid & 63;
  asm volatile("" : "+v"(lane));
  w.lane = lane;
  w.half = lane >> 5;
  w.col = lane & 31;
  const int wrow = (wave % C::NROWG) * C::WROWS;   // the wave's first row among the workgroup's BM
  const int h = (bh % heads_wg) * C::PACK + wrow / C::HEAD_ROWS;   // (one head per workgroup unless heads are packed)
  const int g = (bh / heads_wg) % p.G;
  const int b = bh / (heads_wg * p.G);
  const int hk = h / (p.H / p.Hkv);                // the same for all heads of a pack (the host checks)
  const int stream = C::DIFF ? wave / C::NROWG : 0;   // softmax stream of this wave (uniform)
  const int i0 = qt * C::HEAD_ROWS;                // first query row of the workgroup
  const int iw = i0 + wrow % C::HEAD_ROWS;         // first query row of the wave
  w.b = b; w.g = g; w.h = h;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    w.i[rb] = iw + 32 * rb + w.col;
    w.ic[rb] = w.i[rb] < p.Sq ? w.i[rb] : p.Sq - 1;
    const View& qv = stream == 0 ? p.q : p.q2;     // the wave's own stream
    const uint16_t* qp = (const uint16_t*)qv.ptr + b * qv.sb + g * qv.sg + h * qv.sh + (int64_t)w.ic[rb] * qv.ss;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) w.qf[rb][kk] = *(const bf16x8*)(qp + 16 * kk + 8 * w.half);
    w.qdoc[rb] = 0;
    if constexpr ((MASK & kMaskDoc) != 0) w.qdoc[rb] = p.q_doc[(int64_t)b * p.Sq + w.ic[rb]];
#pragma unroll
    for (int nbias = 0; nbias < C::NBIAS; ++nbias) {
      const BiasView& bv = p.bias[nbias];
      const uint16_t* bhead = (const uint16_t*)bv.ptr + b * bv.sb + g * bv.sg + h * bv.sh;
      w.brow[nbias][rb] = bhead + (int64_t)w.ic[rb] * bv.si;
#pragma unroll
      for (int u = 0; u < W::BNI; ++u) {           // staging: this lane's source row and chunk of load instruction u
        const int r = u * (64 / W::BCH) + lane / W::BCH;
        const int ir = iw + 32 * rb + r < p.Sq ? iw + 32 * rb + r : p.Sq - 1;
        w.bsrc[nbias][rb][u] = bhead + (int64_t)ir * bv.si + (((uint32_t)(lane % W::BCH) ^ W::bias_swz(r)) << 3);
      }
    }
    w.brd[rb] = p.bias_lds_base + wave * p.bias_lds_wave + rb * (32 * W::BROW_BYTES) + w.col * W::BROW_BYTES + w.half * 8;
  }
  w.bsw = W::bias_swz(w.col);
  w.bstage = p.bias_lds_base + wave * p.bias_lds_wave;
  w.lds = lds_raw;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    w.m_run[rb] = -INFINITY;
    w.l_run[rb] = 0.f;
#pragma unroll
    for (int d = 0; d < DVB; ++d) w.oacc[rb][d] = W::zero16();
  }
  w.c_scale = p.scale * kLog2e;                    // raw score -> log2 domain
  w.slope_l2 = 0.f;
  if constexpr (C::MOD == kModAlibi) {
    w.slope_l2 = p.alibi_slopes[h] * kLog2e;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int c = 8 * (e >> 2) + (e & 3);
      w.alibi_c[e] = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(w.slope_l2 * (float)c)));
    }
  }

  // ---- loop-invariant per-lane LDS offsets
#pragma unroll
  for (int kk = 0; kk < KK; ++kk)                  // K ring slot layout: [stream][tile]; a wave reads its stream's tile
    w.ka[kk] = stream * C::K_BYTES + w.col * (D * 2) + swz_k<D>(w.col, 2 * kk + w.half) * 16;
  {
    const int s16 = lane & 15;
    const int key0 = 4 * w.half + (s16 >> 2);      // row this lane addresses in the transposing read
#pragma unroll
    for (int d = 0; d < DVB; ++d) {
      const int ch = 32 * d + 16 * ((lane >> 4) & 1) + 4 * (s16 & 3);   // first of its 4 channels
      // (the ring's base is part of the address register, so that the immediate offsets of the reads stay below 64 KiB)
      w.va[d] = C::V_RING + key0 * (DV * 2) + swz_v<DV>(key0, ch >> 3) * 16 + (ch & 7) * 2;
    }
  }

  // ---- tile skipper (a0): visible key range and document-id summaries
  const int i_last = (i0 + C::HEAD_ROWS - 1 < p.Sq ? i0 + C::HEAD_ROWS : p.Sq) - 1;
  // positions of the workgroup's / the wave's first and last query row: what the positional masks compare with keys
  const int pos0 = i0 + p.q_off, pos_last = i_last + p.q_off, posw = iw + p.q_off;
  int k_lo, k_hi;
  key_range(MASK, pos0, pos_last, p.Sk, p.window, p.prefix, k_lo, k_hi);
  const int t_lo = k_lo / BN;
  const int t_hi = (k_hi + BN - 1) / BN;
  const int nks = (p.Sk + kSumBlock - 1) / kSumBlock;
  // Query-side summaries of the workgroup's and of the wave's rows.  All of them are requested before any is used (past
  // the last block: the last block again, which changes no minimum or maximum), and so are, further down, the key-side
  // answers for the first tiles: the set-up then waits for memory once.
  int2 qs_wg = make_int2(0, 0), qs_wave = make_int2(0, 0);
  constexpr int NQW = C::BM / kSumBlock;
  int2 qraw_wg[NQW], qraw_wave[RB];
  if constexpr ((MASK & kMaskDoc) != 0) {
    const int nqs = (p.Sq + kSumBlock - 1) / kSumBlock;
    const int2* qsum = p.q_sum + (int64_t)b * nqs;
    const int s0 = i0 / kSumBlock, sw = iw / kSumBlock;
#pragma unroll
    for (int ww = 0; ww < NQW; ++ww) qraw_wg[ww] = qsum[min(s0 + ww, nqs - 1)];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) qraw_wave[rb] = qsum[min(sw + rb, nqs - 1)];
  }
  const int2* ksum = (MASK & kMaskDoc) ? p.kv_sum + (int64_t)b * nks : nullptr;
  // A mask given as an expression can come with a map of tile classes, written by block_map_kernel below: one byte per
  // (32-row query block, BN-key tile) -- 0 nothing visible, 1 some, 2 all -- stored [problem][tile][query block] so that
  // the blocks of a workgroup are bytes of one aligned 8-byte word.  Without a map every tile counts as "some".
  constexpr bool kMapped = (MASK & kMaskCustom) != 0;
  static_assert(!kMapped || (RB == 1 && !C::DIFF && C::NROWG <= 8), "tile-class bytes: one per wave, at most eight per workgroup");
  const bool mapped = kMapped && p.block_map != nullptr;
  const unsigned char* mrow = nullptr;             // the word of this workgroup's query blocks in tile 0
  const uint32_t* brow_bits = nullptr;             // this lane's word of hidden-score bits in tile 0 (if the map has them)
  int map_shift = 0;
  if constexpr (kMapped) {
    if (mapped) {
      const int64_t prob = p.map_per_head ? ((int64_t)b * p.G + g) * p.H + h : b;
      const int qb0 = i0 / 32;
      mrow = p.block_map + prob * p.map_nkt * p.map_nqb8 + (qb0 & ~7);
      map_shift = (qb0 & 7) * 8;
      if (p.block_bits != nullptr) brow_bits = p.block_bits + (prob * p.map_nkt * p.map_nqb8 + iw / 32) * 64 + lane;
    }
  }
  // the lane's hidden-score bits of tile t: one coalesced dword per lane
  auto tile_bits_lane = [&](int t) __attribute__((always_inline)) -> uint32_t {
    if constexpr (kMapped) {
      if (brow_bits != nullptr) return brow_bits[(int64_t)min(t, p.map_nkt - 1) * p.map_nqb8 * 64];
    }
    return 0u;
  };
  // the class bytes of this workgroup's query blocks, byte n = wave n's block
  auto my_classes = [&](int2 ks) __attribute__((always_inline)) -> unsigned long long {
    const unsigned long long word = (unsigned long long)(uint32_t)ks.x | ((unsigned long long)(uint32_t)ks.y << 32);
    constexpr unsigned long long keep = C::NROWG >= 8 ? ~0ull : ((1ull << (8 * (C::NROWG & 7))) - 1);
    return (word >> map_shift) & keep;
  };

  // What the skipper knows about tile t (t per lane): the document-id range of its keys, or its word of class bytes.
  auto tile_keys_lane = [&](int t) __attribute__((always_inline)) -> int2 {
    if constexpr (kMapped) {
      if (!mapped) return make_int2(0x01010101, 0x01010101);
      return *(const int2*)(mrow + (int64_t)min(t, p.map_nkt - 1) * p.map_nqb8);
    } else {
      int2 ks = ksum[min(t * NB, nks - 1)];
#pragma unroll
      for (int u = 1; u < NB; ++u)
        if (t * NB + u < nks) {
          const int2 x = ksum[t * NB + u];
          ks.x = min(ks.x, x.x);
          ks.y = max(ks.y, x.y);
        }
      return ks;
    }
  };
  // The same for a uniform t, waiting for the answer: set-up and the search after a run of hidden tiles only.
  auto tile_keys = [&](int t) __attribute__((always_inline)) -> int2 {
    const int2 ks = tile_keys_lane(t);
    return make_int2(__builtin_amdgcn_readfirstlane(ks.x), __builtin_amdgcn_readfirstlane(ks.y));
  };
  // Inside the loop the answer for the tile that the stream will most likely take next is fetched a whole step ahead, with
  // ordinary vector loads (every lane reads the same address).  Vector memory operations complete in order and every step
  // of these kernels ends with a wait for all of this wave's loads, so the answer has arrived by the time it is needed,
  // without a wait of its own.  (Scalar loads cannot be left in flight across a step: they share a counter with the LDS
  // reads, whose counted waits rely on in-order return.)
  int2 kpre[NB];                                   // what those loads return
  uint32_t bpre = 0;                               // ... and the lane's hidden-score bits of that tile (mapped expressions)
  int tpre = -1;                                   // the tile they belong to (uniform)
#pragma unroll
  for (int u = 0; u < NB; ++u) kpre[u] = make_int2(0, 0);
  auto prefetch_keys = [&](int t) __attribute__((always_inline)) {
    tpre = t;
    if constexpr (kMapped) {
      kpre[0] = tile_keys_lane(t);
      bpre = tile_bits_lane(t);
    } else {
#pragma unroll
      for (int u = 0; u < NB; ++u) kpre[u] = ksum[min(t * NB + u, nks - 1)];
    }
  };
  auto fetched_keys = [&]() __attribute__((always_inline)) -> int2 {
    int2 ks = kpre[0];
    if constexpr (!kMapped) {
#pragma unroll
      for (int u = 1; u < NB; ++u)
        if (tpre * NB + u < nks) {
          ks.x = min(ks.x, kpre[u].x);
          ks.y = max(ks.y, kpre[u].y);
        }
    }
    return make_int2(__builtin_amdgcn_readfirstlane(ks.x), __builtin_amdgcn_readfirstlane(ks.y));
  };
  // Set-up: what the skipper knows about the first tiles of the range, requested in one go (with the loads of Q and of
  // the query-side summaries, before anything waits), so that building the first tile list costs one memory round
  // trip instead of one per tile.
  constexpr int NPF = 4;
  int2 kfirst[NPF];
  uint32_t bfirst[NPF];
  if constexpr ((MASK & kMaskDoc) != 0 || kMapped) {
#pragma unroll
    for (int u = 0; u < NPF; ++u) {
      kfirst[u] = tile_keys_lane(t_lo + u);
      bfirst[u] = tile_bits_lane(t_lo + u);
    }
  }
  if constexpr ((MASK & kMaskDoc) != 0) {
    qs_wg = qraw_wg[0];
#pragma unroll
    for (int ww = 1; ww < NQW; ++ww) {
      qs_wg.x = min(qs_wg.x, qraw_wg[ww].x);
      qs_wg.y = max(qs_wg.y, qraw_wg[ww].y);
    }
    qs_wave = qraw_wave[0];
#pragma unroll
    for (int rb = 1; rb < RB; ++rb) {
      qs_wave.x = min(qs_wave.x, qraw_wave[rb].x);
      qs_wave.y = max(qs_wave.y, qraw_wave[rb].y);
    }
  }
  auto first_keys = [&](int t, uint32_t& bw) __attribute__((always_inline)) -> int2 {   // t_lo <= t < t_lo + NPF, uniform
    int2 ks = kfirst[0];
    bw = bfirst[0];
#pragma unroll
    for (int u = 1; u < NPF; ++u)
      if (t - t_lo == u) {
        ks = kfirst[u];
        bw = bfirst[u];
      }
    return make_int2(__builtin_amdgcn_readfirstlane(ks.x), __builtin_amdgcn_readfirstlane(ks.y));
  };
  // Is every score of tile t hidden from the workgroup's rows?  (t and ks may be per lane)
  auto tile_hidden = [&](int t, int2 ks) __attribute__((always_inline)) -> bool {
    if constexpr (kMapped) return my_classes(ks) == 0;
    else return classify_block(MASK, pos0, pos_last, t * BN, t * BN + BN - 1, p.Sk, p.window, p.prefix, qs_wg, ks) == kSkip;
  };
  // First tile at or after t with something visible to the workgroup (t_hi if none), and what the skipper knows about it.
  // (setup: called while the first tile list is built, when the answers for the first NPF tiles are at hand)
  auto next_tile = [&](int t, int2& ks, uint32_t& bw, auto setup) __attribute__((always_inline)) -> int {   // uniform over the workgroup
    ks = make_int2(0, 0);
    bw = 0;
    if constexpr ((MASK & kMaskDoc) != 0 || kMapped) {
      if (t < t_hi) {
        if (decltype(setup)::value && t < t_lo + NPF) {
          ks = first_keys(t, bw);
        } else {
          bw = t == tpre ? bpre : tile_bits_lane(t);
          ks = t == tpre ? fetched_keys() : tile_keys(t);
        }
        // the usual case first: tile t itself has something visible (one uniform check)
        if (tile_hidden(t, ks)) {
          // a run of hidden tiles (the other documents of a long sequence): 64 tiles per round, one per lane
          ++t;
          while (t < t_hi) {
            const int tt = t + w.lane;
            bool keep = false;
            if (tt < t_hi) keep = !tile_hidden(tt, tile_keys_lane(tt));
            const unsigned long long found = __builtin_amdgcn_ballot_w64(keep);
            if (found != 0) {
              t += __builtin_ctzll(found);
              break;
            }
            t += 64;
          }
          t = __builtin_amdgcn_readfirstlane(t < t_hi ? t : t_hi);
          if (t < t_hi) {
            ks = tile_keys(t);
            bw = tile_bits_lane(t);
          }
        }
        if (t < t_hi) prefetch_keys(t + 1);
      }
    }
    return t;                                      // positional masks are already in [t_lo, t_hi)
  };
  int tf_lo = 0, tf_hi = 0;                        // tiles fully visible to this wave's rows (positional masks)
  full_tile_range(MASK, posw, posw + C::WROWS - 1, p.Sk, p.window, p.prefix, BN, tf_lo, tf_hi);
  tf_lo = __builtin_amdgcn_readfirstlane(tf_lo);
  tf_hi = __builtin_amdgcn_readfirstlane(min(tf_hi, t_hi));
  // Tiles that hold a visible key of some row of this wave (positional masks): outside of
  // [tv_lo, tv_hi) every score of the wave is hidden, which needs no per-score mask arithmetic.
  constexpr bool kWaveSkip = (MASK & (kMaskCausal | kMaskWindow | kMaskPrefix)) != 0 &&
                             (MASK & (kMaskDoc | kMaskCustom)) == 0;
  int tv_lo = 0, tv_hi = 0;
  if constexpr (kWaveSkip) {
    int lo, hi;
    key_range(MASK, posw, posw + C::WROWS - 1, p.Sk, p.window, p.prefix, lo, hi);
    tv_lo = __builtin_amdgcn_readfirstlane(lo / BN);
    tv_hi = __builtin_amdgcn_readfirstlane((hi + BN - 1) / BN);
  }
  auto wave_class = [&](int t, int2 ks) __attribute__((always_inline)) -> int {   // uniform over the wave; ks: the tile's id range
    if (t >= t_hi) return kTileSkip;
    const int c = classify_block(MASK, posw, posw + C::WROWS - 1, t * BN, t * BN + BN - 1, p.Sk, p.window, p.prefix,
                                 qs_wave, ks);
    return __builtin_amdgcn_readfirstlane(c);
  };

  auto wave_full = [&](int t, int2 ks) __attribute__((always_inline)) -> bool {   // is tile t fully visible to the wave?
    if constexpr (kMapped) {                       // an arbitrary predicate: evaluated on every score unless the map says "all"
      if (t >= t_hi) return false;
      return ((my_classes(ks) >> (8 * (wave % C::NROWG))) & 0xffull) == 2;
    }
    if constexpr ((MASK & kMaskDoc) != 0) return wave_class(t, ks) == kTileFull;
    else return t >= tf_lo && t < tf_hi;
  };

  // ---- direct global -> LDS loads of one K or V tile (a2): every wave instruction moves
  // 64 x 16 B into 1 KiB of consecutive LDS; the swizzle is applied by choosing which global
  // chunk each lane fetches, which is the same for every instruction of a lane.  Rows past Sk
  // are clamped to the last row (their scores are masked, their probabilities exactly 0).
  const unsigned char* kbase[NS];
  kbase[0] = (const unsigned char*)((const uint16_t*)p.k.ptr + b * p.k.sb + g * p.k.sg + hk * p.k.sh);
  if constexpr (C::DIFF)
    kbase[NS - 1] = (const unsigned char*)((const uint16_t*)p.k2.ptr + b * p.k2.sb + g * p.k2.sg + hk * p.k2.sh);
  const int64_t kss[2] = {p.k.ss * 2, C::DIFF ? p.k2.ss * 2 : 0};   // row strides in bytes
  const unsigned char* vbase = (const unsigned char*)((const uint16_t*)p.v.ptr + b * p.v.sb + g * p.v.sg + hk * p.v.sh);
  const int64_t vss = p.v.ss * 2;
  const int kr_lane = lane / (D / 8), vr_lane = lane / (DV / 8);     // row within an instruction

  // This wave issues instructions wave, wave + NWAVES, ... of a tile (wrapping around when a tile
  // has fewer instructions than the workgroup has waves: the duplicates rewrite the same bytes).
  // The byte offset of a lane inside the tile is loop invariant and fits 32 bits (the host bounds
  // the row stride); per tile only a uniform 64-bit base changes.  In a ragged last tile the
  // lanes whose row is past Sk take row Sk - 1 instead: clamp_k / clamp_v rewrite the offsets
  // then, once, because tiles are visited in increasing order and nothing follows a ragged one.
  constexpr int KPW = (C::K_INSTR + C::NWAVES - 1) / C::NWAVES, VPW = (C::V_INSTR + C::NWAVES - 1) / C::NWAVES;
  uint32_t k_off[NS][KPW], v_off[VPW];
  // (paged keys: a wave takes KPW consecutive instructions instead, i.e. KPW * K_ROWS_PI consecutive tokens -- 8 or 16 --
  // which lie in one page unless the pages are smaller than that: one page-table entry then serves them all)
  static_assert(!C::PAGED || (C::K_INSTR % KPW == 0 && C::V_INSTR % VPW == 0), "a wave's instructions of a paged tile are consecutive");
  auto k_instr = [&](int u) __attribute__((always_inline)) {
    return (C::PAGED ? wave * KPW + u : wave + u * C::NWAVES) % C::K_INSTR;
  };
  auto v_instr = [&](int u) __attribute__((always_inline)) {
    return (C::PAGED ? wave * VPW + u : wave + u * C::NWAVES) % C::V_INSTR;
  };
  // do this wave's instructions of a paged tile share a page?  (uniform)  Then they also share one scalar base, the
  // address of the wave's first token of the tile, and the lanes' offsets carry the instruction's rows as in a dense tile.
  const bool one_page = C::PAGED && (p.block_table == nullptr || (1 << p.page_shift) >= KPW * C::K_ROWS_PI);
  auto k_lane_off = [&](int s, int u, int row) __attribute__((always_inline)) {   // row: the tile row to fetch
    const int dst_row = k_instr(u) * C::K_ROWS_PI + kr_lane;                         // decides the LDS chunk
    return (uint32_t)row * (uint32_t)kss[s] + (uint32_t)swz_k<D>(dst_row, lane % (D / 8)) * 16u;
  };
  auto v_lane_off = [&](int u, int row) __attribute__((always_inline)) {
    const int dst_row = v_instr(u) * C::V_ROWS_PI + vr_lane;
    return (uint32_t)row * (uint32_t)vss + (uint32_t)swz_v<DV>(dst_row, lane % (DV / 8)) * 16u;
  };
  // (paged keys: the uniform base of an instruction already points at its first token, a lane adds its row within
  // the instruction; in a ragged tile tokens past the last one are replaced by the last one, which lies in the page
  // of the instruction's -- likewise cut -- first token)
#pragma unroll
  for (int u = 0; u < KPW; ++u)
#pragma unroll
    for (int s = 0; s < NS; ++s)
      k_off[s][u] = k_lane_off(s, u, C::PAGED ? (one_page ? u * C::K_ROWS_PI : 0) + kr_lane : k_instr(u) * C::K_ROWS_PI + kr_lane);
#pragma unroll
  for (int u = 0; u < VPW; ++u)
    v_off[u] = v_lane_off(u, C::PAGED ? (one_page ? u * C::V_ROWS_PI : 0) + vr_lane : v_instr(u) * C::V_ROWS_PI + vr_lane);
  auto clamp_k = [&](int t) __attribute__((always_inline)) {
    const int nvalid = p.Sk - t * BN;              // uniform
    if (nvalid < BN) {
#pragma unroll
      for (int u = 0; u < KPW; ++u)
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          const int row = k_instr(u) * C::K_ROWS_PI + kr_lane;
          if constexpr (C::PAGED)
            k_off[s][u] = k_lane_off(s, u, min(row, nvalid - 1) - min(k_instr(one_page ? 0 : u) * C::K_ROWS_PI, nvalid - 1));
          else
            k_off[s][u] = k_lane_off(s, u, row < nvalid ? row : nvalid - 1);
        }
    }
  };
  auto clamp_v = [&](int t) __attribute__((always_inline)) {
    const int nvalid = p.Sk - t * BN;
    if (nvalid < BN) {
#pragma unroll
      for (int u = 0; u < VPW; ++u) {
        const int row = v_instr(u) * C::V_ROWS_PI + vr_lane;
        if constexpr (C::PAGED)
          v_off[u] = v_lane_off(u, min(row, nvalid - 1) - min(v_instr(one_page ? 0 : u) * C::V_ROWS_PI, nvalid - 1));
        else
          v_off[u] = v_lane_off(u, row < nvalid ? row : nvalid - 1);
      }
    }
  };
  // paged keys: the page of load instruction u of tile t (every lane the same value; t < t_hi, so the sequence has a token)
  // (the table entry as loaded: nothing may touch it before it is needed, or the wait for it -- and with it for every
  // tile load issued before it -- moves up to here; cut_page() makes it uniform and cuts it to the cache's pages)
  auto page_of_lane = [&](int t, int u) __attribute__((always_inline)) -> int {
    if (p.block_table == nullptr) return b;        // one page per sequence
    const int token = min(t * BN + k_instr(u) * C::K_ROWS_PI, p.Sk - 1);
    return p.block_table[(int64_t)b * p.table_stride + (token >> p.page_shift)];
  };
  auto cut_page = [&](int entry) __attribute__((always_inline)) -> int {
    return max(0, min(__builtin_amdgcn_readfirstlane(entry), p.num_pages - 1));
  };
  // the pages of all of this wave's instructions of tile t, as loaded (per lane) / made uniform
  // (with a shared page only entry 0 is loaded; not even a copy of it is made here: that, too, would wait for it)
  auto pages_of_lane = [&](int t, int (&pg)[KPW]) __attribute__((always_inline)) {
    pg[0] = page_of_lane(t, 0);
#pragma unroll
    for (int u = 1; u < KPW; ++u) pg[u] = one_page ? 0 : page_of_lane(t, u);
  };
  auto cut_pages = [&](const int (&raw)[KPW], int (&pg)[KPW]) __attribute__((always_inline)) {
    pg[0] = cut_page(raw[0]);
#pragma unroll
    for (int u = 1; u < KPW; ++u) pg[u] = one_page ? pg[0] : cut_page(raw[u]);
  };
  auto pages_of = [&](int t, int (&pg)[KPW]) __attribute__((always_inline)) {
    int raw[KPW];
    pages_of_lane(t, raw);
    cut_pages(raw, pg);
  };
  // ... and the address of that instruction's first token in that page (view: the cache as [pages, 1, Hkv, page_size, D])
  // (page and token strides are below 2^32 bytes -- the host checks -- so each product is one 32 x 32 -> 64 bit multiply;
  // the shared scalar unit of the CU is what these kernels load most)
  auto paged_base = [&](const View& view, int t, int u, int page) __attribute__((always_inline)) -> const unsigned char* {
    const int token = min(t * BN + k_instr(u) * C::K_ROWS_PI, p.Sk - 1);
    const int within = p.block_table != nullptr ? (token & p.page_mask) : token;
    const unsigned char* head = (const unsigned char*)((const uint16_t*)view.ptr + hk * view.sh);   // loop invariant
    return head + (uint64_t)(uint32_t)page * (uint32_t)(view.sb * 2) + (uint64_t)(uint32_t)within * (uint32_t)(view.ss * 2);
  };
  // the bases of all of this wave's instructions of tile t
  auto paged_bases = [&](const View& view, int t, const int (&pg)[KPW], const unsigned char* (&base)[KPW]) __attribute__((always_inline)) {
    base[0] = paged_base(view, t, 0, pg[0]);
    if (one_page) {
#pragma unroll
      for (int u = 1; u < KPW; ++u) base[u] = base[0];
    } else {
#pragma unroll
      for (int u = 1; u < KPW; ++u) base[u] = paged_base(view, t, u, pg[u]);
    }
  };
  // one load instruction of a K tile (stream s) / V tile whose first row is at `tile_base`
  auto issue_k = [&](int s, int u, const unsigned char* tile_base, int lds_off) __attribute__((always_inline)) {
    lds_void* dst = (lds_void*)(lds_raw + lds_off + k_instr(u) * 1024);
    __builtin_amdgcn_global_load_lds((global_cvoid*)(tile_base + k_off[s][u]), dst, 16, 0, 0);
  };
  auto issue_v = [&](int u, const unsigned char* tile_base, int lds_off) __attribute__((always_inline)) {
    lds_void* dst = (lds_void*)(lds_raw + lds_off + v_instr(u) * 1024);
    __builtin_amdgcn_global_load_lds((global_cvoid*)(tile_base + v_off[u]), dst, 16, 0, 0);
  };
  auto k_tile_base = [&](int s, int t) __attribute__((always_inline)) { return kbase[s] + (int64_t)(t * BN) * kss[s]; };
  auto v_tile_base = [&](int t) __attribute__((always_inline)) { return vbase + (int64_t)(t * BN) * vss; };
  // whole-tile loads in one burst (prologue, two-stream loop)
  auto load_k = [&](int t, int buf) __attribute__((always_inline)) {
    clamp_k(t);
    int pg[KPW] = {};
    const unsigned char* pb[KPW] = {};
    if constexpr (C::PAGED) {
      pages_of(t, pg);
      paged_bases(p.k, t, pg, pb);
    }
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int u = 0; u < KPW; ++u)
        issue_k(s, u, C::PAGED ? pb[u] : k_tile_base(s, t), C::K_RING + (buf * NS + s) * C::K_BYTES);
  };
  auto load_v = [&](int t, int buf) __attribute__((always_inline)) {
    clamp_v(t);
    int pg[KPW] = {};
    const unsigned char* pb[KPW] = {};
    if constexpr (C::PAGED) {
      pages_of(t, pg);
      paged_bases(p.v, t, pg, pb);
    }
#pragma unroll
    for (int u = 0; u < VPW; ++u)
      issue_v(u, C::PAGED ? pb[u < KPW ? u : 0] : v_tile_base(t), C::V_RING + buf * C::V_BYTES);
  };
  auto wait_loads_and_sync = [&]() __attribute__((always_inline)) {
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wave's direct loads have landed
    __syncthreads();
  };

  {
    // ============ pipelined loop (see the header comment) ============
    // Inside the workgroup's tile list every wave processes every tile; a tile that a wave does
    // not need is simply fully masked for it (its probabilities are exactly 0).
    typename W::Scores sa, sb;                     // the two score tiles in flight
    typename W::Pipe ps;
    typename W::BiasRegs br;
    // tl[0] is the current tile, tl[1] the next, ...; tl[SPB] is the tile whose V and tl[SPB + 1] the tile
    // whose K the current step streams into the rings (t_hi past the end of the list)
    constexpr int SPB = C::SPB, RING = C::RING, NTL = SPB + 2;
    int tl[NTL];
    int2 tks[NTL];                                 // what the skipper knows about those tiles (document masks, mapped expressions)
    uint32_t tbw[NTL];                             // this lane's hidden-score bits of those tiles (mapped expressions)
    tl[0] = next_tile(t_lo, tks[0], tbw[0], std::integral_constant<bool, true>());
    if (tl[0] < t_hi) {
      auto after = [&](int t, int2& ks, uint32_t& bw, auto setup) __attribute__((always_inline)) {
        ks = make_int2(0, 0);
        bw = 0;
        return t < t_hi ? next_tile(t + 1, ks, bw, setup) : t_hi;
      };
#pragma unroll
      for (int u = 1; u < NTL; ++u) tl[u] = after(tl[u - 1], tks[u], tbw[u], std::integral_constant<bool, true>());
      w.template bias_dma<0>(tl[0] * BN);
      if (tl[1] < t_hi) w.template bias_dma<1>(tl[1] * BN);
      // K of tiles tl[0 .. SPB] into slots 0 .. SPB, V of tiles tl[0 .. SPB - 1] into slots 0 .. SPB - 1
      load_k(tl[0], 0);
      load_v(tl[0], 0);
#pragma unroll
      for (int u = 1; u <= SPB; ++u) {
        if (tl[u] < t_hi) load_k(tl[u], u);
        if (u < SPB && tl[u] < t_hi) load_v(tl[u], u);
      }
      wait_loads_and_sync();
      w.template load_bias<0>(br, tl[0] * BN);
      w.template qk<C::K_RING>(sa);
      if constexpr (C::NBIAS > 0) W::template wait_lds<0>();     // staged bias values have arrived
      w.transform(sa, tl[0] * BN, br);
      float mx[RB];
      bool full0 = wave_full(tl[0], tks[0]);
      if (full0) {
        w.rowmax(sa, mx);
        w.advance_max(mx);
      }
      __syncthreads();                             // everyone is done with K ring slot 0
      // uniform state of the tile stream: the ragged tile (if any) and the bases of the next K and
      // V tile to fetch, i.e. of tiles min(tl[SPB + 1], t_hi - 1) and min(tl[SPB], t_hi - 1)
      const int t_rag = p.Sk % BN != 0 ? p.Sk / BN : -1;
      const int64_t kstep[2] = {(int64_t)BN * kss[0], (int64_t)BN * kss[1]}, vstep = (int64_t)BN * vss;
      const unsigned char* kb[NS];
#pragma unroll
      for (int s = 0; s < NS; ++s) kb[s] = k_tile_base(s, tl[SPB + 1] < t_hi ? tl[SPB + 1] : t_hi - 1);
      const unsigned char* vb = v_tile_base(tl[SPB] < t_hi ? tl[SPB] : t_hi - 1);
      // paged keys: pages of the tiles whose K / V the next step loads (uniform), and those of the step after it on
      // their way (vector loads, every lane the same address: they land behind the step's wait for its tile loads)
      int pgk[KPW], pgv[KPW], pgpre[KPW];
      static_assert(!C::PAGED || KPW == VPW, "K and V tiles of paged keys are cut into the same load instructions");
#pragma unroll
      for (int u = 0; u < KPW; ++u) pgk[u] = pgv[u] = pgpre[u] = 0;
      if constexpr (C::PAGED) {
        pages_of(tl[SPB + 1] < t_hi ? tl[SPB + 1] : t_hi - 1, pgk);
        pages_of(tl[SPB] < t_hi ? tl[SPB] : t_hi - 1, pgv);
      }
      // One pipeline step.  cur / nxt hold the scores of the current / next tile.  Step number N
      // (mod 4) fixes the roles at compile time: tile number n of the list lives in ring slot
      // n % RING, so V of the current tile sits in slot N % RING and K of the next tile in slot
      // (N + 1) % RING; the step streams K of the tile SPB + 1 ahead (both streams' tiles for the
      // differential variant) into slot (N + SPB + 1) % RING and V of the tile SPB ahead into slot
      // (N + SPB) % RING.  Between two barriers (SPB steps) the slots read -- K: N + 1 .. N + SPB,
      // V: N .. N + SPB - 1 -- and the slots written -- K: N + SPB + 1 .. N + 2 SPB, V: N + SPB ..
      // N + 2 SPB - 1 -- are disjoint modulo RING = 2 SPB, and everything read was written before
      // the previous barrier; so the waves only meet once per SPB tiles.  The load instructions
      // are spread over phase A (a burst of them right after the barrier stalls every wave of the
      // workgroup in the memory pipeline while the matrix cores idle).  Past the end of the tile
      // list the loads simply repeat the last tile, and the last tile takes the same step: its
      // "next tile" contraction then runs on stale LDS contents and is never used.
      auto step = [&](auto nc, typename W::Scores& cur, typename W::Scores& nxt) __attribute__((always_inline)) {
        constexpr int N = decltype(nc)::value;
        constexpr int slot_vc = N % RING, slot_kn = (N + 1) % RING;            // read: V current, K next
        constexpr int slot_kl = (N + SPB + 1) % RING, slot_vl = (N + SPB) % RING;   // written by this step's loads
        const int t0 = tl[0], t1 = tl[1];
        const int tn = t1;
        const bool fulln = wave_full(t1, tks[1]);
        if (!full0) {                              // fully visible tiles were settled in phase B
          if (kWaveSkip && (t0 < tv_lo || t0 >= tv_hi)) {
            // nothing of the tile is visible to this wave's rows: all -inf, the running max stays
#pragma unroll
            for (int rb = 0; rb < RB; ++rb)
#pragma unroll
              for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) cur[rb][nb][r] = -INFINITY;
          } else {
            w.mask(cur, t0 * BN, tbw[0]);
            w.rowmax(cur, mx);
            w.advance_max(mx);
          }
        }
        if constexpr (C::NBIAS > 0) {
          // bias of the next tile: staged one step ago into buffer (N + 1) % 2 (its values are
          // first used behind the LDS waits of phase A, which cover these reads: LDS returns in
          // order); the tile after it is staged now into the buffer this frees
          if (tn < t_hi) w.template load_bias<(N + 1) % 2>(br, tn * BN);
          if (tl[2] < t_hi) w.template bias_dma<N % 2>(tl[2] * BN);
        }
        const int tk = tl[SPB + 1] < t_hi ? tl[SPB + 1] : t_hi - 1, tv = tl[SPB] < t_hi ? tl[SPB] : t_hi - 1;
        if constexpr ((MASK & kMaskDoc) != 0) {    // tiles may be skipped: no fixed stride between them
#pragma unroll
          for (int s = 0; s < NS; ++s) kb[s] = k_tile_base(s, tk);
          vb = v_tile_base(tv);
        }
        if (__builtin_expect(tk == t_rag, 0)) clamp_k(tk);
        if (__builtin_expect(tv == t_rag, 0)) clamp_v(tv);
        const unsigned char* kbp[KPW];             // paged keys: one base per load instruction
        const unsigned char* vbp[KPW];
        if constexpr (C::PAGED) {
          const int tk_next = tk + 1 < t_hi ? tk + 1 : t_hi - 1;   // the tile whose K the next step loads
          pages_of_lane(tk_next, pgpre);
          paged_bases(p.k, tk, pgk, kbp);
          paged_bases(p.v, tv, pgv, vbp);
        }
        w.template phase_a<C::K_RING + slot_kn * NS * C::K_BYTES>(
            nxt, cur, ps, tn * BN, br, [&](auto fc) __attribute__((always_inline)) {
              constexpr int f = decltype(fc)::value, NF = NB * KK;
              constexpr int NK = NS * KPW, NV = VPW, LN = NK + NV;
              static_for<0, NK>([&](auto ic) __attribute__((always_inline)) {
                constexpr int i = decltype(ic)::value, ss = i / KPW, u = i % KPW;
                if constexpr (f == ((2 * i + 1) * NF) / (2 * LN))
                  issue_k(ss, u, C::PAGED ? kbp[u] : kb[ss], C::K_RING + (slot_kl * NS + ss) * C::K_BYTES);
              });
              static_for<0, NV>([&](auto uc) __attribute__((always_inline)) {
                constexpr int u = decltype(uc)::value;
                if constexpr (f == ((2 * (NK + u) + 1) * NF) / (2 * LN))
                  issue_v(u, C::PAGED ? vbp[u] : vb, C::V_RING + slot_vl * C::V_BYTES);
              });
            });
        w.template phase_b<slot_vc * C::V_BYTES>(ps, cur, nxt, tn * BN, br, fulln);
        if constexpr (N % SPB == SPB - 1) wait_loads_and_sync();
        if constexpr (C::PAGED) {                  // this step's K tile is the next step's V tile
#pragma unroll
          for (int u = 0; u < KPW; ++u) pgv[u] = pgk[u];
          cut_pages(pgpre, pgk);
        }
#pragma unroll
        for (int u = 0; u + 1 < NTL; ++u) {
          tl[u] = tl[u + 1];
          tks[u] = tks[u + 1];
          tbw[u] = tbw[u + 1];
        }
        tl[NTL - 1] = after(tl[NTL - 1], tks[NTL - 1], tbw[NTL - 1], std::integral_constant<bool, false>());
        full0 = fulln;
        if constexpr ((MASK & kMaskDoc) == 0) {    // consecutive tiles: advance the bases until the list ends
          if (tl[SPB] < t_hi) vb += vstep;
#pragma unroll
          for (int s = 0; s < NS; ++s)
            if (tl[SPB + 1] < t_hi) kb[s] += kstep[s];
        }
      };
      while (true) {
        bool done = false;
        static_for<0, 4>([&](auto nc) __attribute__((always_inline)) {
          constexpr int N = decltype(nc)::value;
          if (!done) {
            if constexpr (N % 2 == 0) step(nc, sa, sb);
            else step(nc, sb, sa);
            done = tl[0] >= t_hi;
          }
        });
        if (done) break;
      }
      // the loop may end between two barriers: this wave's last loads have to land, and every wave has to
      // be done reading, before the rings are used again (second q-tile of a pair, epilogue exchange)
      if constexpr (SPB > 1) wait_loads_and_sync();
    }
  }

  // ---- epilogue (a7): normalise by l, combine streams, RMSNorm, gate, store
  const float lam = C::DIFF ? p.lambda[h] : 0.f;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const float lt = half_swap_sum(w.l_run[rb]);
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const float lse_v = lt > 0.f ? w.m_run[rb] * kLn2 + __logf(lt) : -INFINITY;
#pragma unroll
    for (int d = 0; d < DVB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) w.oacc[rb][d][r] *= inv;
    if constexpr (C::DIFF) {
      // The wave of stream 1 hands its normalised rows to the wave of stream 0 that owns the same
      // query rows (same lane, same registers) through LDS: the K/V rings are free by now (every
      // wave has passed the barrier of the last step).  Layout [row group][register quad][lane][4].
      float4* xch = (float4*)lds_raw + (wave % C::NROWG) * (DVB * 4 * 64) + lane;
      if (stream == 1) {
#pragma unroll
        for (int d = 0; d < DVB; ++d)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4)
            xch[(d * 4 + r4) * 64] = make_float4(w.oacc[rb][d][4 * r4], w.oacc[rb][d][4 * r4 + 1],
                                                 w.oacc[rb][d][4 * r4 + 2], w.oacc[rb][d][4 * r4 + 3]);
      }
      __syncthreads();
      if (stream == 0) {
#pragma unroll
        for (int d = 0; d < DVB; ++d)
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const float4 o2 = xch[(d * 4 + r4) * 64];
            w.oacc[rb][d][4 * r4] -= lam * o2.x;
            w.oacc[rb][d][4 * r4 + 1] -= lam * o2.y;
            w.oacc[rb][d][4 * r4 + 2] -= lam * o2.z;
            w.oacc[rb][d][4 * r4 + 3] -= lam * o2.w;
          }
      }
    }
    float ssq = 0.f;
#pragma unroll
    for (int d = 0; d < DVB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) ssq = fmaf(w.oacc[rb][d][r], w.oacc[rb][d][r], ssq);
    float rn = 1.f;
    if constexpr ((C::EPI & kEpiRms) != 0) {
      ssq = half_swap_sum(ssq);
      rn = 1.f / sqrtf(ssq * (1.f / DV) + p.rms_eps);
    }
    const int i = w.i[rb];
    if (i < p.Sq && stream == 0) {
      const int64_t orow = b * p.out.sb + g * p.out.sg + h * p.out.sh + (int64_t)i * p.out.ss;
      const int64_t grow = b * p.gate.sb + g * p.gate.sg + h * p.gate.sh + (int64_t)i * p.gate.ss;
#pragma unroll
      for (int d = 0; d < DVB; ++d)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int ch = 32 * d + 8 * r4 + 4 * w.half;   // 4 consecutive channels ch..ch+3
          float x[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] = w.oacc[rb][d][4 * r4 + e];
          if constexpr ((C::EPI & kEpiRms) != 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] *= rn * (p.rms_weight ? p.rms_weight[ch + e] : 1.f);
          }
          if constexpr ((C::EPI & kEpiGate) != 0) {
            const uint2 gg = *(const uint2*)((const uint16_t*)p.gate.ptr + grow + ch);
            const float g0 = __uint_as_float(gg.x << 16), g1 = __uint_as_float(gg.x & 0xFFFF0000u);
            const float g2 = __uint_as_float(gg.y << 16), g3 = __uint_as_float(gg.y & 0xFFFF0000u);
            x[0] *= fast_rcp(1.f + fast_exp2(-g0 * kLog2e));
            x[1] *= fast_rcp(1.f + fast_exp2(-g1 * kLog2e));
            x[2] *= fast_rcp(1.f + fast_exp2(-g2 * kLog2e));
            x[3] *= fast_rcp(1.f + fast_exp2(-g3 * kLog2e));
          }
          if (p.out_f32) {
            *(float4*)((float*)p.out.ptr + orow + ch) = make_float4(x[0], x[1], x[2], x[3]);
          } else {
            *(uint2*)((uint16_t*)p.out.ptr + orow + ch) = make_uint2(pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3]));
          }
        }
    }
    if (i < p.Sq && p.lse != nullptr && w.half == 0)    // every wave writes the lse of its own stream
      p.lse[b * p.lse_sb + (int64_t)(C::DIFF ? 2 * g + stream : g) * p.lse_sg + h * p.lse_sh + i] = lse_v;
  }
  }  // pass
}

// Tile classes of a mask given as an expression (run-time compiled variants): one wave evaluates the whole predicate --
// the variant's positional base mask and fl_user_mask -- on one (32-row query block, BN-key tile) and writes one byte:
// 0 nothing visible, 1 some, 2 all (a tile that reaches past Sk is never "all": its tail has to be masked).  Rows past
// Sq do not count; query blocks past the last one (the row of a tile is padded to a multiple of 8 blocks) get 0.
// With `bits`, every lane also stores the word of its own 32 scores' hidden bits (64 words per block, in the attention
// kernel's register order), so that the attention kernel applies the mask of a partly visible tile from one coalesced
// load per lane instead of evaluating the expression again.
// Launch: 256 threads, one wave per tile; blockIdx.x runs over [problem][query block][group of 4 tiles].
template <uint32_t MASK, int BN>
__global__ void __launch_bounds__(256) block_map_kernel(const FwdParams p, unsigned char* map, uint32_t* bits) {
  const int lane = threadIdx.x & 63;
  const int groups = (p.map_nkt + 3) / 4;
  const int64_t bid = blockIdx.x;
  const int kt = (int)(bid % groups) * 4 + (int)(threadIdx.x >> 6);
  const int qb = (int)((bid / groups) % p.map_nqb8);
  const int prob = (int)(bid / ((int64_t)groups * p.map_nqb8));
  if (kt >= p.map_nkt) return;                     // uniform over the wave
  int b = prob, g = 0, h = 0;
  if (p.map_per_head) {
    h = prob % p.H;
    g = (prob / p.H) % p.G;
    b = prob / (p.H * p.G);
  }
  // the scores of a lane in the attention kernel's register order: row = lane % 32 of the block, key block nb, register r
  // -> key 32 nb + 8 (r / 4) + r % 4 + 4 (lane / 32) of the tile; bit 16 nb + r of the lane's word = hidden
  const int i = qb * 32 + (lane & 31);
  const int jl = kt * BN + 4 * (lane >> 5);
  bool some_visible = false, some_hidden = false;
  uint32_t word = 0;
  if (i < p.Sq) {
#pragma unroll
    for (int nb = 0; nb < BN / 32; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = jl + 32 * nb + 8 * (r >> 2) + (r & 3);
        bool hide = j >= p.Sk;
        if (!hide)
          hide = is_masked(MASK & (kMaskCausal | kMaskWindow | kMaskPrefix), i + p.q_off, j, p.window, p.prefix, 0, 0) ||
                 fl_user_mask(b, g, h, i + p.q_off, j, p);
        some_visible = some_visible || !hide;
        some_hidden = some_hidden || hide;
        word |= hide ? (1u << (16 * nb + r)) : 0u;
      }
  } else {
    word = ~0u;
  }
  const bool vis = __builtin_amdgcn_ballot_w64(some_visible) != 0, hid = __builtin_amdgcn_ballot_w64(some_hidden) != 0;
  const int64_t block = ((int64_t)prob * p.map_nkt + kt) * p.map_nqb8 + qb;
  if (lane == 0) map[block] = (unsigned char)(vis ? (hid ? 1 : 2) : 0);
  if (bits != nullptr) bits[block * 64 + lane] = word;
}

}  // namespace fl
