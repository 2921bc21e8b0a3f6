// bf16 attention-variant forward kernel for gfx950: both contractions on bf16 MFMA with fp32
// accumulation, scores and softmax state in registers, K/V tiles double-buffered in LDS and
// filled by direct global->LDS loads.
//
// Structure (Sec. 3 of the paper describes the fused pass this realises: score tiles, online
// softmax per tile via a fused max-reduction and rescaled accumulation, multiply by V tiles;
// Sec. 3.2: the key axis is a sequential loop inside the workgroup that owns a query tile;
// Sec. 3.4: running max / running sum with the exp(m_old - m_new) correction; Sec. 3.5: D and
// Dv each fit one tile, so the twin matmul needs no loop over them; Sec. 3.6: 1-D launch whose
// index is decoded in the kernel).
//
// Orientation.  Each wave owns 32 query rows and computes the TRANSPOSED score block
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
#pragma once
#include "fl_params.hpp"

namespace fl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void global_cvoid;

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
// XORs, hence their own inverses.  K is read one 16-byte chunk per lane with 32 consecutive rows
// per instruction; V is read by the transposing load as 4 rows x 64 bytes per 32 lanes.  Both
// layouts spread those accesses over all 64 banks.
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

template <int D_, int DV_, int NWAVES_, int BN_, int MOD_, uint32_t MASK_, int NBIAS_, bool DIFF_,
          uint32_t EPI_>
struct Bf16Cfg {
  static constexpr int D = D_, DV = DV_, NWAVES = NWAVES_, BN = BN_, MOD = MOD_, NBIAS = NBIAS_;
  static constexpr uint32_t MASK = MASK_, EPI = EPI_;
  static constexpr bool DIFF = DIFF_;
  // Differential + RMSNorm divides a nearly cancelling difference by its own rms, which
  // amplifies the bf16 rounding of the probabilities; there P is split into a bf16 high part
  // and a bf16 remainder and the second contraction runs on both.
  static constexpr bool PSPLIT = DIFF_ && (EPI_ & kEpiRms) != 0;
  static constexpr int NT = NWAVES * 64;
  static constexpr int BM = NWAVES * 32;
  static constexpr int NB = BN / 32;               // 32-key blocks per tile
  static constexpr int KK = D / 16;                // MFMA k-steps of the first contraction
  static constexpr int DVB = DV / 32;              // 32-channel blocks of the output
  static constexpr int NS = DIFF ? 2 : 1;          // softmax streams
  static constexpr int K_BYTES = BN * D * 2;
  static constexpr int V_BYTES = BN * DV * 2;
  static constexpr int STAGE_BYTES = NS * K_BYTES + V_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
  static constexpr int K_INSTR = K_BYTES / 1024;   // 64-lane x 16-byte direct loads per K tile
  static constexpr int V_INSTR = V_BYTES / 1024;
};

template <class C>
struct WaveState {
  bf16x8 qf[C::NS][C::KK];                         // Q fragments (B operand)
  f32x16 oacc[C::NS][C::DVB];                      // O^T accumulators
  float m_run[C::NS], l_run[C::NS];                // log2-domain running max; per-lane partial sum
};

// One tile of work for one wave.  FAST: every block of the tile is fully visible to every row
// of the wave (no mask arithmetic, no per-block branches).
template <class C, bool FAST>
__device__ __forceinline__ void process_tile(WaveState<C>& ws, const FwdParams& p, const unsigned char* st,
                                             const int (&cls)[C::NB], int j0, int i, int ic, int lane, int b,
                                             int g, int h, float c_scale, float slope_l2, int qdoc) {
  constexpr int D = C::D, DV = C::DV, NB = C::NB, KK = C::KK, DVB = C::DVB, NS = C::NS;
  constexpr uint32_t MASK = C::MASK;
  constexpr bool kPlain = (C::MOD == kModNone && C::NBIAS == 0);
  const int half = lane >> 5, col = lane & 31;
  const unsigned char* lv = st + NS * C::K_BYTES;

#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const unsigned char* lk = st + s * C::K_BYTES;
    f32x16 sc[NB];
    // ---- first contraction: S^T = K Q^T
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int row = 32 * nb + col;
      if (FAST || cls[nb] != kSkip) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        f32x16 acc = zero;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
          const bf16x8 a = *(const bf16x8*)(lk + row * (D * 2) + swz_k<D>(row, 2 * kk + half) * 16);
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ws.qf[s][kk], acc, 0, 0, 0);
        }
        sc[nb] = acc;
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) sc[nb][r] = -INFINITY;
      }
    }

    // ---- variant transform in registers (Eq. 4 score_mod, biases, masks)
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      if (!FAST && cls[nb] == kSkip) continue;
      const int jb = j0 + 32 * nb + 4 * half;      // key of register r: jb + 8*(r/4) + r%4
      if constexpr (!kPlain) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = jb + 8 * (r >> 2) + (r & 3);
          float x = sc[nb][r];
          if constexpr (C::MOD == kModSoftcap) {
            // cap*tanh(x*scale/cap) in the log2 domain; tanh(y) = 1 - 2/(exp(2y)+1)
            const float e = fast_exp2(x * (2.f * c_scale / p.softcap));
            const float cl = p.softcap * kLog2e;
            x = fmaf(fast_rcp(e + 1.f), -2.f * cl, cl);
          } else {
            x *= c_scale;
          }
          if constexpr (C::MOD == kModAlibi) x -= slope_l2 * fabsf((float)(i - j));
          sc[nb][r] = x;
        }
#pragma unroll
        for (int nbias = 0; nbias < C::NBIAS; ++nbias) {
          const BiasView& bv = p.bias[nbias];
          const int64_t roff = b * bv.sb + g * bv.sg + h * bv.sh + (int64_t)ic * bv.si;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = jb + 8 * (r >> 2) + (r & 3);
            const int64_t off = roff + (int64_t)(j < p.Sk ? j : p.Sk - 1) * bv.sj;
            const float bb = bv.is_f32 ? ((const float*)bv.ptr)[off] : bf16_to_f32(((const uint16_t*)bv.ptr)[off]);
            sc[nb][r] = fmaf(bb, kLog2e, sc[nb][r]);
          }
        }
      }
      if (!FAST && cls[nb] == kPartial) {
        int kd[16];
        if constexpr ((MASK & kMaskDoc) != 0) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = jb + 8 * (r >> 2) + (r & 3);
            kd[r] = p.kv_doc[(int64_t)b * p.Sk + (j < p.Sk ? j : p.Sk - 1)];
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = jb + 8 * (r >> 2) + (r & 3);
          const bool hide = j >= p.Sk || is_masked(MASK, i, j, p.window, p.prefix, qdoc, (MASK & kMaskDoc) ? kd[r] : 0);
          if (hide) sc[nb][r] = -INFINITY;
        }
      }
    }

    // ---- online softmax (Alg. 2 per tile; Sec. 3.4)
    float mx = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[nb][r]);
    mx = half_swap_max(mx);
    if constexpr (kPlain) mx *= c_scale;           // scale > 0 (checked on the host)
    const float m_new = fmaxf(ws.m_run[s], mx);
    const float m_safe = (!FAST && m_new == -INFINITY) ? 0.f : m_new;
    if (__builtin_amdgcn_ballot_w64(m_new > ws.m_run[s]) != 0) {   // rescale only when some max moved
      const float alpha = fast_exp2(ws.m_run[s] - m_safe);
      ws.l_run[s] *= alpha;
#pragma unroll
      for (int d = 0; d < DVB; ++d)
#pragma unroll
        for (int r = 0; r < 16; ++r) ws.oacc[s][d][r] *= alpha;
    }
    ws.m_run[s] = m_new;

    float psum = 0.f;
    bf16x8 pf[NB][2], pl[C::PSPLIT ? NB : 1][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      uint32_t w[8], wl[8];
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        float p0, p1;
        if constexpr (kPlain) {
          p0 = fast_exp2(fmaf(sc[nb][r], c_scale, -m_safe));
          p1 = fast_exp2(fmaf(sc[nb][r + 1], c_scale, -m_safe));
        } else {
          p0 = fast_exp2(sc[nb][r] - m_safe);
          p1 = fast_exp2(sc[nb][r + 1] - m_safe);
        }
        psum += p0 + p1;
        w[r >> 1] = pack_bf16(p0, p1);
        if constexpr (C::PSPLIT)
          wl[r >> 1] = pack_bf16(p0 - __uint_as_float(w[r >> 1] << 16), p1 - __uint_as_float(w[r >> 1] & 0xFFFF0000u));
      }
      pf[nb][0] = __builtin_bit_cast(bf16x8, (i32x4){(int)w[0], (int)w[1], (int)w[2], (int)w[3]});
      pf[nb][1] = __builtin_bit_cast(bf16x8, (i32x4){(int)w[4], (int)w[5], (int)w[6], (int)w[7]});
      if constexpr (C::PSPLIT) {
        pl[nb][0] = __builtin_bit_cast(bf16x8, (i32x4){(int)wl[0], (int)wl[1], (int)wl[2], (int)wl[3]});
        pl[nb][1] = __builtin_bit_cast(bf16x8, (i32x4){(int)wl[4], (int)wl[5], (int)wl[6], (int)wl[7]});
      }
    }
    ws.l_run[s] += psum;

    // ---- second contraction: O^T += V^T P^T
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      if (!FAST && cls[nb] == kSkip) continue;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        // transposing read: each lane supplies the address of 4 channels of one key; the 16-lane
        // group returns, per lane, 4 keys of one channel.
        const int s16 = lane & 15;
        const int key0 = 32 * nb + 16 * ks + 4 * half + (s16 >> 2);
#pragma unroll
        for (int d = 0; d < DVB; ++d) {
          const int ch = 32 * d + 16 * ((lane >> 4) & 1) + 4 * (s16 & 3);   // channel (element) index
          const int c16 = ch >> 3, within = (ch & 7) * 2;
          const unsigned char* a0 = lv + key0 * (DV * 2) + swz_v<DV>(key0, c16) * 16 + within;
          const unsigned char* a1 = lv + (key0 + 8) * (DV * 2) + swz_v<DV>(key0 + 8, c16) * 16 + within;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)a0);
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)a1);
          const s16x8 av = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
          const bf16x8 a = __builtin_bit_cast(bf16x8, av);
          ws.oacc[s][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[nb][ks], ws.oacc[s][d], 0, 0, 0);
          if constexpr (C::PSPLIT)
            ws.oacc[s][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pl[nb][ks], ws.oacc[s][d], 0, 0, 0);
        }
      }
    }
  }
}

template <class C>
__global__ void __launch_bounds__(C::NT) __attribute__((amdgpu_waves_per_eu(2, 2)))
fwd_bf16_kernel(const FwdParams p) {
  constexpr int D = C::D, DV = C::DV, BN = C::BN, NB = C::NB, KK = C::KK, DVB = C::DVB, NS = C::NS;
  constexpr uint32_t MASK = C::MASK;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5;
  const int col = lane & 31;

  // ---- logical grid decode (Sec. 3.6): 1-D launch -> (b, g, h, q-tile)
  const int nq = p.n_qtiles;
  int bid = blockIdx.x;
  int qt, bh;
  if (p.order == 1) {
    // XCD-aware: consecutive workgroup ids go round-robin to the 8 XCDs; give each XCD whole
    // (b, g, h) problems so a head's K/V stay in one L2.  Needs (B*G*H) % 8 == 0 (host checks).
    const int xcd = bid & 7;
    const int idx = bid >> 3;
    bh = (idx / nq) * 8 + xcd;
    qt = nq - 1 - (idx % nq);
  } else {
    qt = nq - 1 - (bid % nq);                      // longest (causal) tiles first
    bh = bid / nq;
  }
  const int h = bh % p.H;
  const int g = (bh / p.H) % p.G;
  const int b = bh / (p.H * p.G);
  const int hk = h / (p.H / p.Hkv);
  const int i0 = qt * C::BM;                       // first query row of the workgroup
  const int iw = i0 + wave * 32;                   // first query row of the wave
  const int i = iw + col;                          // this lane's query row
  const int ic = i < p.Sq ? i : p.Sq - 1;

  WaveState<C> ws;
  {
    const uint16_t* qp = (const uint16_t*)p.q.ptr + b * p.q.sb + g * p.q.sg + h * p.q.sh + (int64_t)ic * p.q.ss;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) ws.qf[0][kk] = *(const bf16x8*)(qp + 16 * kk + 8 * half);
    if constexpr (C::DIFF) {
      const uint16_t* q2 = (const uint16_t*)p.q2.ptr + b * p.q2.sb + g * p.q2.sg + h * p.q2.sh + (int64_t)ic * p.q2.ss;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) ws.qf[1][kk] = *(const bf16x8*)(q2 + 16 * kk + 8 * half);
    }
  }
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    ws.m_run[s] = -INFINITY;
    ws.l_run[s] = 0.f;
#pragma unroll
    for (int d = 0; d < DVB; ++d)
#pragma unroll
      for (int r = 0; r < 16; ++r) ws.oacc[s][d][r] = 0.f;
  }

  const float c_scale = p.scale * kLog2e;          // raw score -> log2 domain
  float slope_l2 = 0.f;
  if constexpr (C::MOD == kModAlibi) slope_l2 = p.alibi_slopes[h] * kLog2e;
  int qdoc = 0;
  if constexpr ((MASK & kMaskDoc) != 0) qdoc = p.q_doc[(int64_t)b * p.Sq + ic];

  // ---- tile skipper: visible key range and document-id summaries
  const int i_last = (i0 + C::BM - 1 < p.Sq ? i0 + C::BM : p.Sq) - 1;
  int k_lo, k_hi;
  key_range(MASK, i0, i_last, p.Sk, p.window, p.prefix, k_lo, k_hi);
  const int t_lo = k_lo / BN;
  const int t_hi = (k_hi + BN - 1) / BN;
  const int nks = (p.Sk + kSumBlock - 1) / kSumBlock;
  int2 qs_wg = make_int2(0, 0), qs_wave = make_int2(0, 0);
  if constexpr ((MASK & kMaskDoc) != 0) {
    const int nqs = (p.Sq + kSumBlock - 1) / kSumBlock;
    const int2* qsum = p.q_sum + (int64_t)b * nqs;
    const int s0 = i0 / kSumBlock;
    qs_wg = qsum[s0];
    for (int w = 1; w < C::NWAVES; ++w)
      if (s0 + w < nqs) {
        const int2 t = qsum[s0 + w];
        qs_wg.x = min(qs_wg.x, t.x);
        qs_wg.y = max(qs_wg.y, t.y);
      }
    qs_wave = qsum[min(s0 + wave, nqs - 1)];
  }
  const int2* ksum = (MASK & kMaskDoc) ? p.kv_sum + (int64_t)b * nks : nullptr;

  auto tile_visible = [&](int t) -> bool {         // uniform over the workgroup
    if constexpr ((MASK & kMaskDoc) != 0) {
      int2 ks = ksum[min(t * NB, nks - 1)];
#pragma unroll
      for (int u = 1; u < NB; ++u)
        if (t * NB + u < nks) {
          const int2 x = ksum[t * NB + u];
          ks.x = min(ks.x, x.x);
          ks.y = max(ks.y, x.y);
        }
      return classify_block(MASK, i0, i_last, t * BN, t * BN + BN - 1, p.Sk, p.window, p.prefix, qs_wg, ks) != kSkip;
    } else {
      return true;                                 // positional masks are already in [t_lo, t_hi)
    }
  };
  auto next_tile = [&](int t) -> int {
    while (t < t_hi && !tile_visible(t)) ++t;
    return t;
  };

  // ---- direct global -> LDS loads of one K/V tile (a2): every wave instruction moves 64 x 16 B
  // into 1 KiB of consecutive LDS; the swizzle is applied by choosing which global chunk each
  // lane fetches.  Rows past Sk are clamped to the last row (their scores are masked, and their
  // probabilities are exactly 0).
  const uint16_t* kbase[NS];
  kbase[0] = (const uint16_t*)p.k.ptr + b * p.k.sb + g * p.k.sg + hk * p.k.sh;
  if constexpr (C::DIFF) kbase[NS - 1] = (const uint16_t*)p.k2.ptr + b * p.k2.sb + g * p.k2.sg + hk * p.k2.sh;
  const int64_t kss[2] = {p.k.ss, C::DIFF ? p.k2.ss : 0};
  const uint16_t* vbase = (const uint16_t*)p.v.ptr + b * p.v.sb + g * p.v.sg + hk * p.v.sh;

  auto load_tile = [&](int t, int buf) {
    unsigned char* st = lds_raw + buf * C::STAGE_BYTES;
    const int j0 = t * BN;
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int u = 0; u < (C::K_INSTR + C::NWAVES - 1) / C::NWAVES; ++u) {
        const int gi = wave + u * C::NWAVES;       // wave-uniform instruction index
        if (C::K_INSTR % C::NWAVES == 0 || gi < C::K_INSTR) {
          const int slot = gi * 64 + lane;
          const int r = slot / (D / 8), pc = slot % (D / 8);
          const int jr = j0 + r < p.Sk ? j0 + r : p.Sk - 1;
          const uint16_t* src = kbase[s] + (int64_t)jr * kss[s] + 8 * swz_k<D>(r, pc);
          __builtin_amdgcn_global_load_lds((global_cvoid*)src, (lds_void*)(st + s * C::K_BYTES + gi * 1024), 16, 0, 0);
        }
      }
#pragma unroll
    for (int u = 0; u < (C::V_INSTR + C::NWAVES - 1) / C::NWAVES; ++u) {
      const int gi = wave + u * C::NWAVES;
      if (C::V_INSTR % C::NWAVES == 0 || gi < C::V_INSTR) {
        const int slot = gi * 64 + lane;
        const int r = slot / (DV / 8), pc = slot % (DV / 8);
        const int jr = j0 + r < p.Sk ? j0 + r : p.Sk - 1;
        const uint16_t* src = vbase + (int64_t)jr * p.v.ss + 8 * swz_v<DV>(r, pc);
        __builtin_amdgcn_global_load_lds((global_cvoid*)src, (lds_void*)(st + NS * C::K_BYTES + gi * 1024), 16, 0, 0);
      }
    }
  };

  auto compute_tile = [&](int t, int buf) {
    const unsigned char* st = lds_raw + buf * C::STAGE_BYTES;
    const int j0 = t * BN;
    int cls[NB];
    bool any = false, all_full = true;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      int2 ks = make_int2(0, 0);
      if constexpr ((MASK & kMaskDoc) != 0) ks = ksum[min(t * NB + nb, nks - 1)];
      cls[nb] = classify_block(MASK, iw, iw + 31, j0 + 32 * nb, j0 + 32 * nb + 31, p.Sk, p.window, p.prefix,
                               qs_wave, ks);
      any = any || cls[nb] != kSkip;
      all_full = all_full && cls[nb] == kFull;
    }
    if (all_full) process_tile<C, true>(ws, p, st, cls, j0, i, ic, lane, b, g, h, c_scale, slope_l2, qdoc);
    else if (any) process_tile<C, false>(ws, p, st, cls, j0, i, ic, lane, b, g, h, c_scale, slope_l2, qdoc);
  };

  // ---- main loop over visible key tiles; the next tile streams into the other LDS buffer
  int t = next_tile(t_lo);
  if (t < t_hi) load_tile(t, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): this wave's direct loads have landed
  __syncthreads();
  int buf = 0;
  while (t < t_hi) {
    const int tn = next_tile(t + 1);
    if (tn < t_hi) load_tile(tn, buf ^ 1);
    compute_tile(t, buf);
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    t = tn;
    buf ^= 1;
  }

  // ---- epilogue: normalise by l, combine streams, RMSNorm, gate, store (a7)
  float inv[NS], lse_v[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const float lt = half_swap_sum(ws.l_run[s]);
    inv[s] = lt > 0.f ? 1.f / lt : 0.f;
    lse_v[s] = lt > 0.f ? ws.m_run[s] * kLn2 + __logf(lt) : -INFINITY;
  }
  const float lam = C::DIFF ? p.lambda[h] : 0.f;
  float ssq = 0.f;
#pragma unroll
  for (int d = 0; d < DVB; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float x = ws.oacc[0][d][r] * inv[0];
      if constexpr (C::DIFF) x -= lam * (ws.oacc[NS - 1][d][r] * inv[NS - 1]);
      ws.oacc[0][d][r] = x;
      ssq = fmaf(x, x, ssq);
    }
  float rn = 1.f;
  if constexpr ((C::EPI & kEpiRms) != 0) {
    ssq = half_swap_sum(ssq);
    rn = 1.f / sqrtf(ssq * (1.f / DV) + p.rms_eps);
  }
  if (i < p.Sq) {
    const int64_t orow = b * p.out.sb + g * p.out.sg + h * p.out.sh + (int64_t)i * p.out.ss;
    const int64_t grow = b * p.gate.sb + g * p.gate.sg + h * p.gate.sh + (int64_t)i * p.gate.ss;
#pragma unroll
    for (int d = 0; d < DVB; ++d)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int ch = 32 * d + 8 * r4 + 4 * half;   // 4 consecutive channels ch..ch+3
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = ws.oacc[0][d][4 * r4 + e];
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
    if (p.lse != nullptr && half == 0) {
#pragma unroll
      for (int s = 0; s < NS; ++s)
        p.lse[b * p.lse_sb + (int64_t)(C::DIFF ? 2 * g + s : g) * p.lse_sg + h * p.lse_sh + i] = lse_v[s];
    }
  }
}

}  // namespace fl
