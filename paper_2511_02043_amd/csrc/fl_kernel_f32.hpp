// fp32 attention-variant forward kernel (plain VALU arithmetic, no MFMA).
//
// This is the fp32-storage specialisation of the fused pass: scores, softmax state and the
// output accumulator are all fp32, the exponentials and tanh use the accurate math-library
// routines, and the result is meant to stay within 1e-5 of an fp64 evaluation.  Every variant
// feature is available here.  It follows the same structure as the bf16 kernel: one workgroup
// owns a tile of query rows, walks the visible key tiles (skipper), keeps (m, l, O) in
// registers and never stores a score (Sec. 3.2 dimension demotion; Sec. 3.4 running max / sum
// with the exp(m_old - m_new) correction).
//
// Work split: 256 threads = 64 query rows x 4 lanes; the 4 lanes of a row split the head
// dimension in interleaved float4 chunks and combine their partial dot products with two
// cross-lane adds.  K and V tiles of 32 keys are staged in LDS and read as broadcasts.
#pragma once
#include "fl_params.hpp"

namespace fl {

constexpr int kF32Rows = 64;     // query rows per workgroup
constexpr int kF32Keys = 32;     // keys per LDS tile
constexpr int kF32Chunk = 8;     // keys per softmax update

__device__ __forceinline__ float quad_sum_f32(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x;
}

template <bool DIFF, int DMAX>
__global__ void __launch_bounds__(256)
fwd_f32_kernel(const FwdParams p) {
  const int D = p.D, Dv = p.Dv;
  constexpr int NCH = DMAX / 16;
  const int MOD = p.mod, NBIAS = p.n_bias;
  const uint32_t MASK = p.mask, EPI = p.epi;
  extern __shared__ float lds[];
  float* ldsK = lds;                               // [kF32Keys][D]
  float* ldsK2 = ldsK + kF32Keys * DMAX;           // [kF32Keys][D]   (differential only)
  float* ldsV = ldsK2 + (DIFF ? kF32Keys * DMAX : 0);   // [kF32Keys][Dv]

  const int tid = threadIdx.x;
  const int sl = tid & 3;
  const int row = tid >> 2;
  const int nq = p.n_qtiles;
  int bid = blockIdx.x;
  const int qt = nq - 1 - (bid % nq);              // longest causal tiles first
  bid /= nq;
  const int h = bid % p.H;  bid /= p.H;
  const int g = bid % p.G;
  const int b = bid / p.G;
  const int hk = h / (p.H / p.Hkv);
  const int i0 = qt * kF32Rows;
  const int i = i0 + row;
  const bool row_ok = i < p.Sq;
  const int ic = row_ok ? i : p.Sq - 1;
  const int ncq = D / 4, ncv = Dv / 4;             // float4 chunks in a q/k row and a v row

  // ---- query slice(s) in registers
  float4 qf[DIFF ? 2 : 1][NCH];
  {
    const float* qp = (const float*)p.q.ptr + b * p.q.sb + g * p.q.sg + h * p.q.sh + ic * p.q.ss;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int ch = sl + 4 * c;
      qf[0][c] = ch < ncq ? *(const float4*)(qp + 4 * ch) : make_float4(0, 0, 0, 0);
    }
    if constexpr (DIFF) {
      const float* q2 = (const float*)p.q2.ptr + b * p.q2.sb + g * p.q2.sg + h * p.q2.sh + ic * p.q2.ss;
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int ch = sl + 4 * c;
        qf[1][c] = ch < ncq ? *(const float4*)(q2 + 4 * ch) : make_float4(0, 0, 0, 0);
      }
    }
  }
  constexpr int NS = DIFF ? 2 : 1;
  float4 o[NS][NCH];
  float m[NS], l[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    m[s] = -INFINITY;
    l[s] = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) o[s][c] = make_float4(0, 0, 0, 0);
  }

  const int qdoc = (MASK & kMaskDoc) ? p.q_doc[(int64_t)b * p.Sq + ic] : 0;
  const float slope = MOD == kModAlibi ? p.alibi_slopes[h] : 0.f;

  // ---- visible key range of this workgroup (positional masks) and tile walk
  int k_lo, k_hi;
  const int i_max = (i0 + kF32Rows - 1 < p.Sq ? i0 + kF32Rows - 1 : p.Sq - 1);
  key_range(MASK, i0 + p.q_off, i_max + p.q_off, p.Sk, p.window, p.prefix, k_lo, k_hi);   // row i sits at position i + q_off
  const int t_lo = k_lo / kF32Keys;
  const int t_hi = (k_hi + kF32Keys - 1) / kF32Keys;

  int2 qs = make_int2(0, 0);
  if ((MASK & kMaskDoc) != 0) {          // summary of the workgroup's 64 rows
    const int nqs = (p.Sq + kSumBlock - 1) / kSumBlock;
    const int2* s = p.q_sum + (int64_t)b * nqs;
    const int s0 = i0 / kSumBlock;
    qs = s[s0];
    if (s0 + 1 < nqs) {
      int2 t = s[s0 + 1];
      qs.x = min(qs.x, t.x);
      qs.y = max(qs.y, t.y);
    }
  }

  for (int t = t_lo; t < t_hi; ++t) {
    const int j0 = t * kF32Keys;
    int2 ks = make_int2(0, 0);
    if ((MASK & kMaskDoc) != 0)
      ks = p.kv_sum[(int64_t)b * ((p.Sk + kSumBlock - 1) / kSumBlock) + t];   // kF32Keys == kSumBlock
    const int cls = classify_block(MASK, i0 + p.q_off, i_max + p.q_off, j0, j0 + kF32Keys - 1, p.Sk, p.window, p.prefix, qs, ks);
    if (cls == kSkip) continue;                    // uniform over the workgroup

    __syncthreads();                               // previous tile fully consumed
    {
      const float* kp = (const float*)p.k.ptr + b * p.k.sb + g * p.k.sg + hk * p.k.sh;
      const float* vp = (const float*)p.v.ptr + b * p.v.sb + g * p.v.sg + hk * p.v.sh;
      for (int e = tid; e < kF32Keys * ncq; e += 256) {
        const int r = e / ncq, c = e % ncq;
        const int j = j0 + r;
        float4 x = make_float4(0, 0, 0, 0);
        if (j < p.Sk) x = *(const float4*)(kp + (int64_t)j * p.k.ss + 4 * c);
        *(float4*)(ldsK + r * D + 4 * c) = x;
        if constexpr (DIFF) {
          const float* k2 = (const float*)p.k2.ptr + b * p.k2.sb + g * p.k2.sg + hk * p.k2.sh;
          float4 y = make_float4(0, 0, 0, 0);
          if (j < p.Sk) y = *(const float4*)(k2 + (int64_t)j * p.k2.ss + 4 * c);
          *(float4*)(ldsK2 + r * D + 4 * c) = y;
        }
      }
      for (int e = tid; e < kF32Keys * ncv; e += 256) {
        const int r = e / ncv, c = e % ncv;
        const int j = j0 + r;
        float4 x = make_float4(0, 0, 0, 0);
        if (j < p.Sk) x = *(const float4*)(vp + (int64_t)j * p.v.ss + 4 * c);
        *(float4*)(ldsV + r * Dv + 4 * c) = x;
      }
    }
    __syncthreads();

#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const float* lk = s == 0 ? ldsK : ldsK2;
      for (int c0 = 0; c0 < kF32Keys; c0 += kF32Chunk) {
        float sc[kF32Chunk];
#pragma unroll
        for (int u = 0; u < kF32Chunk; ++u) {
          const int r = c0 + u;
          float acc = 0.f;
#pragma unroll
          for (int c = 0; c < NCH; ++c) {
            const int ch = sl + 4 * c;
            if (ch < ncq) {
              const float4 kk = *(const float4*)(lk + r * D + 4 * ch);
              acc = fmaf(qf[s][c].x, kk.x, acc);
              acc = fmaf(qf[s][c].y, kk.y, acc);
              acc = fmaf(qf[s][c].z, kk.z, acc);
              acc = fmaf(qf[s][c].w, kk.w, acc);
            }
          }
          acc = quad_sum_f32(acc);
          const int j = j0 + r;
          float x = acc * p.scale;                                   // Eq. 3
          if (MOD == kModSoftcap) x = p.softcap * tanhf(x / p.softcap);   // Eq. 4
          if (MOD == kModAlibi) x -= slope * fabsf((float)(i + p.q_off - j));       // Eq. 4
          for (int nb = 0; nb < NBIAS; ++nb) {
            const BiasView& bv = p.bias[nb];
            const int64_t off = b * bv.sb + g * bv.sg + h * bv.sh + (int64_t)ic * bv.si +
                                (int64_t)(j < p.Sk ? j : 0) * bv.sj;
            x += bv.is_f32 ? ((const float*)bv.ptr)[off]
                           : __uint_as_float((uint32_t)((const uint16_t*)bv.ptr)[off] << 16);
          }
          bool hide = j >= p.Sk;
          if (cls == kPartial) {
            const int kd = (MASK & kMaskDoc) ? p.kv_doc[(int64_t)b * p.Sk + (j < p.Sk ? j : 0)] : 0;
            hide = hide || is_masked(MASK, i + p.q_off, j, p.window, p.prefix, qdoc, kd);
          }
          sc[u] = hide ? -INFINITY : x * kLog2e;                     // log2 domain from here on
        }
        // online softmax update over the chunk (Alg. 2 with a chunk of elements per step)
        float mx = m[s];
#pragma unroll
        for (int u = 0; u < kF32Chunk; ++u) mx = fmaxf(mx, sc[u]);
        const float ms = mx == -INFINITY ? 0.f : mx;
        const float alpha = exp2f(m[s] - ms);
        float pr[kF32Chunk], psum = 0.f;
#pragma unroll
        for (int u = 0; u < kF32Chunk; ++u) {
          pr[u] = exp2f(sc[u] - ms);
          psum += pr[u];
        }
        l[s] = l[s] * alpha + psum;
        m[s] = mx;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          const int ch = sl + 4 * c;
          if (ch < ncv) {
            float4 a = o[s][c];
            a.x *= alpha; a.y *= alpha; a.z *= alpha; a.w *= alpha;
#pragma unroll
            for (int u = 0; u < kF32Chunk; ++u) {
              const float4 vv = *(const float4*)(ldsV + (c0 + u) * Dv + 4 * ch);
              a.x = fmaf(pr[u], vv.x, a.x);
              a.y = fmaf(pr[u], vv.y, a.y);
              a.z = fmaf(pr[u], vv.z, a.z);
              a.w = fmaf(pr[u], vv.w, a.w);
            }
            o[s][c] = a;
          }
        }
      }
    }
  }

  // ---- epilogue: normalise, combine, RMSNorm, gate, store
  float inv[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) inv[s] = l[s] > 0.f ? 1.f / l[s] : 0.f;
  const float lam = DIFF ? p.lambda[h] : 0.f;
  float4 r[NCH];
  float ssq = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    float4 a = o[0][c];
    a.x *= inv[0]; a.y *= inv[0]; a.z *= inv[0]; a.w *= inv[0];
    if constexpr (DIFF) {
      const float4 b2 = o[NS - 1][c];
      a.x -= lam * (b2.x * inv[NS - 1]);
      a.y -= lam * (b2.y * inv[NS - 1]);
      a.z -= lam * (b2.z * inv[NS - 1]);
      a.w -= lam * (b2.w * inv[NS - 1]);
    }
    r[c] = a;
    if (sl + 4 * c < ncv) ssq += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
  }
  float rn = 1.f;
  if ((EPI & kEpiRms) != 0) {
    ssq = quad_sum_f32(ssq);
    rn = 1.f / sqrtf(ssq / (float)Dv + p.rms_eps);
  }
  if (row_ok) {
    float* op = (float*)p.out.ptr + b * p.out.sb + g * p.out.sg + h * p.out.sh + (int64_t)i * p.out.ss;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int ch = sl + 4 * c;
      if (ch < ncv) {
        float4 a = r[c];
        if ((EPI & kEpiRms) != 0) {
          float4 w = make_float4(1, 1, 1, 1);
          if (p.rms_weight) w = *(const float4*)(p.rms_weight + 4 * ch);
          a.x *= rn * w.x; a.y *= rn * w.y; a.z *= rn * w.z; a.w *= rn * w.w;
        }
        if ((EPI & kEpiGate) != 0) {
          const float* gp = (const float*)p.gate.ptr + b * p.gate.sb + g * p.gate.sg + h * p.gate.sh +
                            (int64_t)i * p.gate.ss;
          const float4 gg = *(const float4*)(gp + 4 * ch);
          a.x *= 1.f / (1.f + expf(-gg.x));
          a.y *= 1.f / (1.f + expf(-gg.y));
          a.z *= 1.f / (1.f + expf(-gg.z));
          a.w *= 1.f / (1.f + expf(-gg.w));
        }
        *(float4*)(op + 4 * ch) = a;
      }
    }
    if (p.lse != nullptr && sl == 0) {
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        const float v = l[s] > 0.f ? m[s] * kLn2 + logf(l[s]) : -INFINITY;
        p.lse[b * p.lse_sb + (int64_t)(DIFF ? 2 * g + s : g) * p.lse_sg + h * p.lse_sh + i] = v;
      }
    }
  }
}

}  // namespace fl
