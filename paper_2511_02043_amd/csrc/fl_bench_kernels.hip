// Measurement helpers for bench.py, built into their own small library (libflbench.so): they are not
// part of the attention library or its ABI and compute no attention.
//   flb_mfma_peak   what the matrix cores sustain with nothing else to do: every wave runs a chain of
//                   independent v_mfma_f32_32x32x16_bf16 on register operands (pseudo-random bf16 values of
//                   magnitude 0.25 .. 2, because the board's power limit, and with it the clock, depends on
//                   how many operand bits toggle; zero operands give a far higher figure)
//   flb_copy        a plain 16-bytes-per-lane device copy: the HBM bandwidth reference
//   flb_read        the same loads with nothing written: what a read-only stream (the decode step) can reach
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) int i32x4;

namespace {

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// two bf16 values: random sign and mantissa, exponent in 125 .. 128 (0.25 <= |x| < 4); zero_data: all zero
__device__ __forceinline__ int rand_pair(uint32_t r, int zero_data) {
  const uint32_t lo = (r & 0x807fu) | ((125u + ((r >> 7) & 3u)) << 7);
  const uint32_t hi = ((r >> 16) & 0x807fu) | ((125u + ((r >> 23) & 3u)) << 7);
  return zero_data ? 0 : (int)(lo | (hi << 16));
}

__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
mfma_peak_kernel(float* sink, int iters, int zero_data) {
  const uint32_t id = blockIdx.x * 512u + threadIdx.x;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    i32x4 x, y;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[e] = rand_pair(mix(id * 64u + u * 8u + e), zero_data);
      y[e] = rand_pair(mix(id * 64u + u * 8u + e + 4u), zero_data);
    }
    a[u] = __builtin_bit_cast(bf16x8, x);
    b[u] = __builtin_bit_cast(bf16x8, y);
  }
  f32x16 acc[4];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[u][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[(u + 1) & 3], acc[u], 0, 0, 0);
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + 2) & 3], b[u], acc[u], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[u][r];
  if (s == 1.2345e-30f) sink[id] = s;              // never true: keeps the chain alive
}

__global__ void __launch_bounds__(256) copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// four 16-byte loads in flight per lane; the values are folded so that the loads cannot be dropped
__global__ void __launch_bounds__(256) read_kernel(const uint4* __restrict__ src, uint32_t* sink, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  uint32_t acc = 0;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
  }
  for (; i < n16; i += stride) {
    const uint4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  if (acc == 0x9E3779B9u) sink[0] = acc;           // practically never: keeps the loads alive
}

}  // namespace

extern "C" {

// Launches the MFMA chain: `blocks` workgroups of 8 waves, 8 * iters MFMAs per wave.  `sink` is any
// device buffer of blocks * 512 floats (never written).  Returns the FLOPs of the launch, or -1 on error.
double flb_mfma_peak(float* sink, int blocks, int iters, int zero_data, void* stream) {
  if (sink == nullptr || blocks <= 0 || iters <= 0) return -1.0;
  hipLaunchKernelGGL(mfma_peak_kernel, dim3(blocks), dim3(512), 0, (hipStream_t)stream, sink, iters, zero_data);
  if (hipGetLastError() != hipSuccess) return -1.0;
  return (double)blocks * 8.0 * (double)iters * 8.0 * 32768.0;
}

// Copies `bytes` (a multiple of 16; both pointers 16-byte aligned) from src to dst.  Returns 0, or -1 on error.
int flb_copy(void* dst, const void* src, size_t bytes, void* stream) {
  if (dst == nullptr || src == nullptr || bytes % 16 != 0 || ((uintptr_t)dst | (uintptr_t)src) % 16 != 0) return -1;
  if (bytes == 0) return 0;
  hipLaunchKernelGGL(copy_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst, bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

// Reads `bytes` (a multiple of 16; src 16-byte aligned) and writes nothing (sink: any device word).  Returns 0, or -1 on error.
int flb_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (src == nullptr || sink == nullptr || bytes % 16 != 0 || ((uintptr_t)src) % 16 != 0) return -1;
  if (bytes == 0) return 0;
  hipLaunchKernelGGL(read_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint32_t*)sink, bytes / 16);
  return hipGetLastError() == hipSuccess ? 0 : -1;
}

}  // extern "C"
