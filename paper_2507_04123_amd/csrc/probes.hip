// Measurement probes for the bench: an empty launch, a plain copy, a dense matrix-core loop (gfx950).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "emc2_probe.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__global__ void k_probe_empty() {}

// four independent 16-byte loads in flight per thread before the first store
__global__ void __launch_bounds__(256) k_probe_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

__global__ void __launch_bounds__(256) k_probe_fill(uint4* __restrict__ dst, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = make_uint4(1u, 2u, 3u, 4u);
}

__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// one atomic OR per thread on a pseudo-random 4-byte word of a table of 2^log2_words words
__global__ void __launch_bounds__(256) k_probe_atomic(uint32_t* __restrict__ table, int log2_words, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const uint32_t h = probe_hash((uint32_t)i);
  atomicOr(table + (h & ((1u << log2_words) - 1u)), 1u << (h >> 27));
}

__global__ void __launch_bounds__(256) k_probe_mfma_f16(int64_t iters, float* __restrict__ sink) {
  // operands that the compiler cannot fold: they depend on the thread index
  half8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (_Float16)(0.001f * (float)((threadIdx.x + e) & 7));
    b[e] = (_Float16)(0.002f * (float)((threadIdx.x * 3 + e) & 7));
  }
  floatx16 acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int64_t it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[j][e];
  sink[(int64_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace

extern "C" int32_t emc2_probe_empty(int32_t n_launches, void* stream) {
  for (int32_t i = 0; i < n_launches; ++i) hipLaunchKernelGGL(k_probe_empty, dim3(1), dim3(64), 0, (hipStream_t)stream);
  return (int32_t)hipGetLastError();
}

extern "C" int32_t emc2_probe_copy(void* dst, const void* src, int64_t bytes, void* stream) {
  if (!dst || !src || bytes < 0 || (bytes & 15) || (((uintptr_t)dst | (uintptr_t)src) & 15)) return (int32_t)hipErrorInvalidValue;
  if (bytes == 0) return 0;
  const int64_t n16 = bytes / 16;
  int64_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;   // 16 blocks per CU, the rest by grid stride
  hipLaunchKernelGGL(k_probe_copy, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)dst, (const uint4*)src, n16);
  return (int32_t)hipGetLastError();
}

extern "C" int32_t emc2_probe_fill(void* dst, int64_t bytes, void* stream) {
  if (!dst || bytes < 0 || (bytes & 15) || ((uintptr_t)dst & 15)) return (int32_t)hipErrorInvalidValue;
  if (bytes == 0) return 0;
  const int64_t n16 = bytes / 16;
  int64_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  hipLaunchKernelGGL(k_probe_fill, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)dst, n16);
  return (int32_t)hipGetLastError();
}

extern "C" int32_t emc2_probe_atomic(uint32_t* d_table, int32_t log2_words, int64_t n, void* stream) {
  if (!d_table || log2_words < 0 || log2_words > 31 || n < 0) return (int32_t)hipErrorInvalidValue;
  if (n == 0) return 0;
  hipLaunchKernelGGL(k_probe_atomic, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, d_table, log2_words, n);
  return (int32_t)hipGetLastError();
}

extern "C" int32_t emc2_probe_mfma_f16(int64_t iters, int32_t blocks, float* d_sink, void* stream) {
  if (iters < 0 || blocks < 1 || !d_sink) return (int32_t)hipErrorInvalidValue;
  hipLaunchKernelGGL(k_probe_mfma_f16, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, iters, d_sink);
  return (int32_t)hipGetLastError();
}
