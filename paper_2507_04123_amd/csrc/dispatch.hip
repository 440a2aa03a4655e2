// Scenario-Adaptive Dispatcher (paper Sec. 3.2): every scene goes to one of three experts according to how far
// away its proposal regions are and how clearly they are perceived, and the scenes of a batch are grouped by
// expert so that each expert's stack runs once over its own scenes.
//
// Small batches (the usual case: a few hundred proposals per scene, a handful of scenes) run in ONE launch of
// one block: per-scene maxima in LDS, then a block-wide prefix sum for the grouping.  Large ones take a
// zero / classify / group sequence with the maxima in global memory.
#include "common.h"

// The range test is defined by individually rounded fp32 operations.
#pragma clang fp contract(off)

namespace {

#define EMC2_DISPATCH_LDS_SCENES 8192

// 0 near and clear, 1 near-unclear or far-clear, 2 far and unclear; NaNs count as far / unclear.
__device__ __forceinline__ int classify(const float4 p, float d2, float conf) {
  const float xx = p.x * p.x, yy = p.y * p.y;
  const float r2 = xx + yy;
  const bool far = !(r2 < d2);
  const bool unclear = !(p.w >= conf);
  return (far && unclear) ? 2 : ((far || unclear) ? 1 : 0);
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(v, d, 64);
    if ((int)(threadIdx.x & 63) >= d) v += t;
  }
  return v;
}

// Block-wide (1024 threads) stable grouping of expert[0, n_scenes): thread t owns a contiguous run of scenes.
__device__ void group_scenes(const int32_t* expert, int n_scenes, int32_t* __restrict__ counts, int32_t* __restrict__ order) {
  __shared__ uint32_t wsum[3][16];
  const int per = (n_scenes + 1023) / 1024;
  const int base = (int)threadIdx.x * per;
  uint32_t c[3] = {0u, 0u, 0u};
  for (int j = 0; j < per; ++j)
    if (base + j < n_scenes) {
      const int e = expert[base + j];
      c[0] += e == 0; c[1] += e == 1; c[2] += e == 2;
    }
  uint32_t inc[3];
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    inc[k] = wave_inclusive_scan(c[k]);
    if ((threadIdx.x & 63) == 63) wsum[k][threadIdx.x >> 6] = inc[k];
  }
  __syncthreads();
  uint32_t total[3], before[3];
  const int w = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < 3; ++k) {
    total[k] = 0; before[k] = 0;
    for (int j = 0; j < 16; ++j) {
      if (j < w) before[k] += wsum[k][j];
      total[k] += wsum[k][j];
    }
  }
  uint32_t at[3] = {before[0] + inc[0] - c[0], total[0] + before[1] + inc[1] - c[1],
                    total[0] + total[1] + before[2] + inc[2] - c[2]};
  for (int j = 0; j < per; ++j)
    if (base + j < n_scenes) {
      const int e = expert[base + j];
      const int k = e == 0 ? 0 : (e == 1 ? 1 : 2);
      order[at[k]++] = base + j;
    }
  if (threadIdx.x == 0) {
    counts[0] = (int32_t)total[0];
    counts[1] = (int32_t)total[1];
    counts[2] = (int32_t)total[2];
  }
}

__global__ void __launch_bounds__(1024) k_dispatch_small(const float4* __restrict__ props, const int32_t* __restrict__ scene,
                                                         int64_t n, int n_scenes, float d2, float conf,
                                                         int32_t* __restrict__ expert, int32_t* __restrict__ counts,
                                                         int32_t* __restrict__ order) {
  __shared__ int32_t ex[EMC2_DISPATCH_LDS_SCENES];
  for (int s = threadIdx.x; s < n_scenes; s += 1024) ex[s] = 0;
  __syncthreads();
  for (int64_t i = threadIdx.x; i < n; i += 1024) {
    const int32_t s = scene ? scene[i] : 0;
    if (s < 0 || s >= n_scenes) continue;
    const int e = classify(props[i], d2, conf);
    if (e > 0) atomicMax(&ex[s], e);
  }
  __syncthreads();
  for (int s = threadIdx.x; s < n_scenes; s += 1024) expert[s] = ex[s];
  group_scenes(ex, n_scenes, counts, order);
}

__global__ void __launch_bounds__(256) k_dispatch_zero(int32_t* __restrict__ expert, int n_scenes) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s < n_scenes) expert[s] = 0;
}

__global__ void __launch_bounds__(256) k_dispatch_classify(const float4* __restrict__ props, const int32_t* __restrict__ scene,
                                                           int64_t n, int n_scenes, float d2, float conf,
                                                           int32_t* __restrict__ expert) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t s = scene ? scene[i] : 0;
  if (s < 0 || s >= n_scenes) return;
  const int e = classify(props[i], d2, conf);
  if (e > 0) atomicMax(&expert[s], e);
}

__global__ void __launch_bounds__(1024) k_dispatch_group(const int32_t* __restrict__ expert, int n_scenes,
                                                         int32_t* __restrict__ counts, int32_t* __restrict__ order) {
  group_scenes(expert, n_scenes, counts, order);
}

// Expert-grouped batching.  Position p of `order` holds scene s: its slot inside its expert's group is p minus the
// group's start (the counts of the experts before it).
__global__ void __launch_bounds__(256) k_group_slots(const int32_t* __restrict__ expert, const int32_t* __restrict__ order,
                                                     const int32_t* __restrict__ counts, int n_scenes,
                                                     int32_t* __restrict__ slot) {
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= n_scenes) return;
  const int32_t s = order[p];
  if (s < 0 || s >= n_scenes) return;   // malformed order: leave the slot as it is rather than write out of bounds
  const int32_t e = expert[s];
  const int32_t start = e <= 0 ? 0 : (e == 1 ? counts[0] : counts[0] + counts[1]);
  slot[s] = p - start;
}

// One thread per point: the slot of its scene if that scene runs on `e`, else -1 (the voxelizer drops the point).
__global__ void __launch_bounds__(256) k_group_points(const int32_t* __restrict__ scene, int64_t n_points,
                                                      const int32_t* __restrict__ expert, const int32_t* __restrict__ slot,
                                                      int n_scenes, int e, int32_t* __restrict__ group_batch) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_points) return;
  const int32_t s = scene ? scene[i] : 0;
  group_batch[i] = (s >= 0 && s < n_scenes && expert[s] == e) ? slot[s] : -1;
}

}  // namespace

extern "C" emc2_status emc2_group_points(emc2_ctx* ctx, const int32_t* d_scene, int64_t n_points, const int32_t* d_expert,
                                         const int32_t* d_order, const int32_t* d_counts, int32_t n_scenes, int32_t expert,
                                         int32_t* d_slot, int32_t* d_group_batch, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_expert || !d_order || !d_counts || !d_slot || (n_points > 0 && !d_group_batch))
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_group_points: null argument");
  if (n_points < 0 || n_scenes < 1 || n_scenes > (1 << 20) || expert < 0 || expert > 2)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_group_points: n_points < 0, n_scenes outside [1, 2^20] or expert outside [0, 2]");
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(k_group_slots, dim3((unsigned)emc2_div_up(n_scenes, 256)), dim3(256), 0, s, d_expert, d_order, d_counts,
                     n_scenes, d_slot);
  if (n_points > 0)
    hipLaunchKernelGGL(k_group_points, dim3((unsigned)emc2_div_up(n_points, 256)), dim3(256), 0, s, d_scene, n_points, d_expert,
                       d_slot, n_scenes, expert, d_group_batch);
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_group_points launch");
}

extern "C" emc2_status emc2_dispatch(emc2_ctx* ctx, const float* d_props, const int32_t* d_scene, int64_t n_props,
                                     int32_t n_scenes, float dist, float conf, int32_t* d_expert, int32_t* d_counts,
                                     int32_t* d_order, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_expert || !d_counts || !d_order || (n_props > 0 && !d_props))
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_dispatch: null argument");
  if (n_props < 0 || n_scenes < 1 || n_scenes > (1 << 20))
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_dispatch: n_props < 0 or n_scenes outside [1, 2^20]");
  if (!(dist >= 0.0f) || conf != conf)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_dispatch: the distance threshold must be >= 0 and the confidence threshold a number");
  hipStream_t s = (hipStream_t)stream;
  const float d2 = dist * dist;  // one fp32 rounding, on the host as in the definition
  if (n_scenes <= EMC2_DISPATCH_LDS_SCENES && n_props <= 32768) {
    hipLaunchKernelGGL(k_dispatch_small, dim3(1), dim3(1024), 0, s, (const float4*)d_props, d_scene, n_props, n_scenes, d2, conf,
                       d_expert, d_counts, d_order);
  } else {
    hipLaunchKernelGGL(k_dispatch_zero, dim3((unsigned)emc2_div_up(n_scenes, 256)), dim3(256), 0, s, d_expert, n_scenes);
    if (n_props > 0)
      hipLaunchKernelGGL(k_dispatch_classify, dim3((unsigned)emc2_div_up(n_props, 256)), dim3(256), 0, s, (const float4*)d_props,
                         d_scene, n_props, n_scenes, d2, conf, d_expert);
    hipLaunchKernelGGL(k_dispatch_group, dim3(1), dim3(1024), 0, s, d_expert, n_scenes, d_counts, d_order);
  }
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_dispatch launch");
}
