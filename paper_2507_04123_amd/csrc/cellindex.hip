// Cell index (occupancy bits + prefix-summed ranks): clear, mark, scan.
// The scan is the prefix-sum index search of the paper's Sec. 3.6: after it, the voxel index of
// any active cell is found with one 8-byte load.
#include "common.h"

namespace {

// One block per tile; thread t owns the half line (8 words, 64 bytes) t of the tile.  Flagged lines are zeroed and
// their flags lowered; a tile without a flagged line costs one 128-byte read.
__global__ void __launch_bounds__(256) k_index_clear(uint4* __restrict__ p, lineflag_t* __restrict__ flags) {
  lineflag_t* tf = flags + (int64_t)blockIdx.x * EMC2_LINES_PER_TILE;
  const lineflag_t f = tf[threadIdx.x >> 1];
  if (f) {
    uint4* t = p + ((int64_t)blockIdx.x * EMC2_SCAN_TILE + (int64_t)threadIdx.x * 8) / 2;
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = make_uint4(0u, 0u, 0u, 0u);
  }
  if (!__syncthreads_or(f != 0)) return;  // every thread has read its flag
  if (f && !(threadIdx.x & 1)) tf[threadIdx.x >> 1] = 0;
}

__global__ void __launch_bounds__(256) k_index_mark_coords(cellword_t* __restrict__ idx,
                                                           const int4* __restrict__ coords,
                                                           const int32_t* __restrict__ d_n, int64_t capacity,
                                                           int gx, int gy, int gz, int n_batch,
                                                           lineflag_t* __restrict__ flags) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int4 c = coords[i];  // (b, z, y, x)
  if ((unsigned)c.x >= (unsigned)n_batch || (unsigned)c.y >= (unsigned)gz || (unsigned)c.z >= (unsigned)gy ||
      (unsigned)c.w >= (unsigned)gx)
    return;  // malformed coordinate: ignore rather than write out of bounds
  const uint64_t key = (((uint64_t)c.x * gz + (uint64_t)c.y) * gy + (uint64_t)c.z) * gx + (uint64_t)c.w;
  atomicOr(&idx[key >> 5].x, 1u << ((uint32_t)key & 31u));
  flags[emc2_line_of_key(key)] = 1;
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(v, d, 64);
    if ((int)(threadIdx.x & 63) >= d) v += t;
  }
  return v;
}

// Per-block popcount totals.  Thread t owns the 8 consecutive words [8t, 8t+8) of its tile.
__global__ void __launch_bounds__(256) k_scan_reduce(const cellword_t* __restrict__ idx, int64_t n_words,
                                                     uint32_t* __restrict__ partials,
                                                     const lineflag_t* __restrict__ flags) {
  const bool mine = flags[(int64_t)blockIdx.x * EMC2_LINES_PER_TILE + (threadIdx.x >> 1)] != 0;
  if (!__syncthreads_or(mine)) {  // no bit in this tile
    if (threadIdx.x == 0) partials[blockIdx.x] = 0u;
    return;
  }
  const int64_t base = (int64_t)blockIdx.x * EMC2_SCAN_TILE + (int64_t)threadIdx.x * 8;
  uint32_t s = 0;
  if (mine) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (base + j < n_words) s += __popc(idx[base + j].x);
  }
  __shared__ uint32_t wsum[4];
  const uint32_t inc = wave_inclusive_scan(s);
  if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
  __syncthreads();
  if (threadIdx.x == 0) partials[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// Single block: exclusive scan of the block totals in place, total to *d_total (clamped).
__global__ void __launch_bounds__(1024) k_scan_partials(uint32_t* __restrict__ partials, int64_t n, int64_t capacity,
                                                        int32_t* __restrict__ d_total, int32_t* __restrict__ d_flags) {
  __shared__ uint32_t wsum[16];
  __shared__ uint32_t carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  for (int64_t start = 0; start < n; start += 1024) {
    const int64_t i = start + threadIdx.x;
    const uint32_t v = i < n ? partials[i] : 0u;
    const uint32_t inc = wave_inclusive_scan(v);
    if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
    __syncthreads();
    uint32_t wbase = 0;
    const int w = threadIdx.x >> 6;
    for (int j = 0; j < w; ++j) wbase += wsum[j];
    const uint32_t carry = carry_s;
    if (i < n) partials[i] = carry + wbase + inc - v;
    __syncthreads();
    if (threadIdx.x == 1023) carry_s = carry + wbase + inc;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const uint32_t total = carry_s;
    if ((int64_t)total > capacity) {
      atomicOr(d_flags, EMC2_DEVFLAG_CAPACITY);
      *d_total = (int32_t)capacity;
    } else {
      *d_total = (int32_t)total;
    }
  }
}

// Write each word's exclusive prefix (.y).
__global__ void __launch_bounds__(256) k_scan_apply(cellword_t* __restrict__ idx, int64_t n_words,
                                                    const uint32_t* __restrict__ partials,
                                                    const lineflag_t* __restrict__ flags) {
  const bool mine = flags[(int64_t)blockIdx.x * EMC2_LINES_PER_TILE + (threadIdx.x >> 1)] != 0;
  if (!__syncthreads_or(mine)) return;  // no bit, so no prefix field anybody reads
  const int64_t base = (int64_t)blockIdx.x * EMC2_SCAN_TILE + (int64_t)threadIdx.x * 8;
  uint32_t bits[8];
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    bits[j] = (mine && base + j < n_words) ? idx[base + j].x : 0u;
    s += __popc(bits[j]);
  }
  __shared__ uint32_t wsum[4];
  const uint32_t inc = wave_inclusive_scan(s);
  if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
  __syncthreads();
  uint32_t run = partials[blockIdx.x] + inc - s;
  const int w = threadIdx.x >> 6;
  for (int j = 0; j < w; ++j) run += wsum[j];
  if (mine) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (base + j < n_words) idx[base + j] = make_uint2(bits[j], run);
      run += __popc(bits[j]);
    }
  }
}

// Whole scan in one block (small grids: the coarse levels): thread t owns a contiguous run of words.
__global__ void __launch_bounds__(1024) k_scan_small(cellword_t* __restrict__ idx, int64_t n_words, int64_t capacity,
                                                     int32_t* __restrict__ d_total, int32_t* __restrict__ d_flags) {
  const int per = (int)((n_words + 1023) / 1024);
  const int64_t base = (int64_t)threadIdx.x * per;
  uint32_t s = 0;
  for (int j = 0; j < per; ++j)
    if (base + j < n_words) s += __popc(idx[base + j].x);
  __shared__ uint32_t wsum[16];
  const uint32_t inc = wave_inclusive_scan(s);
  if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
  __syncthreads();
  uint32_t run = inc - s;
  const int w = threadIdx.x >> 6;
  for (int j = 0; j < w; ++j) run += wsum[j];
  for (int j = 0; j < per; ++j)
    if (base + j < n_words) {
      const uint32_t bits = idx[base + j].x;
      idx[base + j] = make_uint2(bits, run);
      run += __popc(bits);
    }
  if (threadIdx.x == 1023) {
    if ((int64_t)run > capacity) {
      atomicOr(d_flags, EMC2_DEVFLAG_CAPACITY);
      *d_total = (int32_t)capacity;
    } else {
      *d_total = (int32_t)run;
    }
  }
}

// Apply step that derives its own base from the block totals (no separate scan of the totals): block b
// sums totals[0..b) cooperatively.  Quadratic in the number of blocks, so only used while that is moderate.
__global__ void __launch_bounds__(256) k_scan_apply_self(cellword_t* __restrict__ idx, int64_t n_words,
                                                         const uint32_t* __restrict__ totals, int64_t capacity,
                                                         int32_t* __restrict__ d_total, int32_t* __restrict__ d_flags,
                                                         const lineflag_t* __restrict__ flags) {
  // a line without bits has no prefix field anybody reads; the last block still reports the total
  const bool has_bits = flags[(int64_t)blockIdx.x * EMC2_LINES_PER_TILE + (threadIdx.x >> 1)] != 0;   // this thread's line
  if (!__syncthreads_or(has_bits) && blockIdx.x != gridDim.x - 1) return;
  __shared__ uint32_t wsum[4];
  __shared__ uint32_t base_s;
  uint32_t part = 0;
  for (int i = threadIdx.x; i < (int)blockIdx.x; i += 256) part += totals[i];
  {
    const uint32_t inc = wave_inclusive_scan(part);
    if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
    __syncthreads();
    if (threadIdx.x == 0) base_s = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    __syncthreads();
  }
  const int64_t base = (int64_t)blockIdx.x * EMC2_SCAN_TILE + (int64_t)threadIdx.x * 8;
  uint32_t bits[8];
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    bits[j] = (has_bits && base + j < n_words) ? idx[base + j].x : 0u;
    s += __popc(bits[j]);
  }
  const uint32_t inc = wave_inclusive_scan(s);
  __syncthreads();
  if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
  __syncthreads();
  uint32_t run = base_s + inc - s;
  const int w = threadIdx.x >> 6;
  for (int j = 0; j < w; ++j) run += wsum[j];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (has_bits && base + j < n_words) idx[base + j] = make_uint2(bits[j], run);
    run += __popc(bits[j]);
  }
  if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 255) {
    if ((int64_t)run > capacity) {
      atomicOr(d_flags, EMC2_DEVFLAG_CAPACITY);
      *d_total = (int32_t)capacity;
    } else {
      *d_total = (int32_t)run;
    }
  }
}

}  // namespace

void emc2_index_clear(emc2_ctx* ctx, cellword_t* idx, hipStream_t stream) {
  hipLaunchKernelGGL(k_index_clear, dim3((unsigned)ctx->slot_tiles), dim3(256), 0, stream, (uint4*)idx,
                     emc2_slot_flags(ctx, idx));
}

void emc2_index_mark_coords(emc2_ctx* ctx, cellword_t* idx, const int32_t* d_coords, const int32_t* d_n,
                            int64_t capacity, const int32_t grid[3], int32_t n_batch, hipStream_t stream) {
  if (capacity < 1) return;
  hipLaunchKernelGGL(k_index_mark_coords, dim3((unsigned)emc2_div_up(capacity, 256)), dim3(256), 0, stream, idx,
                     (const int4*)d_coords, d_n, capacity, grid[0], grid[1], grid[2], n_batch, emc2_slot_flags(ctx, idx));
}

void emc2_index_scan(emc2_ctx* ctx, cellword_t* idx, int64_t n_cells, int64_t capacity, int32_t* d_total,
                     hipStream_t stream) {
  const int64_t n_words = emc2_div_up(n_cells, 32);
  const int64_t n_blocks = emc2_div_up(n_words, EMC2_SCAN_TILE);
  if (n_words <= 8 * 1024) {
    // coarse levels: one block does it all (one launch instead of three)
    hipLaunchKernelGGL(k_scan_small, dim3(1), dim3(1024), 0, stream, idx, n_words, capacity, d_total, ctx->dev_words);
    return;
  }
  hipLaunchKernelGGL(k_scan_reduce, dim3((unsigned)n_blocks), dim3(256), 0, stream, idx, n_words, ctx->partials,
                     emc2_slot_flags(ctx, idx));
  if (n_blocks <= 16384) {   // each apply block re-sums the earlier totals itself: at most 64 KB from L2
    hipLaunchKernelGGL(k_scan_apply_self, dim3((unsigned)n_blocks), dim3(256), 0, stream, idx, n_words, ctx->partials,
                       capacity, d_total, ctx->dev_words, emc2_slot_flags(ctx, idx));
    return;
  }
  hipLaunchKernelGGL(k_scan_partials, dim3(1), dim3(1024), 0, stream, ctx->partials, n_blocks, capacity, d_total,
                     ctx->dev_words);
  hipLaunchKernelGGL(k_scan_apply, dim3((unsigned)n_blocks), dim3(256), 0, stream, idx, n_words, ctx->partials,
                     emc2_slot_flags(ctx, idx));
}
