// Multiscale Pooling of image features into grid cells and multimodal fusion with the LiDAR voxels
// (paper Sec. 3.1: relevant image pixels are projected into 3D by their depth, pooled, and fused with the
// voxel features; Sec. 3.5: the pooling size is a user parameter; Fig. 5 caption: sites that coincide are
// concatenated, the others padded with zeros).
//
// Pooling is a counting sort of the pixels by cell followed by a segmented reduction, so that a feature row
// (2*C bytes) is read exactly once and no floating-point atomics are used except where a cell's pixel list
// crosses the boundary between two reduction blocks:
//   mark     one thread per pixel: lift by depth, cell key, set the cell's bit in the cell index (one atomic
//            per run of neighbouring pixels with the same cell); also zeroes the counters and accumulators
//   scan     prefix sum over the index: rank of a cell = its position in key order; number of cells
//   count    per pixel: rank r, position within the cell from a returning atomic add on counts[r] (one per run)
//   starts   exclusive prefix sum of counts
//   scatter  per pixel: sorted position starts[r] + pos -> pixel id and rank stored there
//   reduce   one block per 256 consecutive sorted rows, 8 lanes per row with 16-byte loads: runs of rows of one
//            cell are combined in registers, cells inside a group of 8 rows are finished there, partial runs
//            meet in LDS (plain stores, owner sums), the (at most one per block boundary) cell that continues
//            into the next block adds its partial result to a small global accumulator
//   finish   per boundary-crossing cell: accumulator -> mean / max -> fp16
#include <hip/hip_fp16.h>
#include <math.h>

#include "common.h"

// The lifting and the cell index are defined by individually rounded IEEE operations in a fixed order.
#pragma clang fp contract(off)

namespace {

struct PoolParams {
  double q[12];
  float lo[3];
  float vs[3];
  int32_t grid[3];
  int32_t batch_index;
  int32_t W;
};

// Cell along one axis: fp32 subtract, fp32 IEEE division, floor; -1 if outside (the voxelizer's rule).
__device__ __forceinline__ int cell_of(float p, float lo, float vs, int g) {
  const float t = (p - lo) / vs;
  if (!(t >= 0.0f) || !(t < (float)g)) return -1;
  return (int)floorf(t);
}

struct PixCell {
  int4 c;        // (b, z, y, x)
  uint64_t key;
  bool keep;
};

// Both pixel passes call this, so they agree on every pixel's fate and cell bit for bit.
__device__ __forceinline__ PixCell lift(const float* __restrict__ depth, int64_t p, int64_t npix, const PoolParams& prm) {
  PixCell r;
  r.keep = false;
  r.key = 0;
  r.c = make_int4(0, 0, 0, 0);
  if (p >= npix) return r;
  const float df = depth[p];
  if (!(df > 0.0f) || !(df <= 3.402823466e38f)) return r;  // no depth, behind the camera, NaN or inf
  const int j = (int)(p / prm.W);
  const int i = (int)(p - (int64_t)j * prm.W);
  const double d = (double)df;
  const double du = d * (double)i, dv = d * (double)j;  // exact products
  float x[3];
#pragma unroll
  for (int a = 0; a < 3; ++a) {
    const double t = prm.q[4 * a + 0] * du + prm.q[4 * a + 1] * dv + prm.q[4 * a + 2] * d + prm.q[4 * a + 3];
    x[a] = (float)t;  // one rounding to fp32
  }
  const int cx = cell_of(x[0], prm.lo[0], prm.vs[0], prm.grid[0]);
  const int cy = cell_of(x[1], prm.lo[1], prm.vs[1], prm.grid[1]);
  const int cz = cell_of(x[2], prm.lo[2], prm.vs[2], prm.grid[2]);
  r.keep = (cx >= 0) && (cy >= 0) && (cz >= 0);
  r.c = make_int4(prm.batch_index, cz, cy, cx);
  r.key = (((uint64_t)prm.batch_index * prm.grid[2] + (uint64_t)cz) * prm.grid[1] + (uint64_t)cy) * prm.grid[0] + (uint64_t)cx;
  return r;
}

// Consecutive pixels of an image row mostly land in the same cell, so only the first lane of a run of equal keys
// touches the index, and only if the bit is not already visible as set (bits are never cleared while this runs, so
// a stale read can only cost a redundant atomic).  The same launch zeroes what later passes accumulate into:
// the per-cell counters (at most min(pixels, capacity) cells exist) and the boundary accumulators.
__global__ void __launch_bounds__(256) k_pool_mark(const float* __restrict__ depth, int64_t npix, PoolParams prm,
                                                   cellword_t* __restrict__ idx, lineflag_t* __restrict__ flags,
                                                   int32_t* __restrict__ counts, int64_t n_counts, uint4* __restrict__ acc16,
                                                   int64_t n_acc16) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p < n_counts) counts[p] = 0;
  if (p < npix)
    for (int64_t a = p; a < n_acc16; a += npix) acc16[a] = make_uint4(0u, 0u, 0u, 0u);
  const PixCell pc = lift(depth, p, npix, prm);
  const uint64_t key = pc.keep ? pc.key : ~0ull;
  const uint64_t prev = __shfl_up((unsigned long long)key, 1, 64);
  if (!pc.keep || ((threadIdx.x & 63) != 0 && prev == key)) return;
  const uint32_t bit = 1u << ((uint32_t)key & 31u);
  if (idx[key >> 5].x & bit) return;
  atomicOr(&idx[key >> 5].x, bit);
  flags[emc2_line_of_key(key)] = 1;
}

// Position of every pixel within its cell.  A run of consecutive lanes with the same rank takes its positions from
// one returning atomic add of the run length (the first lane's), which cuts the atomics by the run length where
// cells are larger than pixels.
__global__ void __launch_bounds__(256) k_pool_count(const float* __restrict__ depth, int64_t npix, PoolParams prm,
                                                    const cellword_t* __restrict__ idx, int64_t capacity,
                                                    int4* __restrict__ coords, int32_t* __restrict__ counts,
                                                    int32_t* __restrict__ pix_rank, int32_t* __restrict__ pix_pos) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const PixCell pc = lift(depth, p, npix, prm);   // keep = false beyond the image
  int32_t r = pc.keep ? cell_lookup(idx, pc.key) : -1;
  if (r >= capacity) r = -1;  // beyond capacity: reported by the scan, dropped here
  const int lane = threadIdx.x & 63;
  const int32_t r_prev = __shfl_up(r, 1, 64);
  const bool head = r >= 0 && (lane == 0 || r != r_prev);
  const uint64_t heads = __ballot(head);
  const uint64_t breaks = __ballot(head || r < 0);
  int32_t pos = 0;
  int start = lane;
  if (r >= 0) {
    const uint64_t upto = heads & (lane == 63 ? ~0ull : ((1ull << (lane + 1)) - 1ull));
    start = 63 - __clzll(upto);                                  // my run's first lane
    const uint64_t above = breaks & ~((2ull << start) - 1ull);   // the next break after it (2ull << 63 wraps to 0)
    const int end = above ? (int)__ffsll((unsigned long long)above) - 1 : 64;
    if (lane == start) pos = atomicAdd(&counts[r], end - start);
  }
  pos = __shfl(pos, start, 64) + (lane - start);
  if (p >= npix) return;
  pix_rank[p] = r;
  if (r < 0) return;
  pix_pos[p] = pos;
  if (pos == 0) coords[r] = pc.c;  // exactly one pixel of every cell gets position 0
}

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(v, d, 64);
    if ((int)(threadIdx.x & 63) >= d) v += t;
  }
  return v;
}

// Exclusive prefix sum of counts[0, n) into starts[0, n], in two launches: block totals, then every block
// derives its base from the totals before it (quadratic in the number of blocks, which stays small).
__global__ void __launch_bounds__(256) k_starts_reduce(const int32_t* __restrict__ counts, const int32_t* __restrict__ d_n,
                                                       int64_t capacity, uint32_t* __restrict__ totals) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t base = (int64_t)blockIdx.x * 2048 + (int64_t)threadIdx.x * 8;
  uint32_t s = 0;
  if (base < n) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (base + j < n) s += (uint32_t)counts[base + j];
  }
  __shared__ uint32_t wsum[4];
  const uint32_t inc = wave_inclusive_scan(s);
  if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
  __syncthreads();
  if (threadIdx.x == 0) totals[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

__global__ void __launch_bounds__(256) k_starts_apply(const int32_t* __restrict__ counts, const int32_t* __restrict__ d_n,
                                                      int64_t capacity, const uint32_t* __restrict__ totals,
                                                      int32_t* __restrict__ starts, int32_t* __restrict__ d_rows) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  if (n == 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      starts[0] = 0;
      *d_rows = 0;
    }
    return;
  }
  if ((int64_t)blockIdx.x * 2048 >= n) return;  // uniform for the block
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
  const int64_t base = (int64_t)blockIdx.x * 2048 + (int64_t)threadIdx.x * 8;
  uint32_t c[8];
  uint32_t s = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    c[j] = (base + j < n) ? (uint32_t)counts[base + j] : 0u;
    s += c[j];
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
    if (base + j < n) starts[base + j] = (int32_t)run;
    run += c[j];
    if (base + j == n - 1) {
      starts[n] = (int32_t)run;
      *d_rows = (int32_t)run;  // number of pooled pixels = length of the sorted list
    }
  }
}

__global__ void __launch_bounds__(256) k_pool_scatter(int64_t npix, const int32_t* __restrict__ pix_rank,
                                                      const int32_t* __restrict__ pix_pos, const int32_t* __restrict__ starts,
                                                      int32_t* __restrict__ perm, int32_t* __restrict__ srank) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= npix) return;
  const int32_t r = pix_rank[p];
  if (r < 0) return;
  const int32_t t = starts[r] + pix_pos[p];
  perm[t] = (int32_t)p;
  srank[t] = r;
}

// Order-preserving map float -> uint32 (and back), so that a maximum can be taken with integer atomics.
__device__ __forceinline__ uint32_t f2ord(float f) {
  const uint32_t b = __float_as_uint(f);
  return b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
}
__device__ __forceinline__ float ord2f(uint32_t u) {
  return __uint_as_float(u ^ ((u >> 31) ? 0x80000000u : 0xffffffffu));
}

__device__ __forceinline__ void unpack8(const uint4 v, float f[8]) {
  const __half2* h = reinterpret_cast<const __half2*>(&v);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float2 t = __half22float2(h[e]);
    f[2 * e] = t.x;
    f[2 * e + 1] = t.y;
  }
}

__device__ __forceinline__ uint4 pack8(const float f[8]) {
  uint4 v;
  __half2* h = reinterpret_cast<__half2*>(&v);
#pragma unroll
  for (int e = 0; e < 4; ++e) h[e] = __floats2half2_rn(f[2 * e], f[2 * e + 1]);
  return v;
}

#define EMC2_POOL_STEPS 8                       // rows per group of 8 lanes
#define EMC2_POOL_RPB (32 * EMC2_POOL_STEPS)    // sorted rows per reduction block (32 groups)

// MODE 0 mean, 1 max.  One block reduces EMC2_POOL_RPB consecutive sorted rows.
//
// A group of 8 lanes takes EMC2_POOL_STEPS consecutive rows (lane l the channels 8l..8l+7 of each 64-channel
// slab); the row ids and their cells, then the rows themselves and the cells' list bounds are loaded in two
// dependent rounds, everything of a round in flight at once.  Rows of one cell are consecutive, so the group
// combines them in registers run by run.  A run that is a whole cell is finished on the spot: the common case
// where cells hold a few pixels.  Only the first run of a group (its cell began earlier: a "head") and the last
// (its cell goes on: a "tail") can be partial; they are parked in LDS with plain stores.  After a barrier the
// group a cell began in owns it: it adds to its tail the heads of the following groups for as long as they
// belong to the same cell (group 0 does the same for the cell that began before the block).  No atomics in
// LDS.  A cell that ends inside the block is finished there; one that crosses the block boundary is added to
// the global accumulator of the block it starts in (the only floating-point atomics of the whole pooling).
template <int MODE>
__global__ void __launch_bounds__(256, 4) k_pool_reduce(const __half* __restrict__ img, const int32_t* __restrict__ perm,
                                                        const int32_t* __restrict__ srank, const int32_t* __restrict__ starts,
                                                        const int32_t* __restrict__ d_rows, int C,
                                                        uint32_t* __restrict__ acc, __half* __restrict__ feats) {
  extern __shared__ __align__(16) float lds[];  // heads [32][C], tails [32][C], then head_cell [32]
  constexpr int RPB = EMC2_POOL_RPB, STEPS = EMC2_POOL_STEPS;
  const int64_t m = *d_rows;
  const int64_t t0 = (int64_t)blockIdx.x * RPB;
  if (t0 >= m) return;  // uniform for the block
  const int64_t t1 = t0 + RPB < m ? t0 + RPB : m;
  float* heads = lds;
  float* tails = lds + 32 * C;
  int32_t* head_cell = reinterpret_cast<int32_t*>(lds + 64 * C);
  const int g = threadIdx.x >> 3, l = threadIdx.x & 7;
  const int64_t tg = t0 + (int64_t)g * STEPS;  // the group's first row
  // first set of loads: which pixel and which cell each row is
  int32_t pix[STEPS], rk[STEPS];
#pragma unroll
  for (int i = 0; i < STEPS; ++i) {
    const int64_t t = tg + i;
    rk[i] = -1;
    pix[i] = 0;
    if (t < t1) {
      rk[i] = srank[t];
      pix[i] = perm[t];
    }
  }
  // second set (depends on the first): the cells' list bounds, the same for every slab
  int32_t ca[STEPS], cb[STEPS];
#pragma unroll
  for (int i = 0; i < STEPS; ++i) {
    ca[i] = 0;
    cb[i] = 0;
    if (rk[i] >= 0) {
      ca[i] = starts[rk[i]];
      cb[i] = starts[rk[i] + 1];
    }
  }
  // the group's head: its first row's cell, if that cell began before the group
  const bool has_head = rk[0] >= 0 && ca[0] < tg;
  if (l == 0) head_cell[g] = has_head ? rk[0] : -1;
  // the group's tail: its last row's cell, if that cell began in the group and goes on beyond it
  int32_t tr = -1, ta = 0, tb = 0;
#pragma unroll
  for (int i = 0; i < STEPS; ++i)
    if (rk[i] >= 0) { tr = rk[i]; ta = ca[i]; tb = cb[i]; }  // rows of a group are valid from the front
  const bool has_tail = tr >= 0 && ta >= tg && tb > tg + STEPS;
  for (int cc = 0; cc < C; cc += 64) {
    const int ch = cc + 8 * l;
    if (ch >= C) continue;
    uint4 v[STEPS];
#pragma unroll
    for (int i = 0; i < STEPS; ++i) {
      v[i] = make_uint4(0u, 0u, 0u, 0u);
      if (rk[i] >= 0) v[i] = *reinterpret_cast<const uint4*>(img + (int64_t)pix[i] * C + ch);
    }
    float run[8];
    int32_t cur = -1, cur_a = 0, cur_b = 0;
    bool cur_first = false;
#pragma unroll
    for (int i = 0; i <= STEPS; ++i) {
      const int32_t r = i < STEPS ? rk[i] : -1;
      if (r != cur) {
        if (cur >= 0) {
          if (cur_a >= tg && cur_b <= tg + STEPS) {  // the whole cell sits in this group's rows: finish it here
            float f[8];
            const float inv = 1.0f / (float)(cur_b - cur_a);
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = MODE == 0 ? run[e] * inv : run[e];
            *reinterpret_cast<uint4*>(feats + (int64_t)cur * C + ch) = pack8(f);
          } else {
            // a head if the run opened the group and its cell began earlier, else the tail
            float* dst = ((cur_first && cur_a < tg) ? heads : tails) + g * C + ch;
            *reinterpret_cast<float4*>(dst) = make_float4(run[0], run[1], run[2], run[3]);
            *reinterpret_cast<float4*>(dst + 4) = make_float4(run[4], run[5], run[6], run[7]);
          }
        }
        cur = r;
        cur_first = i == 0;
        if (i < STEPS) {
          cur_a = ca[i];
          cur_b = cb[i];
          if (r >= 0) unpack8(v[i], run);
        }
      } else if (i < STEPS && r >= 0) {
        float f[8];
        unpack8(v[i], f);
#pragma unroll
        for (int e = 0; e < 8; ++e) run[e] = MODE == 0 ? run[e] + f[e] : fmaxf(run[e], f[e]);
      }
    }
  }
  __syncthreads();
  // owners: the group a cell began in (its tail), and group 0 for the cell that began before the block (a head)
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    int32_t r, a, b;
    int g_next;  // first of the following groups whose head may belong to the cell
    if (which == 0) {
      if (!has_tail) continue;
      r = tr; a = ta; b = tb;
      g_next = g + 1;
    } else {
      if (g != 0 || !has_head || ca[0] >= t0) continue;
      r = rk[0]; a = ca[0]; b = cb[0];
      g_next = 1;
    }
    int g_end = g_next;
    while (g_end < 32 && head_cell[g_end] == r) ++g_end;
    for (int ch = 8 * l; ch < C; ch += 64) {
      float sum[8];
      const float* own = (which == 0 ? tails : heads) + g * C + ch;
#pragma unroll
      for (int e = 0; e < 8; ++e) sum[e] = own[e];
      for (int q = g_next; q < g_end; ++q) {
        const float* h = heads + q * C + ch;
#pragma unroll
        for (int e = 0; e < 8; ++e) sum[e] = MODE == 0 ? sum[e] + h[e] : fmaxf(sum[e], h[e]);
      }
      if (a >= t0 && b <= t1) {  // the whole cell lies in this block's rows
        const float inv = 1.0f / (float)(b - a);
        float f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = MODE == 0 ? sum[e] * inv : sum[e];
        *reinterpret_cast<uint4*>(feats + (int64_t)r * C + ch) = pack8(f);
      } else {  // crosses a block boundary: combine in the accumulator of the block it starts in
        uint32_t* dst = acc + (int64_t)(a / RPB) * C + ch;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          if (MODE == 0) unsafeAtomicAdd(reinterpret_cast<float*>(dst + e), sum[e]);
          else atomicMax(dst + e, f2ord(sum[e]));
        }
      }
    }
  }
}

template <int MODE>
__global__ void __launch_bounds__(256) k_pool_finish(const int32_t* __restrict__ starts, const int32_t* __restrict__ d_n,
                                                     int64_t capacity, int C, int RPB, const uint32_t* __restrict__ acc,
                                                     __half* __restrict__ feats) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int chunks = C >> 3;
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t r = w / chunks;
  if (r >= n) return;
  const int k = (int)(w - r * chunks);
  const int64_t a = starts[r], b = starts[r + 1];
  if (a / RPB == (b - 1) / RPB) return;  // finished by the reduction
  const uint32_t* src = acc + (a / RPB) * C + 8 * k;
  float f[8];
  const float cnt = (float)(b - a);
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = MODE == 0 ? __uint_as_float(src[e]) / cnt : ord2f(src[e]);
  *reinterpret_cast<uint4*>(feats + r * C + 8 * k) = pack8(f);
}

// ------------------------------------------------------------------------------------------------------------
// fusion
// ------------------------------------------------------------------------------------------------------------

__device__ __forceinline__ bool fuse_key(const int4 c, int gx, int gy, int gz, int n_batch, uint64_t* key) {
  if ((unsigned)c.x >= (unsigned)n_batch || (unsigned)c.y >= (unsigned)gz || (unsigned)c.z >= (unsigned)gy ||
      (unsigned)c.w >= (unsigned)gx)
    return false;  // malformed coordinate: ignored everywhere rather than written out of bounds
  *key = (((uint64_t)c.x * gz + (uint64_t)c.y) * gy + (uint64_t)c.z) * gx + (uint64_t)c.w;
  return true;
}

// One thread per input row of either set (LiDAR rows first): set the site's bit in the union index.  The same
// launch presets the source arrays of every possible output row to "none".
__global__ void __launch_bounds__(256) k_fuse_mark(const int4* __restrict__ coords_l, const int32_t* __restrict__ d_n_l,
                                                   int64_t capacity_l, const int4* __restrict__ coords_i,
                                                   const int32_t* __restrict__ d_n_i, int64_t capacity_i,
                                                   cellword_t* __restrict__ idx, lineflag_t* __restrict__ flags, int gx, int gy,
                                                   int gz, int n_batch, int64_t bound, int32_t* __restrict__ src_l,
                                                   int32_t* __restrict__ src_i) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < bound) {
    src_l[t] = -1;
    src_i[t] = -1;
  }
  const bool is_l = t < capacity_l;
  const int64_t i = is_l ? t : t - capacity_l;
  int64_t n = is_l ? *d_n_l : *d_n_i;
  const int64_t cap = is_l ? capacity_l : capacity_i;
  if (n > cap) n = cap;
  if (i >= n) return;
  uint64_t key;
  if (!fuse_key((is_l ? coords_l : coords_i)[i], gx, gy, gz, n_batch, &key)) return;
  atomicOr(&idx[key >> 5].x, 1u << ((uint32_t)key & 31u));
  flags[emc2_line_of_key(key)] = 1;
}

// One thread per input row of either set: its rank in the union index is its output row.
__global__ void __launch_bounds__(256) k_fuse_place(const int4* __restrict__ coords_l, const int32_t* __restrict__ d_n_l,
                                                    int64_t capacity_l, const int4* __restrict__ coords_i,
                                                    const int32_t* __restrict__ d_n_i, int64_t capacity_i,
                                                    const cellword_t* __restrict__ idx, int gx, int gy, int gz, int n_batch,
                                                    int64_t capacity_out, int32_t* __restrict__ src_l,
                                                    int32_t* __restrict__ src_i, int4* __restrict__ coords_out) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const bool is_l = t < capacity_l;
  const int64_t i = is_l ? t : t - capacity_l;
  int64_t n = is_l ? *d_n_l : *d_n_i;
  const int64_t cap = is_l ? capacity_l : capacity_i;
  if (n > cap) n = cap;
  if (i >= n) return;
  const int4 c = (is_l ? coords_l : coords_i)[i];  // (b, z, y, x)
  uint64_t key;
  if (!fuse_key(c, gx, gy, gz, n_batch, &key)) return;
  const int32_t r = cell_lookup(idx, key);
  if (r < 0 || r >= capacity_out) return;
  (is_l ? src_l : src_i)[r] = (int32_t)i;
  coords_out[r] = c;  // where both sets hold the site they write the same value
}

// One thread per (output row, word of VEC bytes): the row is written once, each half copied from its source row
// or zero-filled, the padding beyond the two halves zeroed.
template <typename VEC>
__global__ void __launch_bounds__(256) k_fuse_gather(const VEC* __restrict__ feats_l, const VEC* __restrict__ feats_i,
                                                     const int32_t* __restrict__ src_l, const int32_t* __restrict__ src_i,
                                                     const int32_t* __restrict__ d_n, int64_t capacity, int wl, int wi, int wo,
                                                     VEC* __restrict__ out) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t r = t / wo;
  if (r >= n) return;
  const int w = (int)(t - r * wo);
  VEC v;
  memset(&v, 0, sizeof(VEC));
  if (w < wl) {
    const int32_t s = src_l[r];
    if (s >= 0) v = feats_l[(int64_t)s * wl + w];
  } else if (w < wl + wi) {
    const int32_t s = src_i[r];
    if (s >= 0) v = feats_i[(int64_t)s * wi + (w - wl)];
  }
  out[t] = v;
}

}  // namespace

extern "C" emc2_status emc2_pool_image(emc2_ctx* ctx, const void* d_img, const float* d_depth, int32_t H, int32_t W, int32_t C,
                                       const float Q[12], const emc2_voxel_spec* spec, int32_t batch_index,
                                       emc2_pool_mode mode, int64_t capacity, int32_t* d_coords, void* d_feats,
                                       int32_t* d_counts, int32_t* d_n_cells, int32_t* h_n_cells, int32_t index_slot,
                                       void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_img || !d_depth || !Q || !spec || !d_coords || !d_feats || !d_counts || !d_n_cells)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: null argument");
  if (H < 1 || W < 1) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: bad image size");
  const int64_t npix = (int64_t)H * W;
  if (npix > ctx->max_points)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: %lld pixels > max_points %lld", (long long)npix,
                     (long long)ctx->max_points);
  if (C < 8 || (C & 7) || C > 256)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_pool_image: C must be a multiple of 8 in [8, 256]");
  if (mode != EMC2_POOL_MEAN && mode != EMC2_POOL_MAX) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: bad mode");
  if (capacity < 1 || capacity > ctx->max_voxels)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: capacity %lld outside [1, max_voxels %lld]",
                     (long long)capacity, (long long)ctx->max_voxels);
  if (index_slot < 0 || index_slot >= ctx->n_slots)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: index_slot %d outside [0, %d)", index_slot, ctx->n_slots);
  if (batch_index < 0 || batch_index >= spec->n_batch)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: batch_index outside [0, n_batch)");
  for (int a = 0; a < 3; ++a)
    if (!(spec->vs[a] > 0.0f) || !isfinite(spec->vs[a]) || !isfinite(spec->lo[a]))
      return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: bad cell size / lower bound");
  for (int k = 0; k < 12; ++k)
    if (!isfinite(Q[k])) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: Q is not finite");
  int64_t n_cells = 0;
  if (!emc2_grid_ok(spec->grid, spec->n_batch, &n_cells))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_pool_image: grid/batch out of the supported key range");
  if (n_cells > ctx->max_cells)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: %lld cells > max_cells %lld", (long long)n_cells,
                     (long long)ctx->max_cells);

  hipStream_t s = (hipStream_t)stream;
  cellword_t* idx = ctx->slots[index_slot];
  SlotMeta& mt = ctx->meta[index_slot];
  for (int a = 0; a < 3; ++a) mt.grid[a] = spec->grid[a];
  mt.n_batch = spec->n_batch;
  mt.valid = true;

  PoolParams prm;
  for (int k = 0; k < 12; ++k) prm.q[k] = (double)Q[k];
  for (int a = 0; a < 3; ++a) { prm.lo[a] = spec->lo[a]; prm.vs[a] = spec->vs[a]; prm.grid[a] = spec->grid[a]; }
  prm.batch_index = batch_index;
  prm.W = W;

  const int RPB = EMC2_POOL_RPB;
  const int64_t bound = npix < capacity ? npix : capacity;  // at most this many cells exist
  const dim3 blk(256), pg((unsigned)emc2_div_up(npix, 256));
  const int64_t scan_blocks = emc2_div_up(bound, 2048);
  const int64_t red_blocks = emc2_div_up(npix, RPB);
  if (scan_blocks > ctx->n_pool_totals)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: capacity beyond the context's scan scratch");

  emc2_index_clear(ctx, idx, s);
  hipLaunchKernelGGL(k_pool_mark, pg, blk, 0, s, d_depth, npix, prm, idx, emc2_slot_flags(ctx, idx), d_counts, bound,
                     (uint4*)ctx->pool_acc, red_blocks * C / 4);
  emc2_index_scan(ctx, idx, n_cells, capacity, d_n_cells, s);
  hipLaunchKernelGGL(k_pool_count, pg, blk, 0, s, d_depth, npix, prm, idx, capacity, (int4*)d_coords, d_counts, ctx->pix_rank,
                     ctx->pix_pos);
  hipLaunchKernelGGL(k_starts_reduce, dim3((unsigned)scan_blocks), blk, 0, s, d_counts, d_n_cells, capacity, ctx->pool_totals);
  hipLaunchKernelGGL(k_starts_apply, dim3((unsigned)scan_blocks), blk, 0, s, d_counts, d_n_cells, capacity, ctx->pool_totals,
                     ctx->cell_start, ctx->dev_words + 2);
  hipLaunchKernelGGL(k_pool_scatter, pg, blk, 0, s, npix, ctx->pix_rank, ctx->pix_pos, ctx->cell_start, ctx->pix_perm,
                     ctx->pix_srank);
  const size_t lds_bytes = sizeof(float) * (64 * (size_t)C + 32);  // heads and tails of the 32 groups, their cells
  const dim3 rg((unsigned)red_blocks), fg((unsigned)emc2_div_up(bound * (C / 8), 256));
  if (lds_bytes > 65536) {  // C = 256 only: a little over the default per-block limit (the CU has 160 KB)
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_pool_reduce<0>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&k_pool_reduce<1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  }
  if (mode == EMC2_POOL_MEAN) {
    hipLaunchKernelGGL(k_pool_reduce<0>, rg, blk, lds_bytes, s, (const __half*)d_img, ctx->pix_perm, ctx->pix_srank,
                       ctx->cell_start, ctx->dev_words + 2, C, ctx->pool_acc, (__half*)d_feats);
    hipLaunchKernelGGL(k_pool_finish<0>, fg, blk, 0, s, ctx->cell_start, d_n_cells, capacity, C, RPB, ctx->pool_acc,
                       (__half*)d_feats);
  } else {
    hipLaunchKernelGGL(k_pool_reduce<1>, rg, blk, lds_bytes, s, (const __half*)d_img, ctx->pix_perm, ctx->pix_srank,
                       ctx->cell_start, ctx->dev_words + 2, C, ctx->pool_acc, (__half*)d_feats);
    hipLaunchKernelGGL(k_pool_finish<1>, fg, blk, 0, s, ctx->cell_start, d_n_cells, capacity, C, RPB, ctx->pool_acc,
                       (__half*)d_feats);
  }
  emc2_status st = emc2_check_hip(ctx, hipGetLastError(), "emc2_pool_image launch");
  if (st != EMC2_OK) return st;
  if (h_n_cells) {
    st = emc2_check_hip(ctx, hipMemcpyAsync(ctx->pinned + 1, d_n_cells, sizeof(int32_t), hipMemcpyDeviceToHost, s),
                        "hipMemcpyAsync(n_cells)");
    if (st != EMC2_OK) return st;
    st = emc2_check_hip(ctx, hipStreamSynchronize(s), "hipStreamSynchronize");
    if (st != EMC2_OK) return st;
    *h_n_cells = ctx->pinned[1];
  }
  return EMC2_OK;
}

extern "C" emc2_status emc2_fuse(emc2_ctx* ctx, emc2_dtype dtype, const int32_t* d_coords_l, const void* d_feats_l,
                                 const int32_t* d_n_l, int64_t capacity_l, int32_t c_l, const int32_t* d_coords_i,
                                 const void* d_feats_i, const int32_t* d_n_i, int64_t capacity_i, int32_t c_i,
                                 const int32_t grid[3], int32_t n_batch, int32_t out_slot, int64_t capacity_out, int32_t c_out,
                                 int32_t* d_coords_out, void* d_feats_out, int32_t* d_src_l, int32_t* d_src_i,
                                 int32_t* d_n_out, int32_t* h_n_out, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_coords_l || !d_feats_l || !d_n_l || !d_coords_i || !d_feats_i || !d_n_i || !grid || !d_coords_out || !d_feats_out ||
      !d_n_out)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_fuse: null argument");
  if (dtype != EMC2_F32 && dtype != EMC2_F16 && dtype != EMC2_BF16) return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_fuse: bad dtype");
  if (capacity_l < 1 || capacity_i < 1 || capacity_out < 1 || capacity_out > ctx->max_voxels)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_fuse: capacities must be >= 1 and capacity_out <= max_voxels %lld",
                     (long long)ctx->max_voxels);
  if (c_l < 1 || c_i < 1 || c_l > 4096 || c_i > 4096 || c_out < c_l + c_i || c_out > 8192)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_fuse: bad channel counts (need c_out >= c_l + c_i)");
  if (out_slot < 0 || out_slot >= ctx->n_slots)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_fuse: out_slot %d outside [0, %d)", out_slot, ctx->n_slots);
  int64_t n_cells = 0;
  if (!emc2_grid_ok(grid, n_batch, &n_cells))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_fuse: grid/batch out of the supported key range");
  if (n_cells > ctx->max_cells)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_fuse: %lld cells > max_cells %lld", (long long)n_cells,
                     (long long)ctx->max_cells);
  const int es = dtype == EMC2_F32 ? 4 : 2;
  const int64_t bl = (int64_t)c_l * es, bi = (int64_t)c_i * es, bo = (int64_t)c_out * es;
  if ((bl | bi | bo) & 3)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_fuse: every feature row (both halves and the output) must be a multiple of 4 bytes");

  hipStream_t s = (hipStream_t)stream;
  cellword_t* idx = ctx->slots[out_slot];
  SlotMeta& mt = ctx->meta[out_slot];
  for (int a = 0; a < 3; ++a) mt.grid[a] = grid[a];
  mt.n_batch = n_batch;
  mt.valid = true;
  int32_t* src_l = d_src_l ? d_src_l : ctx->fuse_src;
  int32_t* src_i = d_src_i ? d_src_i : ctx->fuse_src + ctx->max_voxels;

  const dim3 blk(256);
  emc2_index_clear(ctx, idx, s);
  const int64_t bound = capacity_l + capacity_i < capacity_out ? capacity_l + capacity_i : capacity_out;
  const dim3 both((unsigned)emc2_div_up(capacity_l + capacity_i, 256));
  hipLaunchKernelGGL(k_fuse_mark, both, blk, 0, s, (const int4*)d_coords_l, d_n_l, capacity_l, (const int4*)d_coords_i, d_n_i,
                     capacity_i, idx, emc2_slot_flags(ctx, idx), grid[0], grid[1], grid[2], n_batch, bound, src_l, src_i);
  emc2_index_scan(ctx, idx, n_cells, capacity_out, d_n_out, s);
  hipLaunchKernelGGL(k_fuse_place, both, blk, 0, s, (const int4*)d_coords_l, d_n_l, capacity_l, (const int4*)d_coords_i, d_n_i,
                     capacity_i, idx, grid[0], grid[1], grid[2], n_batch, capacity_out, src_l, src_i, (int4*)d_coords_out);
  if (!((bl | bi | bo) & 15)) {
    const int wl = (int)(bl / 16), wi = (int)(bi / 16), wo = (int)(bo / 16);
    hipLaunchKernelGGL(k_fuse_gather<uint4>, dim3((unsigned)emc2_div_up(bound * wo, 256)), blk, 0, s, (const uint4*)d_feats_l,
                       (const uint4*)d_feats_i, src_l, src_i, d_n_out, capacity_out, wl, wi, wo, (uint4*)d_feats_out);
  } else {
    const int wl = (int)(bl / 4), wi = (int)(bi / 4), wo = (int)(bo / 4);
    hipLaunchKernelGGL(k_fuse_gather<uint32_t>, dim3((unsigned)emc2_div_up(bound * wo, 256)), blk, 0, s,
                       (const uint32_t*)d_feats_l, (const uint32_t*)d_feats_i, src_l, src_i, d_n_out, capacity_out, wl, wi, wo,
                       (uint32_t*)d_feats_out);
  }
  emc2_status st = emc2_check_hip(ctx, hipGetLastError(), "emc2_fuse launch");
  if (st != EMC2_OK) return st;
  if (h_n_out) {
    st = emc2_check_hip(ctx, hipMemcpyAsync(ctx->pinned + 1, d_n_out, sizeof(int32_t), hipMemcpyDeviceToHost, s),
                        "hipMemcpyAsync(n_out)");
    if (st != EMC2_OK) return st;
    st = emc2_check_hip(ctx, hipStreamSynchronize(s), "hipStreamSynchronize");
    if (st != EMC2_OK) return st;
    *h_n_out = ctx->pinned[1];
  }
  return EMC2_OK;
}
