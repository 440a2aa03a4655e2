// Multiscale Pooling of image features into grid cells and multimodal fusion with the LiDAR voxels
// (paper Sec. 3.1: relevant image pixels are projected into 3D by their depth, pooled, and fused with the
// voxel features; Sec. 3.5: the pooling size is a user parameter; Fig. 5 caption: sites that coincide are
// concatenated, the others padded with zeros).
//
// Pooling is a counting sort of the pixels by cell followed by a segmented reduction, so that a feature row
// (2*C bytes) is read exactly once and no floating-point atomics touch HBM except where a cell's pixel list
// crosses the boundary between two reduction blocks:
//   mark     one thread per pixel: lift by depth, cell key, set the cell's bit in the cell index
//   scan     prefix sum over the index: rank of a cell = its position in key order; number of cells
//   count    per pixel: rank r, position within the cell from one returning atomic add on counts[r]
//   starts   exclusive prefix sum of counts
//   scatter  per pixel: sorted position starts[r] + pos -> pixel id and rank stored there
//   reduce   one block per RPB consecutive sorted rows: rows are summed (or maximised) into per-cell
//            accumulators in LDS with LDS atomics, 8 lanes per row with 16-byte loads; cells that lie
//            inside the block's rows are finished there, the (at most one per block boundary) cell that
//            continues into the next block adds its partial result to a small global accumulator
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

__global__ void __launch_bounds__(256) k_pool_mark(const float* __restrict__ depth, int64_t npix, PoolParams prm,
                                                   cellword_t* __restrict__ idx, uint32_t* __restrict__ flags) {
  const PixCell pc = lift(depth, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, npix, prm);
  if (!pc.keep) return;
  atomicOr(&idx[pc.key >> 5].x, 1u << ((uint32_t)pc.key & 31u));
  flags[pc.key >> (5 + EMC2_TILE_SHIFT)] = 1u;
}

__global__ void __launch_bounds__(256) k_pool_zero_counts(const int32_t* __restrict__ d_n, int64_t capacity,
                                                          int32_t* __restrict__ counts) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r < n) counts[r] = 0;
}

__global__ void __launch_bounds__(256) k_pool_count(const float* __restrict__ depth, int64_t npix, PoolParams prm,
                                                    const cellword_t* __restrict__ idx, int64_t capacity,
                                                    int4* __restrict__ coords, int32_t* __restrict__ counts,
                                                    int32_t* __restrict__ pix_rank, int32_t* __restrict__ pix_pos) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= npix) return;
  const PixCell pc = lift(depth, p, npix, prm);
  int32_t r = pc.keep ? cell_lookup(idx, pc.key) : -1;
  if (r >= capacity) r = -1;  // beyond capacity: reported by the scan, dropped here
  pix_rank[p] = r;
  if (r < 0) return;
  const int32_t pos = atomicAdd(&counts[r], 1);
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
                                                      int32_t* __restrict__ starts) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  if (n == 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) starts[0] = 0;
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
    if (base + j == n - 1) starts[n] = (int32_t)run;
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

__global__ void __launch_bounds__(256) k_pool_fill_zero(uint4* __restrict__ p, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
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

#define EMC2_POOL_LDS_WORDS 16384  // 64 KB of per-cell accumulators: RPB * C <= 16384

// MODE 0 mean, 1 max.  RPB sorted rows per block (a multiple of 32, at most 256).
template <int MODE>
__global__ void __launch_bounds__(256) k_pool_reduce(const __half* __restrict__ img, const int32_t* __restrict__ perm,
                                                     const int32_t* __restrict__ srank, const int32_t* __restrict__ starts,
                                                     const int32_t* __restrict__ d_n, int64_t capacity, int C, int RPB,
                                                     uint32_t* __restrict__ acc, __half* __restrict__ feats) {
  __shared__ uint32_t lds[EMC2_POOL_LDS_WORDS];
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t m = n > 0 ? (int64_t)starts[n] : 0;
  const int64_t t0 = (int64_t)blockIdx.x * RPB;
  if (t0 >= m) return;  // uniform for the block
  const int64_t t1 = t0 + RPB < m ? t0 + RPB : m;
  const int32_t c_lo = srank[t0], c_hi = srank[t1 - 1];
  const int ncell = c_hi - c_lo + 1;  // every cell has at least one row here, so ncell <= RPB
  for (int i = threadIdx.x; i < ncell * C; i += 256) lds[i] = 0u;  // 0.0f, and below every encoded float
  __syncthreads();
  const int g = threadIdx.x >> 3, l = threadIdx.x & 7;
  const int steps = RPB >> 5;
  for (int cc = 0; cc < C; cc += 64) {
    const int ch = cc + 8 * l;
    if (ch < C) {
      uint4 v[8];
      int32_t slot[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int64_t t = t0 + g + 32 * i;
        slot[i] = -1;
        if (i < steps && t < t1) {
          const int64_t p = perm[t];
          slot[i] = srank[t] - c_lo;
          v[i] = *reinterpret_cast<const uint4*>(img + p * C + ch);
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (slot[i] >= 0) {
          float f[8];
          unpack8(v[i], f);
          uint32_t* a = lds + slot[i] * C + ch;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if (MODE == 0) atomicAdd(reinterpret_cast<float*>(a + e), f[e]);
            else atomicMax(a + e, f2ord(f[e]));
          }
        }
      }
    }
  }
  __syncthreads();
  const int chunks = C >> 3;
  for (int w = threadIdx.x; w < ncell * chunks; w += 256) {
    const int s = w / chunks, k = w - s * chunks;
    const int64_t r = c_lo + s;
    const int64_t a = starts[r], b = starts[r + 1];
    const uint32_t* src = lds + s * C + 8 * k;
    if (a / RPB == (b - 1) / RPB) {  // the whole cell lies in this block's rows
      float f[8];
      const float cnt = (float)(b - a);
#pragma unroll
      for (int e = 0; e < 8; ++e) f[e] = MODE == 0 ? __uint_as_float(src[e]) / cnt : ord2f(src[e]);
      *reinterpret_cast<uint4*>(feats + r * C + 8 * k) = pack8(f);
    } else {  // continues across a block boundary: combine in the accumulator of the block it starts in
      uint32_t* dst = acc + (a / RPB) * C + 8 * k;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (MODE == 0) unsafeAtomicAdd(reinterpret_cast<float*>(dst + e), __uint_as_float(src[e]));
        else atomicMax(dst + e, src[e]);
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

__global__ void __launch_bounds__(256) k_fuse_init(const int32_t* __restrict__ d_n, int64_t capacity,
                                                   int32_t* __restrict__ src_l, int32_t* __restrict__ src_i) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n) return;
  src_l[r] = -1;
  src_i[r] = -1;
}

// One thread per input row: its rank in the union index is its output row.
__global__ void __launch_bounds__(256) k_fuse_place(const int4* __restrict__ coords, const int32_t* __restrict__ d_n_in,
                                                    int64_t capacity_in, const cellword_t* __restrict__ idx, int gx, int gy,
                                                    int gz, int n_batch, int64_t capacity_out, int32_t* __restrict__ src,
                                                    int4* __restrict__ coords_out) {
  int64_t n = *d_n_in;
  if (n > capacity_in) n = capacity_in;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int4 c = coords[i];  // (b, z, y, x)
  if ((unsigned)c.x >= (unsigned)n_batch || (unsigned)c.y >= (unsigned)gz || (unsigned)c.z >= (unsigned)gy ||
      (unsigned)c.w >= (unsigned)gx)
    return;  // malformed coordinate: it was not marked either
  const uint64_t key = (((uint64_t)c.x * gz + (uint64_t)c.y) * gy + (uint64_t)c.z) * gx + (uint64_t)c.w;
  const int32_t r = cell_lookup(idx, key);
  if (r < 0 || r >= capacity_out) return;
  src[r] = (int32_t)i;
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

  const int RPB = C <= 64 ? 256 : (C <= 128 ? 128 : 64);  // RPB * C accumulators fit the block's LDS
  const int64_t bound = npix < capacity ? npix : capacity;  // at most this many cells exist
  const dim3 blk(256), pg((unsigned)emc2_div_up(npix, 256)), cg((unsigned)emc2_div_up(bound, 256));
  const int64_t scan_blocks = emc2_div_up(bound, 2048);
  const int64_t red_blocks = emc2_div_up(npix, RPB);
  if (scan_blocks > ctx->n_pool_totals)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pool_image: capacity beyond the context's scan scratch");

  emc2_index_clear(ctx, idx, s);
  hipLaunchKernelGGL(k_pool_mark, pg, blk, 0, s, d_depth, npix, prm, idx, emc2_slot_flags(ctx, idx));
  emc2_index_scan(ctx, idx, n_cells, capacity, d_n_cells, s);
  hipLaunchKernelGGL(k_pool_zero_counts, cg, blk, 0, s, d_n_cells, capacity, d_counts);
  hipLaunchKernelGGL(k_pool_count, pg, blk, 0, s, d_depth, npix, prm, idx, capacity, (int4*)d_coords, d_counts, ctx->pix_rank,
                     ctx->pix_pos);
  hipLaunchKernelGGL(k_starts_reduce, dim3((unsigned)scan_blocks), blk, 0, s, d_counts, d_n_cells, capacity, ctx->pool_totals);
  hipLaunchKernelGGL(k_starts_apply, dim3((unsigned)scan_blocks), blk, 0, s, d_counts, d_n_cells, capacity, ctx->pool_totals,
                     ctx->cell_start);
  hipLaunchKernelGGL(k_pool_scatter, pg, blk, 0, s, npix, ctx->pix_rank, ctx->pix_pos, ctx->cell_start, ctx->pix_perm,
                     ctx->pix_srank);
  {
    const int64_t n16 = red_blocks * C / 4;  // C is a multiple of 8
    hipLaunchKernelGGL(k_pool_fill_zero, dim3((unsigned)emc2_div_up(n16, 256)), blk, 0, s, (uint4*)ctx->pool_acc, n16);
  }
  const dim3 rg((unsigned)red_blocks), fg((unsigned)emc2_div_up(bound * (C / 8), 256));
  if (mode == EMC2_POOL_MEAN) {
    hipLaunchKernelGGL(k_pool_reduce<0>, rg, blk, 0, s, (const __half*)d_img, ctx->pix_perm, ctx->pix_srank, ctx->cell_start,
                       d_n_cells, capacity, C, RPB, ctx->pool_acc, (__half*)d_feats);
    hipLaunchKernelGGL(k_pool_finish<0>, fg, blk, 0, s, ctx->cell_start, d_n_cells, capacity, C, RPB, ctx->pool_acc,
                       (__half*)d_feats);
  } else {
    hipLaunchKernelGGL(k_pool_reduce<1>, rg, blk, 0, s, (const __half*)d_img, ctx->pix_perm, ctx->pix_srank, ctx->cell_start,
                       d_n_cells, capacity, C, RPB, ctx->pool_acc, (__half*)d_feats);
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
  emc2_index_mark_coords(ctx, idx, d_coords_l, d_n_l, capacity_l, grid, n_batch, s);
  emc2_index_mark_coords(ctx, idx, d_coords_i, d_n_i, capacity_i, grid, n_batch, s);
  emc2_index_scan(ctx, idx, n_cells, capacity_out, d_n_out, s);
  const int64_t bound = capacity_l + capacity_i < capacity_out ? capacity_l + capacity_i : capacity_out;
  hipLaunchKernelGGL(k_fuse_init, dim3((unsigned)emc2_div_up(bound, 256)), blk, 0, s, d_n_out, capacity_out, src_l, src_i);
  hipLaunchKernelGGL(k_fuse_place, dim3((unsigned)emc2_div_up(capacity_l, 256)), blk, 0, s, (const int4*)d_coords_l, d_n_l,
                     capacity_l, idx, grid[0], grid[1], grid[2], n_batch, capacity_out, src_l, (int4*)d_coords_out);
  hipLaunchKernelGGL(k_fuse_place, dim3((unsigned)emc2_div_up(capacity_i, 256)), blk, 0, s, (const int4*)d_coords_i, d_n_i,
                     capacity_i, idx, grid[0], grid[1], grid[2], n_batch, capacity_out, src_i, (int4*)d_coords_out);
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
