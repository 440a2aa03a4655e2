// Voxelization with mean voxel features (paper Sec. 2 / Sec. 3.1 voxelization in the data bridge;
// Sec. 3.5 configurable pool size; Sec. 3.6 (3) prefix-sum index search).
//
// The voxel index of a cell is its rank in the prefix-summed cell index, so no hash table is needed:
// Pass 1 (one thread per point): cell key -> set the cell's bit in the index (one atomic OR per point); the same
//   launch zeroes the output rows pass 2 accumulates into.
// Scan: prefix sum over the index -> the rank of every active cell = its position in key order, and the
//   number of voxels.
// Pass 2 (one thread per point): the same key again -> rank r (one 8-byte load) -> position within the
//   voxel from one returning atomic add on counts[r] -> the point goes to slot `pos` of the voxel's stash
//   (a plain 16-byte store); only points beyond the stash depth are added atomically into the output row.
// Pass 3 (one thread per voxel): sum the stash in the order of the points' values, divide, write the means.
// Device-scope atomics on this part execute at the memory side of the fabric (the L2s of the 8 XCDs are
// not coherent with each other), about 17 G/s in aggregate: two per point instead of seven is what
// this layout buys.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <math.h>

#include "common.h"

// The cell index and the range filter are defined by individually rounded IEEE fp32 operations;
// plain operators under this pragma stay unfused (intrinsics from headers would not).
#pragma clang fp contract(off)

namespace {

struct VoxParams {
  float lo[3];
  float vs[3];
  int32_t grid[3];
  int32_t n_batch;
  float r2_min, r2_max;
  int32_t stride_f;
};

// Cell along one axis per the definition: fp32 subtract, fp32 IEEE division, floor; -1 if outside.
__device__ __forceinline__ int cell_of(float p, float lo, float vs, int g) {
  const float t = (p - lo) / vs;  // separately rounded ops: contraction is off in this file
  if (!(t >= 0.0f) || !(t < (float)g)) return -1;
  return (int)floorf(t);
}

struct PointCell {
  float4 p;       // x, y, z, intensity
  int4 c;         // (b, z, y, x)
  uint64_t key;
  bool keep;
};

// Both point passes call this, so they agree on every point's fate and cell bit for bit.
__device__ __forceinline__ PointCell locate(const float* __restrict__ points, const int32_t* __restrict__ batch, int64_t i,
                                            int64_t n_points, const VoxParams& prm) {
  PointCell r;
  r.keep = i < n_points;
  r.p = make_float4(0.f, 0.f, 0.f, 0.f);
  r.c = make_int4(0, 0, 0, 0);
  r.key = 0;
  if (r.keep) {
    const float* p = points + i * prm.stride_f;
    if ((prm.stride_f & 3) == 0) {
      r.p = *reinterpret_cast<const float4*>(p);
    } else {
      r.p = make_float4(p[0], p[1], p[2], p[3]);
    }
    const int b = batch ? batch[i] : 0;
    const int cx = cell_of(r.p.x, prm.lo[0], prm.vs[0], prm.grid[0]);
    const int cy = cell_of(r.p.y, prm.lo[1], prm.vs[1], prm.grid[1]);
    const int cz = cell_of(r.p.z, prm.lo[2], prm.vs[2], prm.grid[2]);
    const float xx = r.p.x * r.p.x, yy = r.p.y * r.p.y;
    const float r2 = xx + yy;  // each product rounded on its own (no fused multiply-add)
    r.keep = (b >= 0) && (b < prm.n_batch) && (cx >= 0) && (cy >= 0) && (cz >= 0) && (r2 >= prm.r2_min) &&
             (r2 < prm.r2_max) && (fabsf(r.p.w) <= 3.402823466e38f);  // last test rejects NaN/inf intensity
    r.c = make_int4(b, cz, cy, cx);
    r.key = (((uint64_t)b * prm.grid[2] + (uint64_t)cz) * prm.grid[1] + (uint64_t)cy) * prm.grid[0] + (uint64_t)cx;
  }
  return r;
}

__global__ void __launch_bounds__(256) k_vox_mark(const float* __restrict__ points, const int32_t* __restrict__ batch,
                                                  int64_t n_points, VoxParams prm, cellword_t* __restrict__ idx,
                                                  lineflag_t* __restrict__ flags, int64_t zero_rows,
                                                  float4* __restrict__ feats, int32_t* __restrict__ counts) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  // the rows pass 2 accumulates into: there are at most min(n_points, capacity) voxels, one thread each
  if (i < zero_rows) {
    feats[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    counts[i] = 0;
  }
  const PointCell pc = locate(points, batch, i, n_points, prm);
  if (!pc.keep) return;
  atomicOr(&idx[pc.key >> 5].x, 1u << ((uint32_t)pc.key & 31u));
  flags[emc2_line_of_key(pc.key)] = 1;   // this line of the index now holds a bit
}

__global__ void __launch_bounds__(256) k_vox_scatter(const float* __restrict__ points, const int32_t* __restrict__ batch,
                                                     int64_t n_points, VoxParams prm, const cellword_t* __restrict__ idx,
                                                     int64_t capacity, int4* __restrict__ coords,
                                                     float4* __restrict__ feats, int32_t* __restrict__ counts,
                                                     float4* __restrict__ stash) {
  const PointCell pc = locate(points, batch, (int64_t)blockIdx.x * blockDim.x + threadIdx.x, n_points, prm);
  if (!pc.keep) return;
  const int32_t r = cell_lookup(idx, pc.key);
  if (r < 0 || r >= capacity) return;   // beyond capacity: reported by the scan, dropped here
  const int32_t pos = atomicAdd(&counts[r], 1);
  coords[r] = pc.c;                     // every point of the voxel writes the same value
  if (pos < EMC2_VOX_STASH) {
    stash[(int64_t)r * EMC2_VOX_STASH + pos] = pc.p;
  } else {
    float* f = reinterpret_cast<float*>(feats + r);
    unsafeAtomicAdd(f + 0, pc.p.x);
    unsafeAtomicAdd(f + 1, pc.p.y);
    unsafeAtomicAdd(f + 2, pc.p.z);
    unsafeAtomicAdd(f + 3, pc.p.w);
  }
}

template <int LP>  // 0 none, 1 fp16, 2 bf16
__global__ void __launch_bounds__(256) k_vox_finalize(const int32_t* __restrict__ d_n, int64_t capacity,
                                                      const float4* __restrict__ stash, float4* __restrict__ feats,
                                                      const int32_t* __restrict__ counts, void* __restrict__ feats_lp) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n) return;
  const int32_t cnt = counts[r];
  float4 s = feats[r];   // what overflowed the stash (zero for almost every voxel)
  const int k = cnt < EMC2_VOX_STASH ? cnt : EMC2_VOX_STASH;
  // The stash holds the points in arrival order, which differs from run to run.  They are summed in the order
  // of their values (x, then y, z, intensity) instead, so that a voxel of up to EMC2_VOX_STASH points -- nearly
  // every voxel of a LiDAR frame -- gets the same mean, bit for bit, in every run and for every order of the input.
  float4 v[EMC2_VOX_STASH];
#pragma unroll
  for (int j = 0; j < EMC2_VOX_STASH; ++j)
    v[j] = j < k ? stash[r * EMC2_VOX_STASH + j] : make_float4(INFINITY, INFINITY, INFINITY, INFINITY);
  auto before = [](const float4& a, const float4& b) {
    if (a.x != b.x) return a.x < b.x;
    if (a.y != b.y) return a.y < b.y;
    if (a.z != b.z) return a.z < b.z;
    return a.w < b.w;
  };
  auto order = [&](int a, int b) {   // compare-exchange: v[a] <= v[b] afterwards
    if (before(v[b], v[a])) { const float4 t = v[a]; v[a] = v[b]; v[b] = t; }
  };
  static_assert(EMC2_VOX_STASH == 4, "the sorting network below orders four entries");
  order(0, 1); order(2, 3); order(0, 2); order(1, 3); order(1, 2);
#pragma unroll
  for (int j = 0; j < EMC2_VOX_STASH; ++j)
    if (j < k) { s.x += v[j].x; s.y += v[j].y; s.z += v[j].z; s.w += v[j].w; }
  const float c = (float)cnt;
  const float4 m = make_float4(s.x / c, s.y / c, s.z / c, s.w / c);
  feats[r] = m;
  if (LP == 1) {
    __half2* o = reinterpret_cast<__half2*>(feats_lp) + 2 * r;
    o[0] = __floats2half2_rn(m.x, m.y);
    o[1] = __floats2half2_rn(m.z, m.w);
  } else if (LP == 2) {
    __hip_bfloat16* o = reinterpret_cast<__hip_bfloat16*>(feats_lp) + 4 * r;
    o[0] = __float2bfloat16(m.x); o[1] = __float2bfloat16(m.y);
    o[2] = __float2bfloat16(m.z); o[3] = __float2bfloat16(m.w);
  }
}

}  // namespace

extern "C" emc2_status emc2_voxelize(emc2_ctx* ctx, const float* d_points, const int32_t* d_batch, int64_t n_points,
                                     const emc2_voxel_spec* spec, int64_t capacity, int32_t* d_coords, float* d_feats,
                                     int32_t* d_counts, void* d_feats_lp, emc2_dtype lp_dtype, int32_t* d_n_voxels,
                                     int32_t* h_n_voxels, int32_t index_slot, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!spec || !d_coords || !d_feats || !d_counts || !d_n_voxels)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: null argument");
  if (n_points < 0 || (n_points > 0 && !d_points))
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: bad points");
  if (n_points > ctx->max_points)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: n_points %lld > max_points %lld", (long long)n_points,
                     (long long)ctx->max_points);
  if (capacity < 1 || capacity > ctx->max_voxels)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: capacity %lld outside [1, max_voxels %lld]",
                     (long long)capacity, (long long)ctx->max_voxels);
  if (index_slot < 0 || index_slot >= ctx->n_slots)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: index_slot %d outside [0, %d)", index_slot, ctx->n_slots);
  if (spec->stride_f < 4) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: stride_f < 4");
  for (int a = 0; a < 3; ++a)
    if (!(spec->vs[a] > 0.0f) || !isfinite(spec->vs[a]) || !isfinite(spec->lo[a]))
      return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: bad voxel size / lower bound");
  if (d_feats_lp && lp_dtype != EMC2_F16 && lp_dtype != EMC2_BF16)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: lp_dtype must be F16 or BF16");
  int64_t n_cells = 0;
  if (!emc2_grid_ok(spec->grid, spec->n_batch, &n_cells))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_voxelize: grid/batch out of the supported key range");
  if (n_cells > ctx->max_cells)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_voxelize: %lld cells > max_cells %lld", (long long)n_cells,
                     (long long)ctx->max_cells);

  hipStream_t s = (hipStream_t)stream;
  cellword_t* idx = ctx->slots[index_slot];
  SlotMeta& mt = ctx->meta[index_slot];
  for (int a = 0; a < 3; ++a) mt.grid[a] = spec->grid[a];
  mt.n_batch = spec->n_batch;
  mt.valid = true;

  VoxParams prm;
  for (int a = 0; a < 3; ++a) { prm.lo[a] = spec->lo[a]; prm.vs[a] = spec->vs[a]; prm.grid[a] = spec->grid[a]; }
  prm.n_batch = spec->n_batch;
  prm.r2_min = spec->r2_min;
  prm.r2_max = spec->r2_max;
  prm.stride_f = spec->stride_f;

  emc2_index_clear(ctx, idx, s);
  const dim3 pg((unsigned)emc2_div_up(n_points > 0 ? n_points : 1, 256)), blk(256);
  // at most min(n_points, capacity) voxels exist
  const int64_t bound = n_points < capacity ? n_points : capacity;
  if (n_points > 0)
    hipLaunchKernelGGL(k_vox_mark, pg, blk, 0, s, d_points, d_batch, n_points, prm, idx, emc2_slot_flags(ctx, idx), bound,
                       (float4*)d_feats, d_counts);
  emc2_index_scan(ctx, idx, n_cells, capacity, d_n_voxels, s);
  {
    if (bound > 0) {
      const dim3 vg((unsigned)emc2_div_up(bound, 256));
      hipLaunchKernelGGL(k_vox_scatter, pg, blk, 0, s, d_points, d_batch, n_points, prm, idx, capacity, (int4*)d_coords,
                         (float4*)d_feats, d_counts, ctx->stash);
      const int lp = d_feats_lp ? (lp_dtype == EMC2_F16 ? 1 : 2) : 0;
#define FIN(LP)                                                                                                 \
  hipLaunchKernelGGL(k_vox_finalize<LP>, vg, blk, 0, s, d_n_voxels, capacity, ctx->stash, (float4*)d_feats, d_counts, \
                     d_feats_lp)
      if (lp == 0) FIN(0); else if (lp == 1) FIN(1); else FIN(2);
#undef FIN
    }
  }
  emc2_status st = emc2_check_hip(ctx, hipGetLastError(), "emc2_voxelize launch");
  if (st != EMC2_OK) return st;
  if (h_n_voxels) {
    st = emc2_check_hip(ctx, hipMemcpyAsync(ctx->pinned + 1, d_n_voxels, sizeof(int32_t), hipMemcpyDeviceToHost, s),
                        "hipMemcpyAsync(n_voxels)");
    if (st != EMC2_OK) return st;
    st = emc2_check_hip(ctx, hipStreamSynchronize(s), "hipStreamSynchronize");
    if (st != EMC2_OK) return st;
    *h_n_voxels = ctx->pinned[1];
  }
  return EMC2_OK;
}
