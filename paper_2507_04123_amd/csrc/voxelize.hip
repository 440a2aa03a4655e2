// Voxelization with mean voxel features (paper Sec. 2 / Sec. 3.1 voxelization in the data bridge;
// Sec. 3.5 configurable pool size).
//
// Pass 1 (one thread per point): cell key -> open-addressing hash insert with 64-bit atomic CAS;
//   the point's x, y, z, intensity and a count are added atomically into the record it landed in.
//   The thread that wins the CAS for a new key sets the voxel's bit in the cell index and takes a
//   dense id from a wavefront-aggregated counter (one atomic per wave), listing the hash slot.
// Scan: prefix sum over the cell index -> rank of every active cell = its position in key order.
// Pass 2 (one thread per distinct voxel): slot -> key -> rank; write coords, mean, count at rank.
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

__device__ __forceinline__ uint64_t hash64(uint64_t k) {
  k ^= k >> 33;
  k *= 0xff51afd7ed558ccdull;
  k ^= k >> 33;
  return k;
}

// Clears the hash records [0, n_rec) and the two counters used by this call.
__global__ void __launch_bounds__(256) k_table_clear(VoxRec* __restrict__ table, int64_t n_rec,
                                                     int32_t* __restrict__ dev_words) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  uint4* p = reinterpret_cast<uint4*>(table);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < 2 * n_rec; i += stride)
    p[i] = (i & 1) ? make_uint4(0u, 0u, 0u, 0u) : make_uint4(0xFFFFFFFFu, 0xFFFFFFFFu, 0u, 0u);
  if (blockIdx.x == 0 && threadIdx.x == 0) dev_words[1] = 0;
}

// Cell along one axis per the definition: fp32 subtract, fp32 IEEE division, floor; -1 if outside.
__device__ __forceinline__ int cell_of(float p, float lo, float vs, int g) {
  const float t = (p - lo) / vs;  // separately rounded ops: contraction is off in this file
  if (!(t >= 0.0f) || !(t < (float)g)) return -1;
  return (int)floorf(t);
}

__global__ void __launch_bounds__(256) k_vox_insert(const float* __restrict__ points, const int32_t* __restrict__ batch,
                                                    int64_t n_points, VoxParams prm, VoxRec* __restrict__ table,
                                                    uint32_t slot_mask, cellword_t* __restrict__ idx,
                                                    int32_t* __restrict__ uslot, int64_t capacity,
                                                    int32_t* __restrict__ dev_words, uint32_t* __restrict__ flags) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  bool keep = i < n_points;
  float px = 0.f, py = 0.f, pz = 0.f, pi = 0.f;
  uint64_t key = 0;
  if (keep) {
    const float* p = points + i * prm.stride_f;
    if ((prm.stride_f & 3) == 0) {
      const float4 v = *reinterpret_cast<const float4*>(p);
      px = v.x; py = v.y; pz = v.z; pi = v.w;
    } else {
      px = p[0]; py = p[1]; pz = p[2]; pi = p[3];
    }
    const int b = batch ? batch[i] : 0;
    const int cx = cell_of(px, prm.lo[0], prm.vs[0], prm.grid[0]);
    const int cy = cell_of(py, prm.lo[1], prm.vs[1], prm.grid[1]);
    const int cz = cell_of(pz, prm.lo[2], prm.vs[2], prm.grid[2]);
    const float xx = px * px, yy = py * py;
    const float r2 = xx + yy;  // each product rounded on its own (no fused multiply-add)
    keep = (b >= 0) && (b < prm.n_batch) && (cx >= 0) && (cy >= 0) && (cz >= 0) && (r2 >= prm.r2_min) &&
           (r2 < prm.r2_max) && (fabsf(pi) <= 3.402823466e38f);  // last test rejects NaN/inf intensity
    key = (((uint64_t)b * prm.grid[2] + (uint64_t)cz) * prm.grid[1] + (uint64_t)cy) * prm.grid[0] + (uint64_t)cx;
  }
  bool is_new = false;
  uint32_t slot = 0;
  if (keep) {
    slot = (uint32_t)hash64(key) & slot_mask;
    bool placed = false;
    for (uint32_t probe = 0; probe <= slot_mask; ++probe) {
      const unsigned long long prev = atomicCAS(&table[slot].key, EMC2_EMPTY_KEY, (unsigned long long)key);
      if (prev == EMC2_EMPTY_KEY) { is_new = true; placed = true; break; }
      if (prev == key) { placed = true; break; }
      slot = (slot + 1) & slot_mask;
    }
    if (placed) {
      VoxRec* r = table + slot;
      unsafeAtomicAdd(&r->sum[0], px);
      unsafeAtomicAdd(&r->sum[1], py);
      unsafeAtomicAdd(&r->sum[2], pz);
      unsafeAtomicAdd(&r->sum[3], pi);
      atomicAdd(&r->count, 1u);
    } else {
      atomicOr(&dev_words[0], EMC2_DEVFLAG_HASH_FULL);
    }
  }
  // wavefront-ballot compaction of the new voxels: one counter atomic per wave
  const unsigned long long m = __ballot(is_new);
  if (m != 0ull) {
    const int lane = threadIdx.x & 63;
    const int leader = __ffsll((long long)m) - 1;
    int32_t base = 0;
    if (lane == leader) base = atomicAdd(&dev_words[1], __popcll(m));
    base = __shfl(base, leader, 64);
    if (is_new) {
      const int32_t id = base + __popcll(m & ((1ull << lane) - 1ull));
      if (id < capacity) uslot[id] = (int32_t)slot;
      else atomicOr(&dev_words[0], EMC2_DEVFLAG_CAPACITY);
      atomicOr(&idx[key >> 5].x, 1u << ((uint32_t)key & 31u));
      flags[key >> (5 + EMC2_TILE_SHIFT)] = 1u;   // this tile of the index now holds a bit
    }
  }
}

template <int LP>  // 0 none, 1 fp16, 2 bf16
__global__ void __launch_bounds__(256) k_vox_finalize(const VoxRec* __restrict__ table, const int32_t* __restrict__ uslot,
                                                      const cellword_t* __restrict__ idx, const int32_t* __restrict__ dev_words,
                                                      int64_t capacity, int gx, int gy, int gz, int4* __restrict__ coords,
                                                      float4* __restrict__ feats, int32_t* __restrict__ counts,
                                                      void* __restrict__ feats_lp) {
  int64_t n = dev_words[1];
  if (n > capacity) n = capacity;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= n) return;
  const VoxRec rec = table[uslot[id]];
  const int32_t r = cell_lookup(idx, rec.key);
  if (r < 0 || r >= capacity) return;
  coords[r] = decode_key(rec.key, gx, gy, gz);
  const float c = (float)rec.count;
  const float4 m = make_float4(rec.sum[0] / c, rec.sum[1] / c, rec.sum[2] / c, rec.sum[3] / c);
  feats[r] = m;
  counts[r] = (int32_t)rec.count;
  if (LP == 1) {
    __half2* o = reinterpret_cast<__half2*>(feats_lp) + 2 * (int64_t)r;
    o[0] = __floats2half2_rn(m.x, m.y);
    o[1] = __floats2half2_rn(m.z, m.w);
  } else if (LP == 2) {
    __hip_bfloat16* o = reinterpret_cast<__hip_bfloat16*>(feats_lp) + 4 * (int64_t)r;
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

  // hash size for this call: >= 2x the most distinct voxels it can legally hold
  int64_t want = 2 * (n_points < capacity ? n_points : capacity);
  int64_t n_rec = 1024;
  while (n_rec < want) n_rec <<= 1;
  if (n_rec > ctx->table_slots) n_rec = ctx->table_slots;

  VoxParams prm;
  for (int a = 0; a < 3; ++a) { prm.lo[a] = spec->lo[a]; prm.vs[a] = spec->vs[a]; prm.grid[a] = spec->grid[a]; }
  prm.n_batch = spec->n_batch;
  prm.r2_min = spec->r2_min;
  prm.r2_max = spec->r2_max;
  prm.stride_f = spec->stride_f;

  emc2_index_clear(ctx, idx, s);
  {
    int64_t blocks = emc2_div_up(2 * n_rec, 256 * 4);
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_table_clear, dim3((unsigned)blocks), dim3(256), 0, s, ctx->table, n_rec, ctx->dev_words);
  }
  if (n_points > 0)
    hipLaunchKernelGGL(k_vox_insert, dim3((unsigned)emc2_div_up(n_points, 256)), dim3(256), 0, s, d_points, d_batch,
                       n_points, prm, ctx->table, (uint32_t)(n_rec - 1), idx, ctx->uslot, capacity, ctx->dev_words,
                       emc2_slot_flags(ctx, idx));
  emc2_index_scan(ctx, idx, n_cells, capacity, d_n_voxels, s);
  {
    // at most min(n_points, capacity) distinct voxels were listed
    const int64_t bound = n_points < capacity ? n_points : capacity;
    if (bound > 0) {
      const dim3 g((unsigned)emc2_div_up(bound, 256)), b(256);
      const int lp = d_feats_lp ? (lp_dtype == EMC2_F16 ? 1 : 2) : 0;
#define FIN(LP)                                                                                                  \
  hipLaunchKernelGGL(k_vox_finalize<LP>, g, b, 0, s, ctx->table, ctx->uslot, idx, ctx->dev_words, capacity,       \
                     spec->grid[0], spec->grid[1], spec->grid[2], (int4*)d_coords, (float4*)d_feats, d_counts,    \
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
