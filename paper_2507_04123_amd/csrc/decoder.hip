// Decoder-side pieces: the inverse (transposed) kernel map of a stride-2 layer (paper Sec. 3.1: the LiDAR
// branch is a UNet plus a sparse CNN, so features travel back up the resolution levels) and the
// bird's-eye-view flattening of a voxel set (Sec. 3.3: the latency-prioritised expert works on BEV).
#include "common.h"

namespace {

// One thread per fine voxel.  Fine site i is read by the coarse site at (i + 1 - k)/2 where that is integral on
// every axis: per axis one tap (k = 1) for an even coordinate, two (k = 0, 2) for an odd one, so 1 to 8 of the
// 27 entries can be valid; each is one lookup in the coarse level's cell index.
__global__ void __launch_bounds__(256) k_inverse_probe(const int4* __restrict__ fine_coords, const int32_t* __restrict__ d_n_fine,
                                                       int64_t capacity_fine, const cellword_t* __restrict__ coarse_idx,
                                                       const int32_t* __restrict__ d_n_coarse, int gx, int gy, int gz,
                                                       int n_batch, int32_t* __restrict__ nbr) {
  int64_t n = *d_n_fine;
  if (n > capacity_fine) n = capacity_fine;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t n_coarse = *d_n_coarse;
  const int4 c = fine_coords[i];  // (b, z, y, x)
  const bool sane = (unsigned)c.x < (unsigned)n_batch && c.y >= 0 && c.z >= 0 && c.w >= 0;
#pragma unroll
  for (int kz = 0; kz < 3; ++kz) {
    const int tz = c.y + 1 - kz;
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
      const int ty = c.z + 1 - ky;
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) {
        const int tx = c.w + 1 - kx;
        int32_t j = -1;
        const bool par = sane && !((tx | ty | tz) & 1) && tx >= 0 && ty >= 0 && tz >= 0;
        if (par) {
          const int ox = tx >> 1, oy = ty >> 1, oz = tz >> 1;
          if (ox < gx && oy < gy && oz < gz) {
            const uint64_t key = (((uint64_t)c.x * gz + (uint64_t)oz) * gy + (uint64_t)oy) * gx + (uint64_t)ox;
            j = cell_lookup(coarse_idx, key);
            if (j >= n_coarse) j = -1;  // only after a capacity overflow upstream
          }
        }
        nbr[(int64_t)((kz * 3 + ky) * 3 + kx) * capacity_fine + i] = j;
      }
    }
  }
}

__global__ void __launch_bounds__(256) k_fill_zero16(uint4* __restrict__ p, int64_t n16) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

__global__ void __launch_bounds__(256) k_fill_zero4(uint32_t* __restrict__ p, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4) p[i] = 0u;
}

// One thread per (voxel, 4-byte word of its feature row): consecutive threads copy consecutive words, so a
// row moves as whole cache lines on both sides.
__global__ void __launch_bounds__(256) k_bev_scatter(const int4* __restrict__ coords, const uint32_t* __restrict__ feats,
                                                     const int32_t* __restrict__ d_n, int64_t capacity, int gx, int gy, int gz,
                                                     int n_batch, int row_words, uint32_t* __restrict__ out) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t v = t / row_words;
  if (v >= n) return;
  const int w = (int)(t - v * row_words);
  const int4 c = coords[v];  // (b, z, y, x)
  if ((unsigned)c.x >= (unsigned)n_batch || (unsigned)c.y >= (unsigned)gz || (unsigned)c.z >= (unsigned)gy ||
      (unsigned)c.w >= (unsigned)gx)
    return;  // malformed coordinate: ignore rather than write out of bounds
  const int64_t cell = (((int64_t)c.x * gy + c.z) * gx + c.w) * gz + c.y;
  out[cell * row_words + w] = feats[v * row_words + w];
}

}  // namespace

extern "C" emc2_status emc2_build_inverse_kmap(emc2_ctx* ctx, const int32_t* d_fine_coords, const int32_t* d_n_fine,
                                               int64_t capacity_fine, const int32_t grid_coarse[3], int32_t n_batch,
                                               int32_t coarse_slot, const int32_t* d_n_coarse, int32_t* d_nbr,
                                               void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_fine_coords || !d_n_fine || !grid_coarse || !d_n_coarse || !d_nbr)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_inverse_kmap: null argument");
  if (capacity_fine < 1) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_inverse_kmap: capacity_fine < 1");
  int64_t cells = 0;
  if (!emc2_grid_ok(grid_coarse, n_batch, &cells))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_build_inverse_kmap: grid/batch out of the supported key range");
  if (coarse_slot < 0 || coarse_slot >= ctx->n_slots)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_inverse_kmap: coarse_slot outside [0, %d)", ctx->n_slots);
  const SlotMeta& m = ctx->meta[coarse_slot];
  if (!m.valid || m.n_batch != n_batch || m.grid[0] != grid_coarse[0] || m.grid[1] != grid_coarse[1] ||
      m.grid[2] != grid_coarse[2])
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_inverse_kmap: coarse_slot %d does not hold an index for this grid",
                     coarse_slot);
  hipStream_t s = (hipStream_t)stream;
  hipLaunchKernelGGL(k_inverse_probe, dim3((unsigned)emc2_div_up(capacity_fine, 256)), dim3(256), 0, s,
                     (const int4*)d_fine_coords, d_n_fine, capacity_fine, ctx->slots[coarse_slot], d_n_coarse, grid_coarse[0],
                     grid_coarse[1], grid_coarse[2], n_batch, d_nbr);
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_build_inverse_kmap launch");
}

extern "C" emc2_status emc2_bev_flatten(emc2_ctx* ctx, emc2_dtype dtype, const int32_t* d_coords, const void* d_feats,
                                        const int32_t* d_n, int64_t capacity, const int32_t grid[3], int32_t n_batch,
                                        int32_t channels, void* d_out, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_coords || !d_feats || !d_n || !grid || !d_out)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_bev_flatten: null argument");
  if (dtype != EMC2_F32 && dtype != EMC2_F16 && dtype != EMC2_BF16)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_bev_flatten: bad dtype");
  if (capacity < 1 || channels < 1 || channels > 4096)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_bev_flatten: capacity < 1 or channels outside [1, 4096]");
  int64_t cells = 0;
  if (!emc2_grid_ok(grid, n_batch, &cells))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_bev_flatten: grid/batch out of the supported key range");
  const int64_t row_bytes = (int64_t)channels * (dtype == EMC2_F32 ? 4 : 2);
  if (row_bytes % 4 != 0)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_bev_flatten: a feature row must be a multiple of 4 bytes");
  const int row_words = (int)(row_bytes / 4);
  const int64_t words = cells * row_words;
  hipStream_t s = (hipStream_t)stream;
  const int64_t n16 = words / 4;
  if (n16 > 0) {
    int64_t blocks = emc2_div_up(n16, 256 * 4);
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(k_fill_zero16, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)d_out, n16);
  }
  if (words - 4 * n16 > 0)
    hipLaunchKernelGGL(k_fill_zero4, dim3(1), dim3(256), 0, s, (uint32_t*)d_out + 4 * n16, words - 4 * n16);
  const int64_t threads = capacity * row_words;
  hipLaunchKernelGGL(k_bev_scatter, dim3((unsigned)emc2_div_up(threads, 256)), dim3(256), 0, s, (const int4*)d_coords,
                     (const uint32_t*)d_feats, d_n, capacity, grid[0], grid[1], grid[2], n_batch, row_words, (uint32_t*)d_out);
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_bev_flatten launch");
}
