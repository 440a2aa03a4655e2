// Context: owns every scratch buffer of the library; nothing else allocates device memory.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "common.h"

emc2_status emc2_fail(emc2_ctx* ctx, emc2_status st, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

emc2_status emc2_check_hip(emc2_ctx* ctx, hipError_t e, const char* what) {
  if (e == hipSuccess) return EMC2_OK;
  return emc2_fail(ctx, EMC2_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

bool emc2_grid_ok(const int32_t grid[3], int32_t n_batch, int64_t* n_cells) {
  if (!grid || n_batch < 1) return false;
  for (int a = 0; a < 3; ++a)
    if (grid[a] < 1 || grid[a] > (1 << 20)) return false;
  // keep the linear key (and 32*word index arithmetic) comfortably inside 63 bits
  const long double cells = (long double)grid[0] * grid[1] * grid[2] * n_batch;
  if (cells > 1.0e15L) return false;
  *n_cells = (int64_t)grid[0] * grid[1] * grid[2] * n_batch;
  return true;
}

extern "C" emc2_status emc2_create(emc2_ctx** out, int device, int64_t max_points, int64_t max_voxels,
                                   int64_t max_cells, int32_t n_slots) {
  if (!out) return EMC2_ERR_INVALID_ARG;
  *out = nullptr;
  if (max_points < 1 || max_voxels < 1 || max_cells < 1 || n_slots < 1 || n_slots > 64)
    return EMC2_ERR_INVALID_ARG;
  if (max_points > (1ll << 30) || max_voxels > (1ll << 30)) return EMC2_ERR_INVALID_ARG;
  emc2_ctx* ctx = (emc2_ctx*)calloc(1, sizeof(emc2_ctx));
  if (!ctx) return EMC2_ERR_DEVICE;
  ctx->device = device;
  ctx->max_points = max_points;
  ctx->max_voxels = max_voxels;
  ctx->max_cells = max_cells;
  ctx->n_slots = n_slots;
  ctx->err[0] = 0;
  emc2_status st = EMC2_OK;
#define TRY(call, what)                                   \
  do {                                                    \
    st = emc2_check_hip(ctx, (call), what);               \
    if (st != EMC2_OK) goto fail;                         \
  } while (0)
  TRY(hipSetDevice(device), "hipSetDevice");
  // one spare word (a stride-2 mark may spill one word past the grid), rounded up to whole tiles
  ctx->slot_tiles = emc2_div_up(emc2_div_up(max_cells, 32) + 1, EMC2_SCAN_TILE);
  ctx->slot_words = ctx->slot_tiles * EMC2_SCAN_TILE;
  ctx->slots = (cellword_t**)calloc((size_t)n_slots + 2, sizeof(cellword_t*));
  ctx->meta = (SlotMeta*)calloc((size_t)n_slots + 2, sizeof(SlotMeta));
  if (!ctx->slots || !ctx->meta) { st = EMC2_ERR_DEVICE; goto fail; }
  for (int s = 0; s < n_slots + 2; ++s) {
    const size_t bytes = sizeof(cellword_t) * (size_t)ctx->slot_words + sizeof(lineflag_t) * (size_t)(ctx->slot_words >> EMC2_LINE_SHIFT);
    TRY(hipMalloc((void**)&ctx->slots[s], bytes), "hipMalloc(index slot)");
    TRY(hipMemset(ctx->slots[s], 0, bytes), "hipMemset(index slot)");  // establishes the line-flag invariant
  }
  TRY(hipMalloc((void**)&ctx->stash, sizeof(float4) * EMC2_VOX_STASH * (size_t)max_voxels), "hipMalloc(voxel stash)");
  ctx->n_partials = emc2_div_up(ctx->slot_words, EMC2_SCAN_TILE) + 1;
  TRY(hipMalloc((void**)&ctx->partials, sizeof(uint32_t) * (size_t)ctx->n_partials), "hipMalloc(partials)");
  TRY(hipMalloc((void**)&ctx->zero_row, 256), "hipMalloc(zero_row)");
  TRY(hipMemset(ctx->zero_row, 0, 256), "hipMemset(zero_row)");
  TRY(hipMalloc((void**)&ctx->pix_rank, sizeof(int32_t) * 4 * (size_t)max_points), "hipMalloc(pixel scratch)");
  ctx->pix_pos = ctx->pix_rank + max_points;
  ctx->pix_perm = ctx->pix_pos + max_points;
  ctx->pix_srank = ctx->pix_perm + max_points;
  TRY(hipMalloc((void**)&ctx->cell_start, sizeof(int32_t) * ((size_t)max_voxels + 1)), "hipMalloc(cell_start)");
  ctx->n_pool_totals = emc2_div_up(max_voxels, 2048) + 1;
  TRY(hipMalloc((void**)&ctx->pool_totals, sizeof(uint32_t) * (size_t)ctx->n_pool_totals), "hipMalloc(pool_totals)");
  TRY(hipMalloc((void**)&ctx->pool_acc, sizeof(uint32_t) * 256 * ((size_t)max_points / 64 + 2)), "hipMalloc(pool_acc)");
  TRY(hipMalloc((void**)&ctx->fuse_src, sizeof(int32_t) * 2 * (size_t)max_voxels), "hipMalloc(fuse_src)");
  TRY(hipMalloc((void**)&ctx->wpack, (size_t)27 * 128 * 128 * 2), "hipMalloc(wpack)");
  TRY(hipMalloc((void**)&ctx->dev_words, sizeof(int32_t) * 8), "hipMalloc(dev_words)");
  TRY(hipMemset(ctx->dev_words, 0, sizeof(int32_t) * 8), "hipMemset(dev_words)");
  TRY(hipHostMalloc((void**)&ctx->pinned, sizeof(int32_t) * 8, hipHostMallocDefault), "hipHostMalloc");
  TRY(hipDeviceSynchronize(), "hipDeviceSynchronize");
#undef TRY
  *out = ctx;
  return EMC2_OK;
fail:
  emc2_destroy(ctx);
  return st;
}

extern "C" void emc2_destroy(emc2_ctx* ctx) {
  if (!ctx) return;
  (void)hipSetDevice(ctx->device);
  if (ctx->slots) {
    for (int s = 0; s < ctx->n_slots + 2; ++s)
      if (ctx->slots[s]) (void)hipFree(ctx->slots[s]);
    free(ctx->slots);
  }
  free(ctx->meta);
  if (ctx->stash) (void)hipFree(ctx->stash);
  if (ctx->partials) (void)hipFree(ctx->partials);
  if (ctx->zero_row) (void)hipFree(ctx->zero_row);
  if (ctx->wpack) (void)hipFree(ctx->wpack);
  if (ctx->pix_rank) (void)hipFree(ctx->pix_rank);
  if (ctx->cell_start) (void)hipFree(ctx->cell_start);
  if (ctx->pool_totals) (void)hipFree(ctx->pool_totals);
  if (ctx->pool_acc) (void)hipFree(ctx->pool_acc);
  if (ctx->fuse_src) (void)hipFree(ctx->fuse_src);
  if (ctx->dev_words) (void)hipFree(ctx->dev_words);
  if (ctx->pinned) (void)hipHostFree(ctx->pinned);
  free(ctx);
}

extern "C" emc2_status emc2_status_sync(emc2_ctx* ctx, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  hipStream_t s = (hipStream_t)stream;
  emc2_status st = emc2_check_hip(ctx, hipMemcpyAsync(ctx->pinned, ctx->dev_words, sizeof(int32_t),
                                                      hipMemcpyDeviceToHost, s), "hipMemcpyAsync(status)");
  if (st != EMC2_OK) return st;
  st = emc2_check_hip(ctx, hipMemsetAsync(ctx->dev_words, 0, sizeof(int32_t), s), "hipMemsetAsync(status)");
  if (st != EMC2_OK) return st;
  st = emc2_check_hip(ctx, hipStreamSynchronize(s), "hipStreamSynchronize");
  if (st != EMC2_OK) return st;
  const int flags = ctx->pinned[0];
  if (flags & EMC2_DEVFLAG_CAPACITY)
    return emc2_fail(ctx, EMC2_ERR_CAPACITY, "device reported [more voxels than capacity]%s",
                     (flags & EMC2_DEVFLAG_MAP) ? " and [kernel-map entry outside the input rows]" : "");
  if (flags & EMC2_DEVFLAG_MAP)
    return emc2_fail(ctx, EMC2_ERR_MAP, "device reported [kernel-map entry outside the input rows]");
  return EMC2_OK;
}

extern "C" const char* emc2_last_error(const emc2_ctx* ctx) { return ctx ? ctx->err : emc2_static_last_error(); }
