// Internal declarations shared by the translation units of libemc2.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "emc2.h"

// ---------------------------------------------------------------------------------------------
// Cell index: one 8-byte word per 32 consecutive cells of the linear key space
//   .x = occupancy bits (bit j <=> cell 32*w + j is an active voxel)
//   .y = number of active cells in all earlier words (exclusive prefix sum of popcounts)
// Because voxels are listed in ascending key order, the voxel index of an active cell is simply
// its rank: word.y + popcount(word.x & lower-bit mask).  This is the prefix-sum index search of
// the paper's Sec. 3.6, giving an O(1) lookup.
// ---------------------------------------------------------------------------------------------
typedef uint2 cellword_t;

__device__ __forceinline__ int32_t cell_lookup(const cellword_t* __restrict__ idx, uint64_t key) {
  const cellword_t w = idx[key >> 5];
  const uint32_t bit = (uint32_t)key & 31u;
  if (!((w.x >> bit) & 1u)) return -1;
  return (int32_t)(w.y + __popc(w.x & ((1u << bit) - 1u)));
}

// Linear key -> (b, z, y, x).  Keys below 2^32 (every single-frame grid here) take 32-bit divisions, which are
// several times cheaper than the 64-bit ones.
__device__ __forceinline__ int4 decode_key(uint64_t key, int gx, int gy, int gz) {
  if ((key >> 32) == 0) {
    uint32_t k = (uint32_t)key;
    const uint32_t x = k % (uint32_t)gx; k /= (uint32_t)gx;
    const uint32_t y = k % (uint32_t)gy; k /= (uint32_t)gy;
    const uint32_t z = k % (uint32_t)gz; k /= (uint32_t)gz;
    return make_int4((int)k, (int)z, (int)y, (int)x);
  }
  uint64_t k = key;
  const int x = (int)(k % (uint64_t)gx); k /= (uint64_t)gx;
  const int y = (int)(k % (uint64_t)gy); k /= (uint64_t)gy;
  const int z = (int)(k % (uint64_t)gz); k /= (uint64_t)gz;
  return make_int4((int)k, z, y, x);
}

// points a voxel's stash holds before further ones are added atomically (LiDAR voxels hold 1-2 points)
#define EMC2_VOX_STASH 4


// Device status bits (OR-ed by kernels, read by emc2_status_sync).
#define EMC2_DEVFLAG_CAPACITY 1
#define EMC2_DEVFLAG_MAP 2        // a kernel-map entry named a row outside [0, n_in_rows)

// A kernel-map entry as a conv kernel uses it.  Rows past n_out (`dead` = -1, else 0) have no neighbours; an
// entry at or beyond the `n_in` rows the caller says the input holds is treated as absent (never read) and
// remembered in the wave-uniform mask `oob`, which emc2_report_oob turns into a status bit at the kernel's end.
__device__ __forceinline__ int32_t emc2_entry(int32_t j, int32_t dead, int32_t n_in, unsigned long long& oob) {
  j |= dead;
  oob |= __ballot(j >= n_in);
  return j < n_in ? j : -1;
}
__device__ __forceinline__ void emc2_report_oob(unsigned long long oob, int32_t* __restrict__ flags) {
  if (oob != 0ull && (threadIdx.x & 63) == 0) atomicOr(flags, EMC2_DEVFLAG_MAP);
}

struct SlotMeta {
  int32_t grid[3];
  int32_t n_batch;
  bool valid;
};

struct emc2_ctx {
  int device;
  int64_t max_points, max_voxels, max_cells;
  int32_t n_slots;          // user-visible slots; two more internal ones follow
  int64_t slot_words;       // cellwords per slot (a whole number of tiles); the line flags follow them
  int64_t slot_tiles;
  cellword_t** slots;       // host array [n_slots + 2] of device pointers
  SlotMeta* meta;           // host array [n_slots + 2]
  float4* stash;            // [max_voxels][EMC2_VOX_STASH] points of each voxel, in arrival order
  uint32_t* partials;       // scan partial sums
  int64_t n_partials;
  int32_t* dev_words;       // [0] status flags, [2] voxel count of an index rebuilt from coordinates (others unused)
  void* wpack;              // scratch for weights re-ordered per call (27*128*128 16-bit values)
  void* zero_row;           // 256 zero bytes: the feature row an absent neighbour reads
  // image pooling: per-pixel cell rank / position within the cell / sorted order, per-cell list starts
  int32_t *pix_rank, *pix_pos, *pix_perm, *pix_srank;   // [max_points] each
  int32_t* cell_start;      // [max_voxels + 1]
  uint32_t* pool_totals;    // block totals of the scan over the per-cell counts
  int64_t n_pool_totals;
  uint32_t* pool_acc;       // [(max_points/64 + 2) * 256] partial results of cells that cross a block boundary
  int32_t* fuse_src;        // [2 * max_voxels] source rows of a fused set when the caller does not keep them
  int32_t* pinned;          // pinned host staging for counts / status (4 ints)
  char err[256];
};

#define EMC2_SCAN_TILE 2048  // cellwords per scan block (256 threads x 8)
#define EMC2_TILE_SHIFT 11   // log2(EMC2_SCAN_TILE)
#define EMC2_LINE_SHIFT 4    // log2 of the cellwords per flagged line: 16 words = 128 bytes = 512 cells
#define EMC2_LINES_PER_TILE (EMC2_SCAN_TILE >> EMC2_LINE_SHIFT)

// Line flags of an index slot.  The active cells of a LiDAR frame fill a fraction of a percent of the finest
// grid, and scattered objects touch single cache lines of it, so every index slot carries one flag byte per
// 128-byte line (16 words, 512 cells), stored behind its words:
// INVARIANT: a line whose flag is 0 holds no occupancy bit (its prefix fields are unspecified and never
// read: a lookup tests the bit first).  Every kernel that sets bits raises the flag of the line it writes
// (a plain byte store: all writers store the same value); clear, scan, the stride-2 marking and the
// expansion to coordinates read a tile's 128 flag bytes first and touch only the flagged lines.
typedef uint8_t lineflag_t;
static inline lineflag_t* emc2_slot_flags(const emc2_ctx* ctx, cellword_t* idx) {
  return reinterpret_cast<lineflag_t*>(idx + ctx->slot_words);
}
// flag index of the line that holds cell `key`
__host__ __device__ __forceinline__ uint64_t emc2_line_of_key(uint64_t key) { return key >> (5 + EMC2_LINE_SHIFT); }

// host helpers (context.hip)
emc2_status emc2_fail(emc2_ctx* ctx, emc2_status st, const char* fmt, ...);
emc2_status emc2_check_hip(emc2_ctx* ctx, hipError_t e, const char* what);
bool emc2_grid_ok(const int32_t grid[3], int32_t n_batch, int64_t* n_cells);

// cell-index construction (cellindex.hip); all asynchronous on `stream`
// zero every flagged tile of the slot (whatever grid it last held) and lower its flag
void emc2_index_clear(emc2_ctx* ctx, cellword_t* idx, hipStream_t stream);
// exclusive scan of popcounts over ceil(n_cells/32) words; writes min(total, capacity) to d_total
// and raises EMC2_DEVFLAG_CAPACITY when total > capacity
void emc2_index_scan(emc2_ctx* ctx, cellword_t* idx, int64_t n_cells, int64_t capacity, int32_t* d_total,
                     hipStream_t stream);
// set the bits of coords[0..*d_n) (b,z,y,x) in a cleared index
void emc2_index_mark_coords(emc2_ctx* ctx, cellword_t* idx, const int32_t* d_coords, const int32_t* d_n,
                            int64_t capacity, const int32_t grid[3], int32_t n_batch, hipStream_t stream);

// text of the last host-side error of emc2_build_kmap_static (kmap.hip); what emc2_last_error(NULL) returns
const char* emc2_static_last_error();

static inline int64_t emc2_div_up(int64_t a, int64_t b) { return (a + b - 1) / b; }
