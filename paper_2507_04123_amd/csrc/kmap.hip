// Kernel map (rulebook) for the 27 offsets of a 3x3x3 sparse conv (paper Sec. 3.5: only non-empty
// voxels are computed; Sec. 3.6: prefix-sum index search).
//
// SUBM   : for every active voxel o and tap k, look up cell(o) - 1 + k in the input cell index.
// STRIDED: every 32-cell word of the input cell index marks, with bit arithmetic, the outputs whose
//          3x3x3 window contains one of its voxels in the output cell index; the scan ranks them
//          (= ascending key order); the set bits are expanded to coordinates; then every output
//          probes the input index at 2*o - 1 + k.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "common.h"

namespace {

// Keep the even-numbered bits of v (bit 2i -> bit i).
__device__ __forceinline__ uint32_t compress_even_bits(uint64_t v) {
  v &= 0x5555555555555555ull;
  v = (v | (v >> 1)) & 0x3333333333333333ull;
  v = (v | (v >> 2)) & 0x0f0f0f0f0f0f0f0full;
  v = (v | (v >> 4)) & 0x00ff00ff00ff00ffull;
  v = (v | (v >> 8)) & 0x0000ffff0000ffffull;
  v = (v | (v >> 16)) & 0x00000000ffffffffull;
  return (uint32_t)v;
}

// Stride-2 output occupancy, one thread per 32-cell word of the INPUT cell index.  An input at x is read
// by outputs o with 2o-1 <= x <= 2o+1, so with the word's bits S laid out at their absolute x parity,
// output bit i is S[2i-1] | S[2i] | S[2i+1]: a shift-or and an even-bit compress give up to 18 output
// bits at once, which are OR-ed into at most two output words per (z, y) parity combination.  Working on
// words instead of voxels turns hundreds of colliding single-bit atomics per output word into a few.
__global__ void __launch_bounds__(256) k_strided_mark(const cellword_t* __restrict__ in_idx, int64_t n_in_words,
                                                      int64_t n_in_cells, cellword_t* __restrict__ out_idx, int gx, int gy,
                                                      int gz, int gox, int goy, int goz,
                                                      const lineflag_t* __restrict__ in_flags,
                                                      lineflag_t* __restrict__ out_flags) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= n_in_words) return;
  if (!in_flags[w >> EMC2_LINE_SHIFT]) return;   // no bit in this line of the input (uniform for 16 lanes)
  uint32_t bits = in_idx[w].x;
  while (bits) {
    // row segment of the word that starts at the first set bit's row
    const int first = __ffs((int)bits) - 1;
    uint64_t key = (uint64_t)w * 32 + (uint64_t)first;
    if ((int64_t)key >= n_in_cells) return;  // padding bits past the grid are never set; defensive
    const int4 c4 = decode_key(key, gx, gy, gz);
    const int x = c4.w, y = c4.z, z = c4.y;
    const uint64_t b = (uint64_t)c4.x;
    const int room = gx - x;                       // cells left in this row from the first set bit
    const int avail = 32 - first;                  // bits left in this word
    const int len = room < avail ? room : avail;   // segment [first, first + len)
    const uint32_t seg_mask = (len >= 32 ? 0xffffffffu : ((1u << len) - 1u)) << first;
    const uint32_t s = (bits & seg_mask) >> first; // bit j <-> input x + j
    bits &= ~seg_mask;
    const int p = x & 1;
    const uint64_t S = (uint64_t)s << (p + 1);     // bit j+1 <-> input x' = (x - p) + j; one spare bit below
    const uint64_t U = S | (S << 1) | (S >> 1);    // bit 2i+1 <-> S[2i-1+1] | S[2i+1] | S[2i+1+1]
    uint32_t m = compress_even_bits(U >> 1);       // bit i <-> output x = (x >> 1) + i
    const int ob = x >> 1;
    const int left = gox - ob;                     // outputs left in the output row
    if (left < 32) m &= (1u << left) - 1u;
    if (!m) continue;
    const int z0 = z >> 1, nz = ((z & 1) && (z0 + 1 < goz)) ? 2 : 1;
    const int y0 = y >> 1, ny = ((y & 1) && (y0 + 1 < goy)) ? 2 : 1;
    for (int dz = 0; dz < nz; ++dz)
      for (int dy = 0; dy < ny; ++dy) {
        const uint64_t okey = ((b * goz + (uint64_t)(z0 + dz)) * goy + (uint64_t)(y0 + dy)) * gox + (uint64_t)ob;
        const uint32_t sh = (uint32_t)okey & 31u;
        atomicOr(&out_idx[okey >> 5].x, m << sh);
        out_flags[emc2_line_of_key(okey)] = 1;
        if (sh != 0 && (m >> (32u - sh)) != 0) {
          atomicOr(&out_idx[(okey >> 5) + 1].x, m >> (32u - sh));
          out_flags[((okey >> 5) + 1) >> EMC2_LINE_SHIFT] = 1;
        }
      }
  }
}

// One thread per cellword: expand set bits into coordinates at their rank.  The word's first cell is decoded
// once; later bits advance x with carries (a word rarely crosses a row end), so no division per bit.
__global__ void __launch_bounds__(256) k_expand_coords(const cellword_t* __restrict__ idx, int64_t n_words, int64_t capacity,
                                                       int gx, int gy, int gz, const lineflag_t* __restrict__ flags,
                                                       int4* __restrict__ coords) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= n_words) return;
  if (!flags[w >> EMC2_LINE_SHIFT]) return;     // no bit in this line (uniform for 16 lanes)
  const cellword_t cw = idx[w];
  uint32_t bits = cw.x;
  if (!bits) return;
  int64_t r = cw.y;
  int4 c = decode_key((uint64_t)w * 32, gx, gy, gz);  // (b, z, y, x) of bit 0
  int at = 0;                                          // bit position c refers to
  while (bits) {
    const int j = __ffs((int)bits) - 1;
    bits &= bits - 1;
    c.w += j - at;
    at = j;
    while (c.w >= gx) {
      c.w -= gx;
      if (++c.z >= gy) {
        c.z = 0;
        if (++c.y >= gz) {
          c.y = 0;
          ++c.x;
        }
      }
    }
    if (r < capacity) coords[r] = c;
    ++r;
  }
}

// One thread per output voxel.  The three x-taps of a (z, y) row are adjacent bits of the input cell index,
// so a row costs one 8-byte load (two when the bits straddle a word): 9..18 loads per voxel instead of 27.
// S = stride (1 or 2).
template <int S>
__global__ void __launch_bounds__(256) k_probe(const int4* __restrict__ out_coords, const int32_t* __restrict__ d_n_out,
                                               int64_t capacity_out, const cellword_t* __restrict__ in_idx,
                                               const int32_t* __restrict__ d_n_in, int gx, int gy, int gz, int n_batch,
                                               int32_t* __restrict__ nbr) {
  int64_t n = *d_n_out;
  if (n > capacity_out) n = capacity_out;
  const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (o >= n) return;
  const int32_t n_in = *d_n_in;
  int4 c = out_coords[o];  // (b, z, y, x)
  // malformed coordinate: emit an empty column (the per-tap range checks below keep every lookup in bounds)
  const bool sane = (unsigned)c.x < (unsigned)n_batch && (unsigned)c.y <= (1u << 20) && (unsigned)c.z <= (1u << 20) &&
                    (unsigned)c.w <= (1u << 20);
  if (!sane) c = make_int4(0, 0, 0, 0);
  const int bx = c.w * S - 1, by = c.z * S - 1, bz = c.y * S - 1;
  const int lo = bx < 0 ? 0 : bx;                    // x range of this voxel's taps inside the grid
  const int hi = bx + 2 >= gx ? gx - 1 : bx + 2;
#pragma unroll
  for (int kz = 0; kz < 3; ++kz) {
    const int iz = bz + kz;
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
      const int iy = by + ky;
      const bool row_ok = sane && (iz >= 0) && (iz < gz) && (iy >= 0) && (iy < gy) && (lo <= hi);
      const uint64_t row = (((uint64_t)c.x * gz + (uint64_t)(row_ok ? iz : 0)) * gy + (uint64_t)(row_ok ? iy : 0)) * gx;
      const uint64_t w_lo = (row + (uint64_t)lo) >> 5, w_hi = (row + (uint64_t)hi) >> 5;
      cellword_t cw0 = make_uint2(0u, 0u), cw1 = make_uint2(0u, 0u);
      if (row_ok) {
        cw0 = in_idx[w_lo];
        cw1 = (w_hi != w_lo) ? in_idx[w_hi] : cw0;
      }
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) {
        const int ix = bx + kx;
        int32_t j = -1;
        if (row_ok && ix >= lo && ix <= hi) {
          const uint64_t key = row + (uint64_t)ix;
          const cellword_t cw = ((key >> 5) == w_lo) ? cw0 : cw1;
          const uint32_t bit = (uint32_t)key & 31u;
          if ((cw.x >> bit) & 1u) j = (int32_t)(cw.y + __popc(cw.x & ((1u << bit) - 1u)));
        }
        if (j >= n_in) j = -1;  // only after a capacity overflow upstream
        // written once, read by a later kernel: a streaming store keeps the map from displacing the index in the caches
        __builtin_nontemporal_store(j, &nbr[(int64_t)((kz * 3 + ky) * 3 + kx) * capacity_out + o]);
      }
    }
  }
}

__global__ void k_copy_count(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int64_t capacity,
                             int32_t* __restrict__ d_flags) {
  int32_t n = *src;
  if (n > capacity) {
    atomicOr(d_flags, EMC2_DEVFLAG_CAPACITY);
    n = (int32_t)capacity;
  }
  *dst = n;
}

__global__ void __launch_bounds__(256) k_copy_coords(const int4* __restrict__ src, int4* __restrict__ dst,
                                                     const int32_t* __restrict__ d_n, int64_t capacity) {
  int64_t n = *d_n;
  if (n > capacity) n = capacity;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

// The whole call, on whatever context it is given: one made by emc2_create, or the per-device one whose scratch
// is the static array further down.
emc2_status build_kmap_on(emc2_ctx* ctx, emc2_conv_kind kind, const int32_t* d_in_coords, const int32_t* d_n_in,
                          int64_t capacity_in, const int32_t grid_in[3], int32_t n_batch, int32_t in_slot, int32_t out_slot,
                          int64_t capacity_out, int32_t* d_out_coords, int32_t* d_n_out, int32_t* d_nbr, int32_t grid_out[3],
                          int32_t* h_n_out, void* stream) {
  if (kind != EMC2_CONV_SUBM && kind != EMC2_CONV_STRIDED)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_kmap: bad kind");
  if (!d_in_coords || !d_n_in || !grid_in || !d_n_out || !d_nbr || !grid_out)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_kmap: null argument");
  if (capacity_in < 1 || capacity_in > ctx->max_voxels || capacity_out < 1 || capacity_out > ctx->max_voxels)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_kmap: capacity outside [1, max_voxels]");
  if (kind == EMC2_CONV_STRIDED && !d_out_coords)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_kmap: STRIDED needs d_out_coords");
  int64_t cells_in = 0, cells_out = 0;
  if (!emc2_grid_ok(grid_in, n_batch, &cells_in))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_build_kmap: grid/batch out of the supported key range");
  int32_t go[3];
  for (int a = 0; a < 3; ++a) go[a] = kind == EMC2_CONV_SUBM ? grid_in[a] : (grid_in[a] - 1) / 2 + 1;
  (void)emc2_grid_ok(go, n_batch, &cells_out);
  if (cells_in > ctx->max_cells)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_kmap: %lld cells > max_cells %lld", (long long)cells_in,
                     (long long)ctx->max_cells);
  if (in_slot < -1 || in_slot >= ctx->n_slots || out_slot < -1 || out_slot >= ctx->n_slots)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_kmap: slot outside [-1, %d)", ctx->n_slots);
  if (kind == EMC2_CONV_STRIDED && out_slot >= 0 && out_slot == in_slot)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_kmap: out_slot must differ from in_slot");
  if (in_slot >= 0) {
    const SlotMeta& m = ctx->meta[in_slot];
    if (!m.valid || m.n_batch != n_batch || m.grid[0] != grid_in[0] || m.grid[1] != grid_in[1] || m.grid[2] != grid_in[2])
      return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_build_kmap: in_slot %d does not hold an index for this grid", in_slot);
  }
  for (int a = 0; a < 3; ++a) grid_out[a] = go[a];

  hipStream_t s = (hipStream_t)stream;
  const int tmp_in = ctx->n_slots, tmp_out = ctx->n_slots + 1;
  cellword_t* in_idx;
  if (in_slot >= 0) {
    in_idx = ctx->slots[in_slot];
  } else {
    // rebuild the input index from the (ascending, distinct) coordinates; ranks then equal positions
    in_idx = ctx->slots[tmp_in];
    emc2_index_clear(ctx, in_idx, s);
    emc2_index_mark_coords(ctx, in_idx, d_in_coords, d_n_in, capacity_in, grid_in, n_batch, s);
    emc2_index_scan(ctx, in_idx, cells_in, capacity_in, ctx->dev_words + 2, s);
  }

  const int32_t* out_coords = d_in_coords;
  if (kind == EMC2_CONV_SUBM) {
    // the count only needs a kernel when it moves or can be clamped
    if (d_n_out != d_n_in || capacity_out < capacity_in)
      hipLaunchKernelGGL(k_copy_count, dim3(1), dim3(1), 0, s, d_n_in, d_n_out, capacity_out, ctx->dev_words);
    if (d_out_coords && d_out_coords != d_in_coords) {
      const int64_t m = capacity_in < capacity_out ? capacity_in : capacity_out;
      hipLaunchKernelGGL(k_copy_coords, dim3((unsigned)emc2_div_up(m, 256)), dim3(256), 0, s, (const int4*)d_in_coords,
                         (int4*)d_out_coords, d_n_out, m);
    }
    const int64_t m = capacity_in < capacity_out ? capacity_in : capacity_out;
    hipLaunchKernelGGL(k_probe<1>, dim3((unsigned)emc2_div_up(m, 256)), dim3(256), 0, s, (const int4*)d_in_coords, d_n_out,
                       capacity_out, in_idx, d_n_out, grid_in[0], grid_in[1], grid_in[2], n_batch, d_nbr);
  } else {
    cellword_t* out_idx = ctx->slots[out_slot >= 0 ? out_slot : tmp_out];
    if (out_slot >= 0) {
      SlotMeta& m = ctx->meta[out_slot];
      for (int a = 0; a < 3; ++a) m.grid[a] = go[a];
      m.n_batch = n_batch;
      m.valid = true;
    }
    emc2_index_clear(ctx, out_idx, s);
    {
      const int64_t n_in_words = emc2_div_up(cells_in, 32);
      hipLaunchKernelGGL(k_strided_mark, dim3((unsigned)emc2_div_up(n_in_words, 256)), dim3(256), 0, s, in_idx, n_in_words,
                         cells_in, out_idx, grid_in[0], grid_in[1], grid_in[2], go[0], go[1], go[2],
                         emc2_slot_flags(ctx, in_idx), emc2_slot_flags(ctx, out_idx));
    }
    emc2_index_scan(ctx, out_idx, cells_out, capacity_out, d_n_out, s);
    const int64_t n_words = emc2_div_up(cells_out, 32);
    hipLaunchKernelGGL(k_expand_coords, dim3((unsigned)emc2_div_up(n_words, 256)), dim3(256), 0, s, out_idx, n_words,
                       capacity_out, go[0], go[1], go[2], emc2_slot_flags(ctx, out_idx), (int4*)d_out_coords);
    out_coords = d_out_coords;
    hipLaunchKernelGGL(k_probe<2>, dim3((unsigned)emc2_div_up(capacity_out, 256)), dim3(256), 0, s, (const int4*)out_coords,
                       d_n_out, capacity_out, in_idx, d_n_in, grid_in[0], grid_in[1], grid_in[2], n_batch, d_nbr);
  }
  emc2_status st = emc2_check_hip(ctx, hipGetLastError(), "emc2_build_kmap launch");
  if (st != EMC2_OK) return st;
  if (h_n_out) {
    st = emc2_check_hip(ctx, hipMemcpyAsync(ctx->pinned + 2, d_n_out, sizeof(int32_t), hipMemcpyDeviceToHost, s),
                        "hipMemcpyAsync(n_out)");
    if (st != EMC2_OK) return st;
    st = emc2_check_hip(ctx, hipStreamSynchronize(s), "hipStreamSynchronize");
    if (st != EMC2_OK) return st;
    *h_n_out = ctx->pinned[2];
  }
  return EMC2_OK;
}

}  // namespace

extern "C" emc2_status emc2_build_kmap(emc2_ctx* ctx, emc2_conv_kind kind, const int32_t* d_in_coords,
                                       const int32_t* d_n_in, int64_t capacity_in, const int32_t grid_in[3],
                                       int32_t n_batch, int32_t in_slot, int32_t out_slot, int64_t capacity_out,
                                       int32_t* d_out_coords, int32_t* d_n_out, int32_t* d_nbr, int32_t grid_out[3],
                                       int32_t* h_n_out, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  return build_kmap_on(ctx, kind, d_in_coords, d_n_in, capacity_in, grid_in, n_batch, in_slot, out_slot, capacity_out,
                       d_out_coords, d_n_out, d_nbr, grid_out, h_n_out, stream);
}

// ---------------------------------------------------------------------------------------------------------
// emc2_build_kmap_static: the same call for callers that must not allocate.  Everything emc2_build_kmap keeps in
// a context's scratch (two cell-index slots with their line flags, the scan's partial sums, the status and
// count words) lives in one file-scope device array instead; each GPU holds its own copy at its own address,
// looked up once per device, and a host-side context structure per device points into it.
// ---------------------------------------------------------------------------------------------------------
namespace {

constexpr int64_t kStaticMaxCells = EMC2_STATIC_KMAP_MAX_CELLS;
constexpr int64_t kStaticTiles = (kStaticMaxCells / 32 + 1 + EMC2_SCAN_TILE - 1) / EMC2_SCAN_TILE;   // as emc2_create sizes a slot
constexpr int64_t kStaticWords = kStaticTiles * EMC2_SCAN_TILE;
constexpr size_t kStaticSlotBytes = sizeof(cellword_t) * (size_t)kStaticWords + sizeof(lineflag_t) * (size_t)(kStaticWords >> EMC2_LINE_SHIFT);
constexpr size_t kStaticSlotPitch = (kStaticSlotBytes + 255) / 256 * 256;
constexpr size_t kStaticPartialsBytes = ((size_t)(kStaticTiles + 1) * sizeof(uint32_t) + 255) / 256 * 256;
constexpr size_t kStaticBytes = 2 * kStaticSlotPitch + kStaticPartialsBytes + 256;   // + status / count words

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kStaticMaxDevices = 64;
struct StaticKmap {
  bool ready;
  unsigned char* ptr;        // this device's address of `scratch`
  emc2_ctx ctx;              // host-side view of the scratch: no device memory of its own
  cellword_t* slots[2];
  SlotMeta meta[2];
};
StaticKmap g_static[kStaticMaxDevices];
std::mutex g_static_mutex;
char g_static_err[256] = "";

emc2_status static_fail(emc2_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_static_err, sizeof(g_static_err), fmt, ap);
  va_end(ap);
  return st;
}

__global__ void __launch_bounds__(256) k_static_zero(uint4* __restrict__ p, int64_t n16) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n16) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

// hand the accumulated status bits to the caller's word and clear them for the next call
__global__ void k_static_status(int32_t* __restrict__ dev_words, int32_t* __restrict__ d_status) {
  *d_status = dev_words[0];
  dev_words[0] = 0;
}

}  // namespace

const char* emc2_static_last_error() { return g_static_err; }

extern "C" emc2_status emc2_build_kmap_static(emc2_conv_kind kind, const int32_t* d_in_coords, const int32_t* d_n_in,
                                              int64_t capacity_in, const int32_t grid_in[3], int32_t n_batch,
                                              int64_t capacity_out, int32_t* d_out_coords, int32_t* d_n_out,
                                              int32_t* d_nbr, int32_t grid_out[3], int32_t* d_status, void* stream) {
  std::lock_guard<std::mutex> lock(g_static_mutex);   // host-side state only; device work is ordered by `stream`
  int device = -1;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return static_fail(EMC2_ERR_DEVICE, "emc2_build_kmap_static: hipGetDevice: %s", hipGetErrorString(e));
  if (device < 0 || device >= kStaticMaxDevices)
    return static_fail(EMC2_ERR_UNSUPPORTED, "emc2_build_kmap_static: device %d outside [0, %d)", device, kStaticMaxDevices);
  int64_t cells = 0;
  if (!grid_in || !emc2_grid_ok(grid_in, n_batch, &cells))
    return static_fail(EMC2_ERR_INVALID_ARG, "emc2_build_kmap_static: bad grid / batch");
  if (cells > kStaticMaxCells)
    return static_fail(EMC2_ERR_INVALID_ARG,
                       "emc2_build_kmap_static: %lld cells exceed the static scratch's %lld (EMC2_STATIC_KMAP_MAX_CELLS); "
                       "use emc2_build_kmap with a context",
                       (long long)cells, (long long)kStaticMaxCells);
  hipStream_t s = (hipStream_t)stream;
  StaticKmap& sk = g_static[device];
  if (!sk.ready) {
    // this device's copy of the array: the symbol's name is not an address host code may pass to a kernel
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p)
      return static_fail(EMC2_ERR_DEVICE, "emc2_build_kmap_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
    sk.ptr = (unsigned char*)p;
    memset(&sk.ctx, 0, sizeof(sk.ctx));
    sk.ctx.device = device;
    sk.ctx.max_points = 0;
    sk.ctx.max_voxels = 1ll << 30;         // a kernel map needs no per-voxel scratch
    sk.ctx.max_cells = kStaticMaxCells;
    sk.ctx.n_slots = 0;                    // no caller-visible slots: both are the call's internal ones
    sk.ctx.slot_tiles = kStaticTiles;
    sk.ctx.slot_words = kStaticWords;
    sk.slots[0] = (cellword_t*)sk.ptr;
    sk.slots[1] = (cellword_t*)(sk.ptr + kStaticSlotPitch);
    sk.ctx.slots = sk.slots;
    sk.ctx.meta = sk.meta;
    sk.ctx.partials = (uint32_t*)(sk.ptr + 2 * kStaticSlotPitch);
    sk.ctx.n_partials = kStaticTiles + 1;
    sk.ctx.dev_words = (int32_t*)(sk.ptr + 2 * kStaticSlotPitch + kStaticPartialsBytes);
    // the line-flag invariant (a line without its flag holds no bit) and the status word start from zero; a fill
    // kernel rather than a memset, so that a first call under stream capture records nothing unusual
    const int64_t n16 = (int64_t)(kStaticBytes / 16);
    hipLaunchKernelGGL(k_static_zero, dim3((unsigned)emc2_div_up(n16, 256)), dim3(256), 0, s, (uint4*)sk.ptr, n16);
    e = hipGetLastError();
    if (e != hipSuccess) return static_fail(EMC2_ERR_DEVICE, "emc2_build_kmap_static: zero fill: %s", hipGetErrorString(e));
    sk.ready = true;
  }
  const emc2_status st = build_kmap_on(&sk.ctx, kind, d_in_coords, d_n_in, capacity_in, grid_in, n_batch, -1, -1, capacity_out,
                                       d_out_coords, d_n_out, d_nbr, grid_out, nullptr, stream);
  if (st != EMC2_OK) {
    snprintf(g_static_err, sizeof(g_static_err), "%s", sk.ctx.err);
    return st;
  }
  if (d_status) {
    hipLaunchKernelGGL(k_static_status, dim3(1), dim3(1), 0, s, sk.ctx.dev_words, d_status);
    e = hipGetLastError();
    if (e != hipSuccess) return static_fail(EMC2_ERR_DEVICE, "emc2_build_kmap_static: status copy: %s", hipGetErrorString(e));
  }
  return EMC2_OK;
}
