/*
 * CPU oracle for the EMC2 LiDAR hot path.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the
 * bench's cpu_baseline leg may call this; the product path never does.  It shares no code, header,
 * table or helper with the HIP library.
 *
 * Plain, slow, obviously-correct definitions:
 *   - voxelization (paper Sec. 2 "process point clouds via voxelization", Sec. 3.1 data bridge,
 *     Sec. 3.5 configurable pool size): sort points by linear cell key, one run per voxel, mean of
 *     the run in fp64;
 *   - kernel map for the 27 offsets of a 3x3x3 sparse conv (Sec. 3.5 "computing nonzero voxels
 *     only"; Sec. 3.6 index search): sorted key list + binary search;
 *   - sparse conv (Sec. 3.5, O(N x C_v)): per offset, nested loops, fp64 accumulation, then the
 *     folded-BN affine + ReLU epilogue (Sec. 3.6 graph fusion) in fp64, rounded once to fp32;
 *   - point -> image projection with bilinear gather and zero fill for unmatched points
 *     (Sec. 3.1 / Fig. 5 caption), fp64;
 *   - inverse (transposed) kernel map for the decoder half of the LiDAR UNet (Sec. 3.1: "a UNet and a
 *     sparse CNN"): the pairs of a stride-2 map with the roles of input and output swapped;
 *   - bird's-eye-view flattening of a voxel set (Sec. 3.3, latency-prioritised expert works on BEV
 *     projections): scatter into a dense, zero-filled, z-collapsed tensor;
 *   - Multiscale Pooling (Sec. 3.1, Sec. 3.5, Fig. 5): image pixels with depth are lifted into 3D,
 *     grouped by the cell of a grid of configurable cell size, and their features pooled per cell
 *     (mean or max);
 *   - multimodal fusion (Sec. 3.1, Fig. 5 caption): the union of LiDAR voxels and pooled image cells,
 *     features concatenated, the missing half zero-filled;
 *   - Scenario-Adaptive Dispatcher (Sec. 3.2): one of three experts per scene from the distances and
 *     confidences of its proposal regions, the scenes grouped by expert, and the batch ids of the points for
 *     the group of one expert;
 *   - quantised sparse convolution (Sec. 3.6 (2) names model quantisation without giving a scheme; the
 *     scheme here is this build's own): int8 features and weights, exact integer accumulation, a
 *     per-channel fp32 multiply-add, optional ReLU, optional re-quantisation to int8; and the same with 8-bit
 *     floating-point (E4M3) features and weights, whose products and sums are exact in fp64.
 *
 * Compile: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no fast-math: the cell index is
 * defined by IEEE fp32 subtract, divide, floor).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define EMC2O_ERR_ARG (-1)
#define EMC2O_ERR_CAPACITY (-2)
#define EMC2O_ERR_NOMEM (-3)

static int g_threads = 1;

void emc2o_set_threads(int n) { g_threads = n < 1 ? 1 : n; }

int emc2o_get_threads(void) { return g_threads; }

int emc2o_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------------------------------- */
/* voxelization                                                                                */
/* ------------------------------------------------------------------------------------------- */

typedef struct {
  uint64_t key;
  int64_t idx;
} keyed_t;

static int cmp_keyed(const void* a, const void* b) {
  const keyed_t* p = (const keyed_t*)a;
  const keyed_t* q = (const keyed_t*)b;
  if (p->key != q->key) return p->key < q->key ? -1 : 1;
  if (p->idx != q->idx) return p->idx < q->idx ? -1 : 1;
  return 0;
}

/* Cell index along one axis: fp32 subtract, fp32 true division, floor.  Returns -1 if outside. */
static int cell_of(float p, float lo, float vs, int g) {
  volatile float d = p - lo; /* volatile: keep each op a separately rounded fp32 op */
  volatile float t = d / vs;
  float tt = t;
  if (!(tt >= 0.0f) || !(tt < (float)g)) return -1; /* also rejects NaN and +-inf */
  return (int)floorf(tt);
}

/*
 * points: [n][stride_f] fp32, columns 0..3 = x, y, z, intensity.  batch: [n] or NULL (=> 0).
 * Outputs in ascending key order, key = ((b*Gz + z)*Gy + y)*Gx + x:
 *   coords[v] = (b, z, y, x), feats[v] = mean (x, y, z, intensity) over all points of the voxel
 *   (fp64 sum, one rounding to fp32), counts[v] = number of points.
 * Returns the number of voxels, or a negative error.
 */
int64_t emc2o_voxelize(const float* points, const int32_t* batch, int64_t n, int32_t stride_f,
                       const float lo[3], const float vs[3], const int32_t grid[3], int32_t n_batch,
                       float r2_min, float r2_max, int64_t capacity, int32_t* coords, float* feats,
                       int32_t* counts) {
  if (n < 0 || stride_f < 4 || n_batch < 1 || grid[0] < 1 || grid[1] < 1 || grid[2] < 1)
    return EMC2O_ERR_ARG;
  keyed_t* ks = (keyed_t*)malloc(sizeof(keyed_t) * (size_t)(n > 0 ? n : 1));
  if (!ks) return EMC2O_ERR_NOMEM;
  int64_t m = 0;
  const uint64_t gx = (uint64_t)grid[0], gy = (uint64_t)grid[1], gz = (uint64_t)grid[2];
  for (int64_t i = 0; i < n; ++i) {
    const float* p = points + i * stride_f;
    int b = batch ? batch[i] : 0;
    if (b < 0 || b >= n_batch) continue;
    if (!isfinite(p[3])) continue;
    int cx = cell_of(p[0], lo[0], vs[0], grid[0]);
    int cy = cell_of(p[1], lo[1], vs[1], grid[1]);
    int cz = cell_of(p[2], lo[2], vs[2], grid[2]);
    if (cx < 0 || cy < 0 || cz < 0) continue;
    volatile float xx = p[0] * p[0];
    volatile float yy = p[1] * p[1];
    volatile float r2 = xx + yy;
    float rr = r2;
    if (!(rr >= r2_min) || !(rr < r2_max)) continue;
    ks[m].key = (((uint64_t)b * gz + (uint64_t)cz) * gy + (uint64_t)cy) * gx + (uint64_t)cx;
    ks[m].idx = i;
    ++m;
  }
  qsort(ks, (size_t)m, sizeof(keyed_t), cmp_keyed);
  int64_t v = 0;
  int64_t i = 0;
  while (i < m) {
    int64_t j = i;
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    while (j < m && ks[j].key == ks[i].key) {
      const float* p = points + ks[j].idx * stride_f;
      for (int c = 0; c < 4; ++c) s[c] += (double)p[c];
      ++j;
    }
    if (v >= capacity) {
      free(ks);
      return EMC2O_ERR_CAPACITY;
    }
    uint64_t k = ks[i].key;
    coords[4 * v + 3] = (int32_t)(k % gx);
    k /= gx;
    coords[4 * v + 2] = (int32_t)(k % gy);
    k /= gy;
    coords[4 * v + 1] = (int32_t)(k % gz);
    k /= gz;
    coords[4 * v + 0] = (int32_t)k;
    double cnt = (double)(j - i);
    for (int c = 0; c < 4; ++c) feats[4 * v + c] = (float)(s[c] / cnt);
    counts[v] = (int32_t)(j - i);
    ++v;
    i = j;
  }
  free(ks);
  return v;
}

/* ------------------------------------------------------------------------------------------- */
/* kernel maps                                                                                 */
/* ------------------------------------------------------------------------------------------- */

static int cmp_u64(const void* a, const void* b) {
  uint64_t p = *(const uint64_t*)a, q = *(const uint64_t*)b;
  return p < q ? -1 : (p > q ? 1 : 0);
}

static uint64_t key_of(int64_t b, int64_t z, int64_t y, int64_t x, const int32_t g[3]) {
  return (((uint64_t)b * (uint64_t)g[2] + (uint64_t)z) * (uint64_t)g[1] + (uint64_t)y) *
             (uint64_t)g[0] + (uint64_t)x;
}

/* Index of `key` in the ascending array keys[n], or -1. */
static int64_t find_key(const uint64_t* keys, int64_t n, uint64_t key) {
  int64_t lo = 0, hi = n;
  while (lo < hi) {
    int64_t mid = lo + (hi - lo) / 2;
    if (keys[mid] < key) lo = mid + 1; else hi = mid;
  }
  return (lo < n && keys[lo] == key) ? lo : -1;
}

/*
 * kind 0 = submanifold (s=1, p=1): output sites = input sites, same order.
 * kind 1 = strided   (s=2, p=1): output o active iff some tap reads an active input; outputs in
 *          ascending key order on grid_out = (G-1)/2+1.
 * Tap k = (kz*3 + ky)*3 + kx reads input i = o*s - 1 + (kx, ky, kz) (cross-correlation).
 * nbr[k*capacity_out + o] = index of that input among in_coords, or -1.
 * in_coords must be ascending in key (what emc2o_voxelize / this function produce).
 * Returns n_out or a negative error.
 */
int64_t emc2o_build_kmap(int32_t kind, const int32_t* in_coords, int64_t n_in, const int32_t grid_in[3],
                         int32_t n_batch, int64_t capacity_out, int32_t* out_coords, int32_t* nbr,
                         int32_t grid_out[3]) {
  if (kind != 0 && kind != 1) return EMC2O_ERR_ARG;
  if (n_in < 0 || n_batch < 1) return EMC2O_ERR_ARG;
  const int s = kind == 0 ? 1 : 2;
  for (int a = 0; a < 3; ++a) grid_out[a] = kind == 0 ? grid_in[a] : (grid_in[a] - 1) / 2 + 1;

  uint64_t* in_keys = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(n_in > 0 ? n_in : 1));
  if (!in_keys) return EMC2O_ERR_NOMEM;
  for (int64_t i = 0; i < n_in; ++i) {
    const int32_t* c = in_coords + 4 * i;
    if (c[0] < 0 || c[0] >= n_batch || c[1] < 0 || c[1] >= grid_in[2] || c[2] < 0 ||
        c[2] >= grid_in[1] || c[3] < 0 || c[3] >= grid_in[0]) {
      free(in_keys);
      return EMC2O_ERR_ARG;
    }
    in_keys[i] = key_of(c[0], c[1], c[2], c[3], grid_in);
    if (i > 0 && in_keys[i] <= in_keys[i - 1]) { /* must be strictly ascending */
      free(in_keys);
      return EMC2O_ERR_ARG;
    }
  }

  int64_t n_out = 0;
  const int32_t* oc = NULL;
  int32_t* tmp_out = NULL;
  if (kind == 0) {
    n_out = n_in;
    if (n_out > capacity_out) { free(in_keys); return EMC2O_ERR_CAPACITY; }
    if (out_coords && out_coords != in_coords) memcpy(out_coords, in_coords, sizeof(int32_t) * 4 * (size_t)n_in);
    oc = in_coords;
  } else {
    /* every (input, tap) whose o = (i + 1 - k)/2 is integral and inside grid_out is a candidate */
    uint64_t* cand = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(n_in > 0 ? 27 * n_in : 1));
    if (!cand) { free(in_keys); return EMC2O_ERR_NOMEM; }
    int64_t nc = 0;
    for (int64_t i = 0; i < n_in; ++i) {
      const int32_t* c = in_coords + 4 * i;
      for (int kz = 0; kz < 3; ++kz)
        for (int ky = 0; ky < 3; ++ky)
          for (int kx = 0; kx < 3; ++kx) {
            int tx = c[3] + 1 - kx, ty = c[2] + 1 - ky, tz = c[1] + 1 - kz;
            if (tx < 0 || ty < 0 || tz < 0) continue;
            if ((tx & 1) || (ty & 1) || (tz & 1)) continue;
            int ox = tx / 2, oy = ty / 2, oz = tz / 2;
            if (ox >= grid_out[0] || oy >= grid_out[1] || oz >= grid_out[2]) continue;
            cand[nc++] = key_of(c[0], oz, oy, ox, grid_out);
          }
    }
    qsort(cand, (size_t)nc, sizeof(uint64_t), cmp_u64);
    int64_t u = 0;
    for (int64_t i = 0; i < nc; ++i)
      if (i == 0 || cand[i] != cand[i - 1]) cand[u++] = cand[i];
    n_out = u;
    if (n_out > capacity_out) { free(cand); free(in_keys); return EMC2O_ERR_CAPACITY; }
    tmp_out = out_coords;
    const uint64_t gx = (uint64_t)grid_out[0], gy = (uint64_t)grid_out[1], gz = (uint64_t)grid_out[2];
    for (int64_t o = 0; o < n_out; ++o) {
      uint64_t k = cand[o];
      tmp_out[4 * o + 3] = (int32_t)(k % gx); k /= gx;
      tmp_out[4 * o + 2] = (int32_t)(k % gy); k /= gy;
      tmp_out[4 * o + 1] = (int32_t)(k % gz); k /= gz;
      tmp_out[4 * o + 0] = (int32_t)k;
    }
    free(cand);
    oc = tmp_out;
  }

  for (int kz = 0; kz < 3; ++kz)
    for (int ky = 0; ky < 3; ++ky)
      for (int kx = 0; kx < 3; ++kx) {
        const int k = (kz * 3 + ky) * 3 + kx;
        for (int64_t o = 0; o < n_out; ++o) {
          const int32_t* c = oc + 4 * o;
          int64_t ix = (int64_t)c[3] * s - 1 + kx;
          int64_t iy = (int64_t)c[2] * s - 1 + ky;
          int64_t iz = (int64_t)c[1] * s - 1 + kz;
          int64_t j = -1;
          if (ix >= 0 && ix < grid_in[0] && iy >= 0 && iy < grid_in[1] && iz >= 0 && iz < grid_in[2])
            j = find_key(in_keys, n_in, key_of(c[0], iz, iy, ix, grid_in));
          nbr[(int64_t)k * capacity_out + o] = (int32_t)j;
        }
      }
  free(in_keys);
  return n_out;
}

/*
 * Inverse of a stride-2 map.  The stride-2 map lists pairs (coarse output j, tap k, fine input i =
 * down[k][j]); the transposed convolution sends the coarse features back along the same pairs:
 *     y_fine[i] = sum over pairs (j, k, i) of x_coarse[j] * W[k].
 * As a gather table for the fine sites: inv[k*capacity_fine + i] = j if down[k*capacity_coarse + j] == i,
 * else -1.  A fine site is read by at most one coarse site per tap (i = 2j - 1 + k fixes j), so the
 * table is well defined; a second claim on the same entry is reported as an argument error.
 * Returns the number of pairs, or a negative error.
 */
int64_t emc2o_invert_kmap(const int32_t* down, int64_t n_coarse, int64_t capacity_coarse, int64_t n_fine,
                          int64_t capacity_fine, int32_t* inv) {
  if (n_coarse < 0 || n_fine < 0 || n_coarse > capacity_coarse || n_fine > capacity_fine) return EMC2O_ERR_ARG;
  for (int k = 0; k < 27; ++k)
    for (int64_t i = 0; i < capacity_fine; ++i) inv[(int64_t)k * capacity_fine + i] = -1;
  int64_t pairs = 0;
  for (int k = 0; k < 27; ++k)
    for (int64_t j = 0; j < n_coarse; ++j) {
      const int32_t i = down[(int64_t)k * capacity_coarse + j];
      if (i < 0) continue;
      if (i >= n_fine) return EMC2O_ERR_ARG;
      if (inv[(int64_t)k * capacity_fine + i] != -1) return EMC2O_ERR_ARG;
      inv[(int64_t)k * capacity_fine + i] = (int32_t)j;
      ++pairs;
    }
  return pairs;
}

/*
 * Bird's-eye-view flattening: out[b][y][x][z*C + c] = feats[v][c] for the voxel v at (b, z, y, x), zero
 * where no voxel sits.  out is [n_batch][Gy][Gx][Gz*C] float.  Returns the number of voxels placed, or a
 * negative error (coordinate outside the grid, or two voxels at one cell).
 */
int64_t emc2o_bev_flatten(const int32_t* coords, const float* feats, int64_t n, const int32_t grid[3],
                          int32_t n_batch, int32_t c, float* out) {
  if (n < 0 || c < 1 || n_batch < 1) return EMC2O_ERR_ARG;
  const int64_t gx = grid[0], gy = grid[1], gz = grid[2];
  const int64_t total = (int64_t)n_batch * gy * gx * gz * c;
  for (int64_t t = 0; t < total; ++t) out[t] = 0.0f;
  unsigned char* taken = (unsigned char*)calloc((size_t)((int64_t)n_batch * gy * gx * gz > 0 ? (int64_t)n_batch * gy * gx * gz : 1), 1);
  if (!taken) return EMC2O_ERR_NOMEM;
  for (int64_t v = 0; v < n; ++v) {
    const int32_t* q = coords + 4 * v;
    if (q[0] < 0 || q[0] >= n_batch || q[1] < 0 || q[1] >= gz || q[2] < 0 || q[2] >= gy || q[3] < 0 || q[3] >= gx) {
      free(taken);
      return EMC2O_ERR_ARG;
    }
    const int64_t cell = (((int64_t)q[0] * gy + q[2]) * gx + q[3]) * gz + q[1];
    if (taken[cell]) { free(taken); return EMC2O_ERR_ARG; }
    taken[cell] = 1;
    for (int32_t ch = 0; ch < c; ++ch) out[cell * c + ch] = feats[v * c + ch];
  }
  free(taken);
  return n;
}

/* ------------------------------------------------------------------------------------------- */
/* Multiscale Pooling and multimodal fusion                                                    */
/* ------------------------------------------------------------------------------------------- */

/*
 * Multiscale Pooling of an image feature map into the cells of a voxel grid.
 *
 * Pixel (row j, col i) sits at (u, v) = (i, j), as in the projection above.  It is relevant iff its
 * depth d (distance along the camera's optical axis, the w of the projection) is finite and > 0.
 * Its 3D position in the LiDAR frame is X = Q (d*u, d*v, d, 1) with Q the 3x4 inverse of the
 * projection (given, fp32): each row evaluated left to right in fp64 without fused multiply-add,
 * then rounded once to fp32; the cell is the voxelizer's (fp32 subtract, divide, floor).  Pixels
 * outside the grid are dropped.  Every cell that receives at least one pixel becomes one output,
 * in ascending key order:
 *   coords[c] = (b, z, y, x) with b = batch_index, counts[c] = pixels pooled,
 *   feats[c][ch] = mode 0: mean over the cell's pixels (fp64 sum, one rounding to fp32)
 *                  mode 1: max  over the cell's pixels.
 * xyz (optional, [H][W][3] float): the lifted position of every pixel, NaN where not relevant.
 * Returns the number of cells or a negative error.
 */
int64_t emc2o_pool_image(const float* img, const float* depth, int32_t h, int32_t wd, int32_t c,
                         const float q[12], const float lo[3], const float vs[3], const int32_t grid[3],
                         int32_t n_batch, int32_t batch_index, int32_t mode, int64_t capacity,
                         int32_t* coords, float* feats, int32_t* counts, float* xyz) {
  if (h < 1 || wd < 1 || c < 1 || n_batch < 1 || batch_index < 0 || batch_index >= n_batch ||
      (mode != 0 && mode != 1) || grid[0] < 1 || grid[1] < 1 || grid[2] < 1)
    return EMC2O_ERR_ARG;
  const int64_t npix = (int64_t)h * wd;
  keyed_t* ks = (keyed_t*)malloc(sizeof(keyed_t) * (size_t)npix);
  double* acc = (double*)malloc(sizeof(double) * (size_t)c);
  if (!ks || !acc) { free(ks); free(acc); return EMC2O_ERR_NOMEM; }
  int64_t m = 0;
  for (int64_t j = 0; j < h; ++j) {
    for (int64_t i = 0; i < wd; ++i) {
      const int64_t pix = j * wd + i;
      const float df = depth[pix];
      float x3[3] = {NAN, NAN, NAN};
      if (isfinite(df) && df > 0.0f) {
        const double d = (double)df;
        const double du = d * (double)i, dv = d * (double)j;
        for (int r = 0; r < 3; ++r) {
          const double t = (double)q[4 * r + 0] * du + (double)q[4 * r + 1] * dv +
                           (double)q[4 * r + 2] * d + (double)q[4 * r + 3];
          x3[r] = (float)t;
        }
        const int cx = cell_of(x3[0], lo[0], vs[0], grid[0]);
        const int cy = cell_of(x3[1], lo[1], vs[1], grid[1]);
        const int cz = cell_of(x3[2], lo[2], vs[2], grid[2]);
        if (cx >= 0 && cy >= 0 && cz >= 0) {
          ks[m].key = key_of(batch_index, cz, cy, cx, grid);
          ks[m].idx = pix;
          ++m;
        }
      }
      if (xyz) { xyz[3 * pix] = x3[0]; xyz[3 * pix + 1] = x3[1]; xyz[3 * pix + 2] = x3[2]; }
    }
  }
  qsort(ks, (size_t)m, sizeof(keyed_t), cmp_keyed);
  int64_t n = 0, a = 0;
  while (a < m) {
    int64_t b = a;
    while (b < m && ks[b].key == ks[a].key) ++b;
    if (n >= capacity) { free(ks); free(acc); return EMC2O_ERR_CAPACITY; }
    for (int ch = 0; ch < c; ++ch) acc[ch] = mode == 0 ? 0.0 : -INFINITY;
    for (int64_t t = a; t < b; ++t) {
      const float* row = img + ks[t].idx * c;
      for (int ch = 0; ch < c; ++ch) {
        if (mode == 0) acc[ch] += (double)row[ch];
        else if ((double)row[ch] > acc[ch]) acc[ch] = (double)row[ch];
      }
    }
    const double cnt = (double)(b - a);
    for (int ch = 0; ch < c; ++ch) feats[n * c + ch] = (float)(mode == 0 ? acc[ch] / cnt : acc[ch]);
    uint64_t k = ks[a].key;
    coords[4 * n + 3] = (int32_t)(k % (uint64_t)grid[0]); k /= (uint64_t)grid[0];
    coords[4 * n + 2] = (int32_t)(k % (uint64_t)grid[1]); k /= (uint64_t)grid[1];
    coords[4 * n + 1] = (int32_t)(k % (uint64_t)grid[2]); k /= (uint64_t)grid[2];
    coords[4 * n + 0] = (int32_t)k;
    counts[n] = (int32_t)(b - a);
    ++n;
    a = b;
  }
  free(ks);
  free(acc);
  return n;
}

/* Keys of a coordinate list that must be strictly ascending and inside the grid; NULL on violation. */
static uint64_t* checked_keys(const int32_t* coords, int64_t n, const int32_t grid[3], int32_t n_batch) {
  uint64_t* keys = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(n > 0 ? n : 1));
  if (!keys) return NULL;
  for (int64_t i = 0; i < n; ++i) {
    const int32_t* q = coords + 4 * i;
    if (q[0] < 0 || q[0] >= n_batch || q[1] < 0 || q[1] >= grid[2] || q[2] < 0 || q[2] >= grid[1] ||
        q[3] < 0 || q[3] >= grid[0]) { free(keys); return NULL; }
    keys[i] = key_of(q[0], q[1], q[2], q[3], grid);
    if (i > 0 && keys[i] <= keys[i - 1]) { free(keys); return NULL; }
  }
  return keys;
}

/*
 * Multimodal fusion of two sparse sets on one grid: LiDAR voxels (coords_l, feats_l[.][cl]) and pooled
 * image cells (coords_i, feats_i[.][ci]), both in ascending key order.  Output: the union of their
 * sites in ascending key order, features concatenated [LiDAR | image]; an image cell with no voxel at
 * its coordinate gets a zero LiDAR half (Fig. 5 caption), a voxel with no image cell a zero image half.
 * src_l / src_i (optional): index of the row of each input that feeds output row r, or -1.
 * Returns the number of fused sites, or a negative error.
 */
int64_t emc2o_fuse(const int32_t* coords_l, const float* feats_l, int64_t n_l, int32_t cl,
                   const int32_t* coords_i, const float* feats_i, int64_t n_i, int32_t ci,
                   const int32_t grid[3], int32_t n_batch, int64_t capacity, int32_t* coords, float* feats,
                   int32_t* src_l, int32_t* src_i) {
  if (n_l < 0 || n_i < 0 || cl < 1 || ci < 1 || n_batch < 1) return EMC2O_ERR_ARG;
  uint64_t* kl = checked_keys(coords_l, n_l, grid, n_batch);
  uint64_t* ki = checked_keys(coords_i, n_i, grid, n_batch);
  if (!kl || !ki) { free(kl); free(ki); return EMC2O_ERR_ARG; }
  const int32_t cf = cl + ci;
  int64_t a = 0, b = 0, n = 0;
  while (a < n_l || b < n_i) {
    /* the smaller head key comes next; equal keys are one site fed by both */
    const int take_l = a < n_l && (b >= n_i || kl[a] <= ki[b]);
    const int take_i = b < n_i && (a >= n_l || ki[b] <= kl[a]);
    if (n >= capacity) { free(kl); free(ki); return EMC2O_ERR_CAPACITY; }
    const int32_t* q = take_l ? coords_l + 4 * a : coords_i + 4 * b;
    for (int t = 0; t < 4; ++t) coords[4 * n + t] = q[t];
    for (int ch = 0; ch < cl; ++ch) feats[n * cf + ch] = take_l ? feats_l[a * cl + ch] : 0.0f;
    for (int ch = 0; ch < ci; ++ch) feats[n * cf + cl + ch] = take_i ? feats_i[b * ci + ch] : 0.0f;
    if (src_l) src_l[n] = take_l ? (int32_t)a : -1;
    if (src_i) src_i[n] = take_i ? (int32_t)b : -1;
    a += take_l;
    b += take_i;
    ++n;
  }
  free(kl);
  free(ki);
  return n;
}

/* ------------------------------------------------------------------------------------------- */
/* Scenario-Adaptive Dispatcher                                                                */
/* ------------------------------------------------------------------------------------------- */

/*
 * Expert of every scene (Sec. 3.2).  props[i] = (x, y, z, confidence) of proposal region i, scene[i] its
 * scene.  A proposal is "far" unless fl(fl(x*x) + fl(y*y)) < fl(D*D) (range in the ground plane, compared
 * squared in fp32), "unclear" unless confidence >= C; a NaN therefore counts as far / unclear.
 *   expert 2 (accuracy-prioritised):  some proposal is far and unclear;
 *   expert 1 (versatile efficiency):  otherwise, some proposal is near and unclear, or far and clear;
 *   expert 0 (latency-prioritised):   otherwise (every proposal near and clear; also a scene without any).
 * counts[e] = scenes of expert e; order = the scene indices grouped by expert (0, then 1, then 2), ascending
 * within a group: the batches each expert's stack runs on.  Proposals with a scene id outside
 * [0, n_scenes) are ignored.  Returns 0 or a negative error.
 */
int32_t emc2o_dispatch(const float* props, const int32_t* scene, int64_t n, int32_t n_scenes, float dist,
                       float conf, int32_t* expert, int32_t* counts, int32_t* order) {
  if (n < 0 || n_scenes < 0 || !(dist >= 0.0f)) return EMC2O_ERR_ARG;
  volatile float d2v = dist * dist;
  const float d2 = d2v;
  for (int32_t s = 0; s < n_scenes; ++s) expert[s] = 0;
  for (int64_t i = 0; i < n; ++i) {
    const int32_t s = scene ? scene[i] : 0;
    if (s < 0 || s >= n_scenes) continue;
    const float* p = props + 4 * i;
    volatile float xx = p[0] * p[0];
    volatile float yy = p[1] * p[1];
    volatile float r2v = xx + yy;
    const float r2 = r2v;
    const int far = !(r2 < d2);
    const int unclear = !(p[3] >= conf);
    const int e = (far && unclear) ? 2 : ((far || unclear) ? 1 : 0);
    if (e > expert[s]) expert[s] = e;
  }
  counts[0] = counts[1] = counts[2] = 0;
  for (int32_t s = 0; s < n_scenes; ++s) counts[expert[s]]++;
  int32_t at[3] = {0, counts[0], counts[0] + counts[1]};
  for (int32_t s = 0; s < n_scenes; ++s) order[at[expert[s]]++] = s;
  return 0;
}

/*
 * Expert-grouped batching (Sec. 3.2: every scene is routed to one expert, so each expert's network runs on the
 * scenes routed to it).  Given the dispatcher's outputs, the points of the batch get the batch ids of expert e's
 * group: slot[s] = position of scene s inside its expert's part of `order` (for every scene, whatever its expert);
 * group_batch[i] = slot[scene[i]] if scene i's expert is e, else -1 (the voxelizer drops such points; also for a
 * scene id outside [0, n_scenes)).  Written the slow way: the position is found by searching `order`.
 * Returns 0 or a negative error (an `order` that is not a grouping of the scenes by `expert`).
 */
int32_t emc2o_group_points(const int32_t* scene, int64_t n_points, const int32_t* expert, const int32_t* order,
                           const int32_t* counts, int32_t n_scenes, int32_t e, int32_t* slot, int32_t* group_batch) {
  if (n_scenes < 1 || n_points < 0 || e < 0 || e > 2) return EMC2O_ERR_ARG;
  if (counts[0] < 0 || counts[1] < 0 || counts[2] < 0 || counts[0] + counts[1] + counts[2] != n_scenes) return EMC2O_ERR_ARG;
  for (int32_t s = 0; s < n_scenes; ++s) {
    if (expert[s] < 0 || expert[s] > 2) return EMC2O_ERR_ARG;
    int32_t start = 0;
    for (int32_t x = 0; x < expert[s]; ++x) start += counts[x];
    int32_t found = -1;
    for (int32_t p = start; p < start + counts[expert[s]]; ++p)
      if (order[p] == s) { found = p - start; break; }
    if (found < 0) return EMC2O_ERR_ARG;
    slot[s] = found;
  }
  for (int64_t i = 0; i < n_points; ++i) {
    const int32_t s = scene ? scene[i] : 0;
    group_batch[i] = (s >= 0 && s < n_scenes && expert[s] == e) ? slot[s] : -1;
  }
  return 0;
}

/* ------------------------------------------------------------------------------------------- */
/* sparse convolution                                                                          */
/* ------------------------------------------------------------------------------------------- */

/*
 * acc[o][c'] = sum over taps k with nbr[k][o] >= 0, sum over c: x[nbr[k][o]][c] * W[k][c][c'];
 * y = epi(acc): 0 identity, 1 acc*scale+shift, 2 max(0, acc*scale+shift).  All in fp64, one
 * rounding to fp32 at the end.  x and w are fp32 (16-bit data is passed already rounded and
 * up-cast, which is exact).  Returns the number of multiply-accumulates done (= pairs*Cin*Cout),
 * or a negative error.
 */
int64_t emc2o_spconv(const float* x, int64_t n_in, const float* w, const float* scale,
                     const float* shift, int32_t epilogue, const int32_t* nbr, int64_t nbr_stride,
                     int64_t n_out, int32_t cin, int32_t cout, float* y) {
  if (n_out < 0 || n_out > nbr_stride || cin < 1 || cout < 1 || epilogue < 0 || epilogue > 2)
    return EMC2O_ERR_ARG;
  if (epilogue != 0 && (!scale || !shift)) return EMC2O_ERR_ARG;
  double* acc = (double*)calloc((size_t)(n_out > 0 ? n_out : 1) * (size_t)cout, sizeof(double));
  if (!acc) return EMC2O_ERR_NOMEM;
  int64_t macs = 0;
  int bad = 0;
  for (int k = 0; k < 27; ++k) {
    const float* wk = w + (int64_t)k * cin * cout;
    const int32_t* nk = nbr + (int64_t)k * nbr_stride;
    int64_t pairs = 0;
#pragma omp parallel for num_threads(g_threads) schedule(static) reduction(+ : pairs) reduction(| : bad)
    for (int64_t o = 0; o < n_out; ++o) {
      int64_t j = nk[o];
      if (j < 0) continue;
      if (j >= n_in) { bad |= 1; continue; }
      ++pairs;
      const float* xr = x + j * cin;
      double* ar = acc + o * cout;
      for (int c = 0; c < cin; ++c) {
        const double xv = (double)xr[c];
        const float* wr = wk + (int64_t)c * cout;
        for (int d = 0; d < cout; ++d) ar[d] += xv * (double)wr[d];
      }
    }
    macs += pairs * cin * cout;
  }
  if (bad) { free(acc); return EMC2O_ERR_ARG; }
  for (int64_t o = 0; o < n_out; ++o)
    for (int d = 0; d < cout; ++d) {
      double v = acc[o * cout + d];
      if (epilogue != 0) v = v * (double)scale[d] + (double)shift[d];
      if (epilogue == 2 && !(v > 0.0)) v = 0.0;
      y[o * cout + d] = (float)v;
    }
  free(acc);
  return macs;
}

/* ------------------------------------------------------------------------------------------- */
/* projection + bilinear gather                                                                */
/* ------------------------------------------------------------------------------------------- */

/* ------------------------------------------------------------------------------------------- */
/* quantised sparse convolution                                                                */
/* ------------------------------------------------------------------------------------------- */

/* q = clamp(rint(fl(x * inv_scale)), -127, 127), ties to even; NaN -> 0. */
static int8_t quant_i8(float x, float inv_scale) {
  volatile float t = x * inv_scale;
  float r = rintf(t); /* default rounding mode: to nearest, ties to even */
  if (!(r == r)) return 0;
  if (r > 127.0f) r = 127.0f;
  if (r < -127.0f) r = -127.0f;
  return (int8_t)r;
}

int32_t emc2o_quantize_i8(const float* x, int64_t n, float inv_scale, int8_t* q) {
  if (n < 0) return EMC2O_ERR_ARG;
  for (int64_t i = 0; i < n; ++i) q[i] = quant_i8(x[i], inv_scale);
  return 0;
}

/*
 * acc[o][c'] = sum over taps k with nbr[k][o] >= 0, sum over c: xq[nbr[k][o]][c] * wq[k][c][c'], exact integers;
 * v = fl(fl((float)acc * mul[c']) + add[c'])   (int -> fp32 to nearest; product and sum rounded separately, no
 * fused multiply-add); relu: v = max(v, 0).  out_v receives v.  If out_q is given it receives
 * quant_i8(v, inv_out_scale).  Returns the number of multiply-accumulates, or a negative error.
 */
int64_t emc2o_spconv_i8(const int8_t* xq, int64_t n_in, const int8_t* wq, const float* mul, const float* add,
                        int32_t relu, float inv_out_scale, const int32_t* nbr, int64_t nbr_stride, int64_t n_out,
                        int32_t cin, int32_t cout, float* out_v, int8_t* out_q) {
  if (n_out < 0 || n_out > nbr_stride || cin < 1 || cout < 1 || !mul || !add) return EMC2O_ERR_ARG;
  int64_t* acc = (int64_t*)calloc((size_t)(n_out > 0 ? n_out : 1) * (size_t)cout, sizeof(int64_t));
  if (!acc) return EMC2O_ERR_NOMEM;
  int64_t macs = 0;
  for (int k = 0; k < 27; ++k) {
    const int8_t* wk = wq + (int64_t)k * cin * cout;
    for (int64_t o = 0; o < n_out; ++o) {
      const int32_t j = nbr[(int64_t)k * nbr_stride + o];
      if (j < 0) continue;
      if (j >= n_in) { free(acc); return EMC2O_ERR_ARG; }
      const int8_t* xr = xq + (int64_t)j * cin;
      int64_t* ar = acc + o * cout;
      for (int c = 0; c < cin; ++c) {
        const int64_t xv = xr[c];
        const int8_t* wr = wk + (int64_t)c * cout;
        for (int cc = 0; cc < cout; ++cc) ar[cc] += xv * (int64_t)wr[cc];
      }
      macs += (int64_t)cin * cout;
    }
  }
  for (int64_t o = 0; o < n_out; ++o)
    for (int cc = 0; cc < cout; ++cc) {
      const float a = (float)acc[o * cout + cc];
      volatile float p = a * mul[cc];
      volatile float sum = p + add[cc];
      float v = sum;
      if (relu && !(v > 0.0f)) v = 0.0f;
      out_v[o * cout + cc] = v;
      if (out_q) out_q[o * cout + cc] = quant_i8(v, inv_out_scale);
    }
  free(acc);
  return macs;
}

/* ------------------------------------------------------------------------------------------- */
/* fp8 (E4M3) sparse convolution                                                               */
/* ------------------------------------------------------------------------------------------- */

/*
 * The 8-bit floating-point format used here is E4M3 without infinities (1 sign bit, 4 exponent bits with bias 7,
 * 3 mantissa bits): code s.eeee.mmm is (-1)^s 2^(e-7) (1 + m/8) for e > 0 and (-1)^s 2^(-6) (m/8) for e = 0; the two
 * codes with all exponent and mantissa bits set are not numbers; the largest finite value is 448 (code 0x7E).
 */
double emc2o_e4m3_value(uint8_t code) {
  const int s = code >> 7, e = (code >> 3) & 15, m = code & 7;
  if (e == 15 && m == 7) return NAN;
  const double mag = e > 0 ? ldexp(1.0 + m / 8.0, e - 7) : ldexp(m / 8.0, -6);
  return s ? -mag : mag;
}

/*
 * Quantiser: the finite E4M3 value nearest to t = fl(x * inv_scale) (the product rounded to fp32), ties to the code
 * with an even mantissa, |t| beyond 448 (also infinities) saturating to +-448, NaN -> +0; zero keeps its sign bit clear
 * (-0 and values that round to zero give code 0x00).  Written as a search over the 127 positive codes: no bit tricks.
 */
static uint8_t quant_e4m3(float x, float inv_scale) {
  volatile float tf = x * inv_scale;
  const double t = (double)tf;
  if (!(t == t)) return 0;
  const double a = fabs(t);
  int best = 0;
  double best_d = a; /* distance to code 0 */
  for (int c = 1; c <= 0x7E; ++c) {
    const double d = fabs(a - emc2o_e4m3_value((uint8_t)c));
    if (d < best_d || (d == best_d && (c & 1) == 0)) { best = c; best_d = d; }
  }
  if (best == 0) return 0;
  return (uint8_t)(best | (t < 0 ? 0x80 : 0));
}

int32_t emc2o_quantize_e4m3(const float* x, int64_t n, float inv_scale, uint8_t* q) {
  if (n < 0) return EMC2O_ERR_ARG;
  for (int64_t i = 0; i < n; ++i) q[i] = quant_e4m3(x[i], inv_scale);
  return 0;
}

/*
 * acc[o][c'] = sum over taps k with nbr[k][o] >= 0, sum over c: value(xq[nbr[k][o]][c]) * value(wq[k][c][c']), in fp64
 * (every product of two E4M3 values is exact there, and so is a sum of a few thousand of them), rounded once to
 * fp32; then, as in the int8 scheme, v = fl(fl(acc * mul[c']) + add[c']) with separately rounded product and sum,
 * relu: v = max(v, 0).  A code that is not a number anywhere in xq or wq is an error.  Returns the number of
 * multiply-accumulates, or a negative error.
 */
int64_t emc2o_spconv_e4m3(const uint8_t* xq, int64_t n_in, const uint8_t* wq, const float* mul, const float* add,
                          int32_t relu, const int32_t* nbr, int64_t nbr_stride, int64_t n_out, int32_t cin, int32_t cout,
                          float* out_v) {
  if (n_out < 0 || n_out > nbr_stride || cin < 1 || cout < 1 || !mul || !add) return EMC2O_ERR_ARG;
  for (int64_t i = 0; i < n_in * cin; ++i)
    if ((xq[i] & 0x7F) == 0x7F) return EMC2O_ERR_ARG;
  for (int64_t i = 0; i < (int64_t)27 * cin * cout; ++i)
    if ((wq[i] & 0x7F) == 0x7F) return EMC2O_ERR_ARG;
  /* decode every operand once (each code to its value), then the plain loops */
  double* acc = (double*)calloc((size_t)(n_out > 0 ? n_out : 1) * (size_t)cout, sizeof(double));
  double* xv = (double*)malloc(sizeof(double) * (size_t)(n_in > 0 ? n_in : 1) * (size_t)cin);
  double* wv = (double*)malloc(sizeof(double) * (size_t)27 * cin * cout);
  if (!acc || !xv || !wv) { free(acc); free(xv); free(wv); return EMC2O_ERR_NOMEM; }
  for (int64_t i = 0; i < n_in * cin; ++i) xv[i] = emc2o_e4m3_value(xq[i]);
  for (int64_t i = 0; i < (int64_t)27 * cin * cout; ++i) wv[i] = emc2o_e4m3_value(wq[i]);
  int64_t macs = 0;
  int bad = 0;
  for (int k = 0; k < 27; ++k) {
    const double* wk = wv + (int64_t)k * cin * cout;
#ifdef _OPENMP
#pragma omp parallel for schedule(static) reduction(+ : macs) reduction(| : bad)
#endif
    for (int64_t o = 0; o < n_out; ++o) {
      const int32_t j = nbr[(int64_t)k * nbr_stride + o];
      if (j < 0) continue;
      if (j >= n_in) { bad |= 1; continue; }
      const double* xr = xv + (int64_t)j * cin;
      double* ar = acc + o * cout;
      for (int c = 0; c < cin; ++c) {
        const double x1 = xr[c];
        const double* wr = wk + (int64_t)c * cout;
        for (int cc = 0; cc < cout; ++cc) ar[cc] += x1 * wr[cc];
      }
      macs += (int64_t)cin * cout;
    }
  }
  free(xv);
  free(wv);
  if (bad) { free(acc); return EMC2O_ERR_ARG; }
  for (int64_t o = 0; o < n_out; ++o)
    for (int cc = 0; cc < cout; ++cc) {
      const float a = (float)acc[o * cout + cc];
      volatile float p = a * mul[cc];
      volatile float sum = p + add[cc];
      float v = sum;
      if (relu && !(v > 0.0f)) v = 0.0f;
      out_v[o * cout + cc] = v;
    }
  free(acc);
  return macs;
}

/*
 * (U, V, w) = P (x, y, z, 1); u = U/w, v = V/w; valid iff w > 0, 0 <= u <= W-1, 0 <= v <= H-1.
 * Pixel (row j, col i) sits at (u, v) = (i, j).  Bilinear blend of the four surrounding pixels
 * (upper neighbours clamped to the last row/col); invalid points get an all-zero row.
 * img: [H][W][C] fp32 (fp16 data up-cast exactly).  out: [n][C] fp32, valid: [n] u8,
 * uv: [n][2] fp64 or NULL (written for every point with w != 0, NaN otherwise).
 */
int32_t emc2o_project_gather(const float* points, int32_t stride_f, int64_t n, const float pm[12],
                             const float* img, int32_t h, int32_t wd, int32_t c, float* out,
                             uint8_t* valid, double* uv) {
  if (n < 0 || stride_f < 3 || h < 1 || wd < 1 || c < 1) return EMC2O_ERR_ARG;
  for (int64_t i = 0; i < n; ++i) {
    const float* p = points + i * stride_f;
    const double x = p[0], y = p[1], z = p[2];
    const double uu = (double)pm[0] * x + (double)pm[1] * y + (double)pm[2] * z + (double)pm[3];
    const double vv = (double)pm[4] * x + (double)pm[5] * y + (double)pm[6] * z + (double)pm[7];
    const double ww = (double)pm[8] * x + (double)pm[9] * y + (double)pm[10] * z + (double)pm[11];
    float* o = out + i * c;
    int ok = 0;
    double u = NAN, v = NAN;
    if (ww > 0.0) {
      u = uu / ww;
      v = vv / ww;
      ok = (u >= 0.0 && u <= (double)(wd - 1) && v >= 0.0 && v <= (double)(h - 1));
    } else if (ww < 0.0) {
      u = uu / ww;
      v = vv / ww;
    }
    if (uv) { uv[2 * i] = u; uv[2 * i + 1] = v; }
    valid[i] = (uint8_t)ok;
    if (!ok) {
      for (int ch = 0; ch < c; ++ch) o[ch] = 0.0f;
      continue;
    }
    int i0 = (int)floor(u), j0 = (int)floor(v);
    int i1 = i0 + 1 < wd ? i0 + 1 : wd - 1;
    int j1 = j0 + 1 < h ? j0 + 1 : h - 1;
    double a = u - (double)i0, b = v - (double)j0;
    const float* p00 = img + ((int64_t)j0 * wd + i0) * c;
    const float* p01 = img + ((int64_t)j0 * wd + i1) * c;
    const float* p10 = img + ((int64_t)j1 * wd + i0) * c;
    const float* p11 = img + ((int64_t)j1 * wd + i1) * c;
    for (int ch = 0; ch < c; ++ch) {
      double g = (1.0 - a) * (1.0 - b) * (double)p00[ch] + a * (1.0 - b) * (double)p01[ch] +
                 (1.0 - a) * b * (double)p10[ch] + a * b * (double)p11[ch];
      o[ch] = (float)g;
    }
  }
  return 0;
}
