/*
 * emc2.h -- C-ABI of the MI355X (gfx950) hot path of the EMC2 LiDAR branch:
 *   multi-scale voxelization  ->  27-offset kernel map  ->  sparse 3D conv (+ fused affine/ReLU)
 *   ->  point-to-image projection with bilinear feature gather,
 * and on the same data structures: inverse kernel map + bird's-eye-view flattening (decoder side),
 * Multiscale Pooling of image features + multimodal fusion, the scene dispatcher, an int8 sparse conv.
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers (HBM, on the context's device); h_* and plain
 *     struct/array arguments are HOST pointers.  The caller owns every input and output buffer;
 *     the context owns all scratch (per-voxel point stash, cell-index slots, scan partials, per-pixel
 *     sort arrays of the pooling, status word), allocated once in emc2_create.  No call below
 *     allocates or frees device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls validate their
 *     arguments synchronously, enqueue kernels on `stream` and return; they never block unless a
 *     host count pointer (h_n_*) is given.  Counts (n_voxels, n_out) are produced in DEVICE memory
 *     so that downstream calls need no host round trip: launches are sized by `capacity`, kernels
 *     bound themselves by the device count.
 *   - Errors found on the host are returned at once.  Errors only the device can see (more voxels
 *     than `capacity`; a kernel-map entry at or beyond the input's row count) set a device status word;
 *     emc2_status_sync returns and clears it.  After such an error the outputs of that call are
 *     truncated (capacity) or computed without the offending entries (map), and every access stayed
 *     in bounds.
 *   - emc2_voxelize, emc2_build_kmap, emc2_build_inverse_kmap (reads an index slot), emc2_pool_image,
 *     emc2_fuse and emc2_spconv with EMC2_W_PLAIN weights on an MFMA shape share the context's scratch
 *     and index slots: issue them on one stream at a time.  emc2_spconv with packed (or non-MFMA)
 *     weights, emc2_spconv_i8, emc2_quantize_i8, the weight-packing calls into caller memory,
 *     emc2_bev_flatten, emc2_dispatch and emc2_project_gather touch no mutable context state and may
 *     run on other streams concurrently, ordered by the caller's events (a conv must wait for the
 *     call that wrote the map and features it reads).
 *   - Voxel order everywhere: ascending key ((b*Gz + z)*Gy + y)*Gx + x, i.e. lexicographic
 *     (b, z, y, x).  Coordinates are int32 quadruples (b, z, y, x).
 */
#ifndef EMC2_H_
#define EMC2_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  EMC2_OK = 0,
  EMC2_ERR_INVALID_ARG = 1, /* null/mis-sized argument, size beyond what the context was made for */
  EMC2_ERR_CAPACITY = 2,    /* more voxels than `capacity`                                         */
  EMC2_ERR_UNSUPPORTED = 3, /* channel count / dtype / key width the kernels do not cover          */
  EMC2_ERR_DEVICE = 4,      /* a HIP runtime call failed; see emc2_last_error                      */
  EMC2_ERR_MAP = 5          /* a kernel-map entry named a row outside the input (found on the device) */
} emc2_status;

typedef struct emc2_ctx emc2_ctx;

/*
 * Create a context on `device`.
 *   max_points : largest n_points any emc2_voxelize call will pass; also the largest H*W of an image
 *                given to emc2_pool_image.
 *   max_voxels : largest voxel count (capacity) of any level.
 *   max_cells  : largest n_batch*Gx*Gy*Gz of any grid that is voxelized or mapped.
 *   n_slots    : number of cell-index slots kept alive at once (>= 1; see emc2_voxelize).
 * Scratch is about 32 B per point + 76 B per voxel + 8 B per 32 cells per index slot.
 */
emc2_status emc2_create(emc2_ctx** out, int device, int64_t max_points, int64_t max_voxels,
                        int64_t max_cells, int32_t n_slots);
void emc2_destroy(emc2_ctx* ctx);

/* Synchronise `stream`, return the device status accumulated since the last call (EMC2_OK if none),
 * and clear it. */
emc2_status emc2_status_sync(emc2_ctx* ctx, void* stream);

/* Text of the last host-side error on this context (never NULL); with ctx = NULL, of the last failed call
 * that takes no context (emc2_build_kmap_static). */
const char* emc2_last_error(const emc2_ctx* ctx);

/* Voxel grid: the "pool size" is a runtime parameter (paper Sec. 3.5, Multiscale Pooling is
 * user-configurable); the grid extent is given, never derived from bounds. */
typedef struct {
  float lo[3];      /* lower bound x, y, z                                             */
  float vs[3];      /* voxel size  x, y, z  (> 0)                                      */
  int32_t grid[3];  /* Gx, Gy, Gz                                                      */
  int32_t n_batch;  /* number of frames B >= 1                                         */
  float r2_min;     /* keep a point iff r2_min <= fl(fl(x*x)+fl(y*y)) < r2_max         */
  float r2_max;     /*   (0, +inf) switches the range filter off                       */
  int32_t stride_f; /* floats per point row (>= 4): x, y, z, intensity, ...            */
} emc2_voxel_spec;

typedef enum { EMC2_F32 = 0, EMC2_F16 = 1, EMC2_BF16 = 2, EMC2_I8 = 3 } emc2_dtype;  /* I8: quantised conv only */

/*
 * Voxelization with mean voxel features (paper Sec. 2: LiDAR methods process point clouds via
 * voxelization; Sec. 3.1: the data bridge prepares voxel features for the experts; Sec. 3.5:
 * configurable pool size -> call once per scale for multi-scale output).
 *
 * A point is kept iff, per axis a, t = fl(fl(p_a - lo_a) / vs_a) (IEEE fp32, true division)
 * satisfies 0 <= t < G_a, its batch id is in [0, n_batch), its intensity is finite and it passes
 * the range filter.  Its cell is floor(t).  Outputs, in ascending key order:
 *   d_coords [capacity][4] int32 (b, z, y, x)
 *   d_feats  [capacity][4] fp32  mean (x, y, z, intensity) over ALL points of the voxel
 *   d_counts [capacity]    int32 points per voxel
 *   d_feats_lp [capacity][4] copy of d_feats rounded (RNE) to `lp_dtype` (F16/BF16); NULL to skip
 *   d_n_voxels  device int32 (always written); h_n_voxels host int32, NULL = no sync
 * d_batch: [n_points] int32 or NULL (all points in frame 0).
 * index_slot in [0, n_slots): the cell index of the produced voxel set is left in that slot for
 * emc2_build_kmap to reuse; it stays valid until another call writes the same slot.
 * A voxel of up to four points is summed in fp32 in the order of the points' values, so its mean is the same bit for
 * bit in every run and for every order of the input; the points beyond the fourth are added with fp32 atomics
 * (order not fixed; result within a few ulp of exact).  Rows [n_voxels, min(n_points, capacity)) of d_feats and
 * d_counts are zeroed.
 */
emc2_status emc2_voxelize(emc2_ctx* ctx, const float* d_points, const int32_t* d_batch,
                          int64_t n_points, const emc2_voxel_spec* spec, int64_t capacity,
                          int32_t* d_coords, float* d_feats, int32_t* d_counts, void* d_feats_lp,
                          emc2_dtype lp_dtype, int32_t* d_n_voxels, int32_t* h_n_voxels,
                          int32_t index_slot, void* stream);

typedef enum { EMC2_CONV_SUBM = 0, EMC2_CONV_STRIDED = 1 } emc2_conv_kind;

/*
 * Kernel map (rulebook) of a 3x3x3 sparse convolution over the non-empty voxels (paper Sec. 3.5:
 * only non-empty voxels are computed, O(N*C_v); Sec. 3.6: prefix-sum index search).
 *
 * Tap k = (kz*3 + ky)*3 + kx, kx,ky,kz in {0,1,2}.  Output site o reads input site
 * i = o*s - 1 + (kx, ky, kz) in the same frame (cross-correlation), with
 *   SUBM    : s = 1, outputs == inputs (same order), grid_out = grid_in;
 *   STRIDED : s = 2 (k3 s2 p1), grid_out = (G-1)/2 + 1 per axis; output o is active iff at least
 *             one of its 27 taps reads an active input; outputs in ascending key order.
 * d_nbr[k*capacity_out + o] = index of the input voxel read by (o, k), or -1.
 *
 *   d_in_coords [n_in][4] ascending key; d_n_in device int32 count.
 *   in_slot  : index slot holding the cell index of exactly these inputs (left there by
 *              emc2_voxelize or by a STRIDED call's out_slot), or -1 to rebuild it from d_in_coords.
 *   out_slot : STRIDED only: slot that receives the cell index of the outputs (or -1: internal,
 *              not kept).  Must differ from in_slot.
 *   d_out_coords [capacity_out][4]: STRIDED: written.  SUBM: may be NULL or == d_in_coords;
 *              otherwise receives a copy.
 *   d_n_out  device int32 (written; SUBM: copy of *d_n_in); h_n_out host, NULL = no sync.
 *   grid_out host int32[3], written.
 * capacity_out must be >= the true output count (else EMC2_ERR_CAPACITY via the status word; the
 * map is then truncated to the first capacity_out outputs).
 */
emc2_status emc2_build_kmap(emc2_ctx* ctx, emc2_conv_kind kind, const int32_t* d_in_coords,
                            const int32_t* d_n_in, int64_t capacity_in, const int32_t grid_in[3],
                            int32_t n_batch, int32_t in_slot, int32_t out_slot, int64_t capacity_out,
                            int32_t* d_out_coords, int32_t* d_n_out, int32_t* d_nbr,
                            int32_t grid_out[3], int32_t* h_n_out, void* stream);

/*
 * emc2_build_kmap for callers that cannot allocate device memory and therefore cannot hold a context: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, arguments and results
 * as emc2_build_kmap with in_slot = out_slot = -1 (the cell index is rebuilt from d_in_coords, nothing is kept),
 * but the scratch (two cell-index slots, scan partials, status word: about 8.4 MB) is a static device array that
 * every GPU the library runs on holds until the process ends.  It allocates and frees nothing, on the host or
 * on the device, and never synchronises.
 *   - Works on the CURRENT device; d_* pointers must belong to it.
 *   - n_batch*Gx*Gy*Gz of grid_in must not exceed EMC2_STATIC_KMAP_MAX_CELLS: EMC2_ERR_INVALID_ARG otherwise
 *     (text through emc2_last_error(NULL)); larger grids need a context.
 *   - d_status: device int32 that receives this call's status bits (0 = fine, bit 0 = more outputs than
 *     capacity_out: results truncated but in bounds), or NULL to ignore them.
 *   - Every call on a GPU shares that GPU's one array: calls that overlap in time on one GPU (two streams, two
 *     host threads) race and give wrong maps.  Issue them on one stream, or order them with events.
 *   - The first call on a device also enqueues a one-time zero fill of the array on `stream`.
 */
#define EMC2_STATIC_KMAP_MAX_CELLS (1 << 24)
emc2_status emc2_build_kmap_static(emc2_conv_kind kind, const int32_t* d_in_coords, const int32_t* d_n_in,
                                   int64_t capacity_in, const int32_t grid_in[3], int32_t n_batch, int64_t capacity_out,
                                   int32_t* d_out_coords, int32_t* d_n_out, int32_t* d_nbr, int32_t grid_out[3],
                                   int32_t* d_status, void* stream);

typedef enum { EMC2_EPI_NONE = 0, EMC2_EPI_AFFINE = 1, EMC2_EPI_AFFINE_RELU = 2 } emc2_epilogue;

/* Weight layouts accepted by emc2_spconv: plain [27][Cin][Cout], or the matrix-core fragment order
 * produced by emc2_pack_weights (same byte size; only for channel counts the MFMA kernels cover). */
typedef enum { EMC2_W_PLAIN = 0, EMC2_W_PACKED = 1 } emc2_wlayout;

/*
 * 1 if (dtype, Cin, Cout) runs on the MFMA kernels (and therefore accepts EMC2_W_PACKED), else 0.
 * Host-only query about this library's kernel selection: no GPU work, and no passage of the paper stands
 * behind it.
 */
int32_t emc2_spconv_uses_mfma(emc2_dtype dtype, int32_t cin, int32_t cout);

/*
 * Re-order static weights once (model-load time) into the MFMA fragment order, so that the conv
 * does not have to do it per call (paper Sec. 3.6: graph-level optimisation of static operands).
 *   d_w [27][Cin][Cout] and d_packed [27*Cin*Cout], both of `dtype` (F16/BF16); must not overlap.
 * EMC2_ERR_UNSUPPORTED if emc2_spconv_uses_mfma(dtype, cin, cout) == 0.
 */
emc2_status emc2_pack_weights(emc2_ctx* ctx, emc2_dtype dtype, const void* d_w, int32_t cin, int32_t cout,
                              void* d_packed, void* stream);

/*
 * Sparse convolution over a kernel map, output-stationary gather-GEMM (paper Sec. 3.5: customised
 * 3D sparse convolution, the bulk of inference time; Sec. 3.6: graph fusion -> the folded-BN affine
 * and ReLU are fused into the epilogue):
 *   acc[o][c'] = sum_{k : nbr[k][o] >= 0} sum_c in[nbr[k][o]][c] * w[k][c][c']      (fp32 accumulate)
 *   out[o][c'] = acc | acc*scale[c'] + shift[c'] | max(0, acc*scale[c'] + shift[c'])
 *   d_in  [n_in][Cin], d_out [capacity_out][Cout], d_w: all of `dtype`;
 *   d_w in `w_layout`: EMC2_W_PLAIN = [27][Cin][Cout] (on the MFMA path it is re-ordered into
 *   context scratch by one extra small kernel per call), EMC2_W_PACKED = output of emc2_pack_weights
 *   d_scale, d_shift [Cout] fp32 (NULL iff EMC2_EPI_NONE)
 *   d_nbr [27][capacity_out] from emc2_build_kmap; d_n_out device int32 count of outputs.
 *   n_in_rows: rows of d_in the caller vouches for (its voxel count if known on the host, else the capacity
 *   the buffer was allocated with).  An entry of d_nbr at or beyond it is treated as absent -- nothing is read
 *   through it -- and EMC2_ERR_MAP is reported through the status word.
 *   For F16/BF16, d_in, d_w and d_out must be 16-byte aligned (EMC2_ERR_INVALID_ARG otherwise): rows move as
 *   8- and 16-byte pieces.
 * F16/BF16 run on MFMA for Cin in {16,32,64,128} and Cout in {32,64,128}; other channel counts
 * (Cin <= 1024, Cout <= 256) and F32 run on the vector ALU.  Rows [n_out, capacity_out) of d_out
 * are not written.
 *   map_hint: EMC2_CONV_SUBM / EMC2_CONV_STRIDED if d_nbr came from emc2_build_kmap with that kind, else
 *   EMC2_MAP_ANY.  A scheduling hint only (submanifold maps over key-sorted voxels let the three kx
 *   taps of a (dz, dy) pair share one fetch of input rows): results do not depend on it, for any table.
 */
#define EMC2_MAP_ANY (-1)
/*
 * Name of the device kernel emc2_spconv launches for these arguments ("k_spconv_span", "k_spconv_direct",
 * "k_spconv_mfma", "k_spconv_rows", "k_spconv_small" or "k_spconv_alu"): lets a profile be matched to a layer.  Host-only
 * query about this library's kernel selection (no GPU work, no passage of the paper behind it); the string
 * is static.  NULL for a dtype emc2_spconv rejects.
 */
const char* emc2_spconv_kernel(emc2_dtype dtype, int32_t cin, int32_t cout, int32_t map_hint);
emc2_status emc2_spconv(emc2_ctx* ctx, emc2_dtype dtype, const void* d_in, const void* d_w, emc2_wlayout w_layout,
                        const float* d_scale, const float* d_shift, emc2_epilogue epilogue,
                        const int32_t* d_nbr, int32_t map_hint, const int32_t* d_n_out, int64_t capacity_out,
                        int64_t n_in_rows, int32_t cin, int32_t cout, void* d_out, void* stream);

/*
 * Inverse (transposed) kernel map of a stride-2 layer, for the decoder half of the LiDAR UNet (paper
 * Sec. 3.1: the data bridge extracts LiDAR features with a UNet and a sparse CNN).  The stride-2 map
 * pairs coarse output j with fine input i = 2j - 1 + (kx, ky, kz) at tap k; the transposed convolution
 * sends coarse features back along the same pairs, y_fine[i] = sum_{(j,k,i)} x_coarse[j] * W[k], which is
 * emc2_spconv over the table built here:
 *   d_nbr[k*capacity_fine + i] = index of the coarse voxel at (i + 1 - k)/2 if that is integral on every
 *   axis and the coarse cell is active, else -1.
 *   d_fine_coords [n_fine][4] (b, z, y, x), d_n_fine device count: the sites that receive features.
 *   coarse_slot: index slot holding the cell index of the coarse level (the out_slot of the
 *   emc2_build_kmap(STRIDED) call that produced it); grid_coarse its grid; d_n_coarse its device count.
 * Integer work only; rows [n_fine, capacity_fine) of d_nbr are not written.
 */
emc2_status emc2_build_inverse_kmap(emc2_ctx* ctx, const int32_t* d_fine_coords, const int32_t* d_n_fine,
                                    int64_t capacity_fine, const int32_t grid_coarse[3], int32_t n_batch,
                                    int32_t coarse_slot, const int32_t* d_n_coarse, int32_t* d_nbr, void* stream);

/*
 * Bird's-eye-view flattening (paper Sec. 3.3: the latency-prioritised expert runs 2D CNNs on BEV
 * projections; Sec. 3.2: LiDAR information "compressed into bird's eye view"): the voxel set becomes a
 * dense, zero-filled tensor with the height axis folded into the channels,
 *   d_out[b][y][x][z*C + c] = d_feats[v][c]  for the voxel v at (b, z, y, x),   0 where no voxel sits.
 *   d_out [n_batch][Gy][Gx][Gz*C] of `dtype` (fully written by the call); d_feats [n][C] of `dtype`;
 *   C*sizeof(dtype) must be a multiple of 4.  Voxels with coordinates outside the grid are ignored.
 * A copy: bit-exact in every dtype.
 */
emc2_status emc2_bev_flatten(emc2_ctx* ctx, emc2_dtype dtype, const int32_t* d_coords, const void* d_feats,
                             const int32_t* d_n, int64_t capacity, const int32_t grid[3], int32_t n_batch,
                             int32_t channels, void* d_out, void* stream);

typedef enum { EMC2_POOL_MEAN = 0, EMC2_POOL_MAX = 1 } emc2_pool_mode;

/*
 * Multiscale Pooling of an image feature map into the cells of a voxel grid (paper Sec. 3.1: the data bridge
 * projects the relevant image pixels into 3D by their depth and pools them before fusion; Sec. 3.5: the
 * pooling size is a user parameter, here the cell size spec->vs; Fig. 5).
 *
 * Pixel (row j, col i) sits at (u, v) = (i, j), as in emc2_project_gather.  It is relevant iff its depth d
 * (distance along the optical axis, the w of the projection) is finite and > 0: the caller marks pixels outside
 * the proposal regions by a depth of 0.  Its position in the LiDAR frame is X = Q (d*u, d*v, d, 1), Q the 3x4
 * inverse of the projection: each row evaluated left to right in fp64 without fused multiply-add, rounded once
 * to fp32; its cell is the voxelizer's (t = fl(fl(X_a - lo_a) / vs_a), kept iff 0 <= t < G_a, cell floor(t)).
 * Every cell that receives a pixel becomes one output, in ascending key order:
 *   d_coords [capacity][4] int32 (batch_index, z, y, x);  d_counts [capacity] int32 pixels pooled (entries past
 *            the cell count may be zeroed);
 *   d_feats  [capacity][C] fp16: per channel the mean (fp32 sums, order not fixed, one rounding to fp16) or the
 *            maximum (exact) over the cell's pixels;
 *   d_n_cells device int32 (always written); h_n_cells host int32, NULL = no sync.
 *   d_img [H][W][C] fp16 with finite values, C a multiple of 8 in [8, 256]; d_depth [H][W] fp32; Q host float[12];
 *   H*W <= max_points.  Of spec only lo, vs, grid and n_batch are used (no range filter).
 * index_slot: receives the cell index of the produced set (as emc2_voxelize does), so a kernel map can be built
 * over the pooled cells directly.  EMC2_ERR_CAPACITY through the status word if more than `capacity` cells exist.
 */
emc2_status emc2_pool_image(emc2_ctx* ctx, const void* d_img, const float* d_depth, int32_t H, int32_t W, int32_t C,
                            const float Q[12], const emc2_voxel_spec* spec, int32_t batch_index, emc2_pool_mode mode,
                            int64_t capacity, int32_t* d_coords, void* d_feats, int32_t* d_counts, int32_t* d_n_cells,
                            int32_t* h_n_cells, int32_t index_slot, void* stream);

/*
 * Multimodal fusion of the LiDAR voxels with the pooled image cells of the same grid (paper Sec. 3.1; Fig. 5
 * caption: image features that share a voxel's 3D coordinate are concatenated with that voxel's features, the
 * others with zero-filled features).  The output is the union of the two site sets in ascending key order,
 *   d_feats_out[r] = [ LiDAR row or zeros (c_l) | image row or zeros (c_i) | zeros (c_out - c_l - c_i) ],
 * a voxel set like any other: its cell index is left in out_slot, so emc2_build_kmap can follow, and c_out may
 * pad the rows to a channel count the matrix-core convolution takes.
 *   d_coords_l [n_l][4], d_feats_l [n_l][c_l], d_n_l device count (likewise _i): each a set without repeated
 *   sites, in any order; coordinates outside the grid are ignored.  All features of `dtype`; c_l, c_i and c_out
 *   rows must be multiples of 4 bytes (16-byte multiples take the fast path).
 *   d_coords_out [capacity_out][4], d_feats_out [capacity_out][c_out]; d_src_l / d_src_i [capacity_out] int32 or
 *   NULL: the input row that feeds output row r, -1 where that half is zero-filled.
 *   d_n_out device int32 (always written); h_n_out host, NULL = no sync.
 * A copy: bit-exact in every dtype.  EMC2_ERR_CAPACITY through the status word if the union exceeds capacity_out.
 */
emc2_status emc2_fuse(emc2_ctx* ctx, emc2_dtype dtype, const int32_t* d_coords_l, const void* d_feats_l,
                      const int32_t* d_n_l, int64_t capacity_l, int32_t c_l, const int32_t* d_coords_i,
                      const void* d_feats_i, const int32_t* d_n_i, int64_t capacity_i, int32_t c_i,
                      const int32_t grid[3], int32_t n_batch, int32_t out_slot, int64_t capacity_out, int32_t c_out,
                      int32_t* d_coords_out, void* d_feats_out, int32_t* d_src_l, int32_t* d_src_i, int32_t* d_n_out,
                      int32_t* h_n_out, void* stream);

/*
 * Quantised sparse convolution (paper Sec. 3.6 (2): model quantisation is one of the deployment optimisations; the
 * paper gives no scheme, this one is the library's own):
 *   acc[o][c'] = sum_{k : nbr[k][o] >= 0} sum_c xq[nbr[k][o]][c] * wq[k][c][c']        int8 x int8 -> int32, exact
 *   v          = fl(fl((float)acc * mul[c']) + add[c'])                                 fp32, no fused multiply-add
 *   v          = max(v, 0) if relu
 *   out        = F16: v rounded to nearest even;  I8: clamp(rint(fl(v * inv_out_scale)), -127, 127), ties to even
 * mul[c'] carries input scale x weight scale x folded-BN scale, add[c'] the folded-BN shift: the caller folds them.
 *   d_in [n_in][Cin] int8; d_w_packed from emc2_pack_weights_i8 (d_w [27][Cin][Cout] int8 -> same byte size);
 *   d_mul, d_add [Cout] fp32; d_nbr, d_n_out, capacity_out, n_in_rows as for emc2_spconv (entries at or beyond
 *   n_in_rows are absent and reported); d_out [capacity_out][Cout] of out_dtype; d_in, d_w_packed, d_out 16-byte aligned.
 * Cin in {64, 128}, Cout in {32, 64} (emc2_spconv_i8_supported, a host-only query about this library's kernels with
 * no passage of the paper behind it; others EMC2_ERR_UNSUPPORTED).  Every step is
 * exact or individually rounded, so the result does not depend on the order of anything.
 * emc2_quantize_i8: q[i] = clamp(rint(fl((float)x[i] * inv_scale)), -127, 127) (NaN -> 0) for x of F32 or F16.
 */
int32_t emc2_spconv_i8_supported(int32_t cin, int32_t cout);
emc2_status emc2_quantize_i8(emc2_ctx* ctx, emc2_dtype dtype, const void* d_x, int64_t n, float inv_scale, int8_t* d_q,
                             void* stream);
emc2_status emc2_pack_weights_i8(emc2_ctx* ctx, const int8_t* d_w, int32_t cin, int32_t cout, void* d_packed, void* stream);
emc2_status emc2_spconv_i8(emc2_ctx* ctx, const int8_t* d_in, const void* d_w_packed, const float* d_mul,
                           const float* d_add, int32_t relu, emc2_dtype out_dtype, float inv_out_scale,
                           const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int64_t n_in_rows, int32_t cin,
                           int32_t cout, void* d_out, void* stream);

/*
 * The same quantised convolution with 8-bit floating-point operands (paper Sec. 3.6 (2) again; the scheme is the
 * library's own).  Format: E4M3 -- 1 sign, 4 exponent (bias 7), 3 mantissa bits, no infinities, largest value 448,
 * the two codes with all exponent and mantissa bits set are not numbers and must not occur in the operands.
 *   acc[o][c'] = sum_{k : nbr[k][o] >= 0} sum_c value(xq[nbr[k][o]][c]) * value(wq[k][c][c'])   products exact, sums fp32
 *   v          = fl(fl(acc * mul[c']) + add[c']);  v = max(v, 0) if relu;  out = v as F32, or rounded to F16
 * The products are exact; the accumulation is the matrix cores' own (the 32 products of one instruction are aligned
 * to the largest before they are added, which drops low bits), so the result agrees with the exactly accumulated one
 * to a few 1e-4 of the output's magnitude when the operands span the format's range, and exactly when every partial
 * sum is a small integer.
 *   d_in [n_in][Cin] uint8 codes; d_w_packed: the [27][Cin][Cout] codes re-ordered by emc2_pack_weights_i8 (a byte
 *   permutation, whatever the bytes encode); shapes, d_nbr, d_n_out, capacity_out, n_in_rows, alignment as for
 *   emc2_spconv_i8.
 * emc2_quantize_e4m3: q[i] = the finite code nearest to fl((float)x[i] * inv_scale), ties to the even code, beyond 448
 * (and infinities) saturating, NaN -> 0, zero always +0; x of F32 or F16.  Exact (byte results).
 */
emc2_status emc2_quantize_e4m3(emc2_ctx* ctx, emc2_dtype dtype, const void* d_x, int64_t n, float inv_scale, uint8_t* d_q,
                               void* stream);
emc2_status emc2_spconv_e4m3(emc2_ctx* ctx, const uint8_t* d_in, const void* d_w_packed, const float* d_mul,
                             const float* d_add, int32_t relu, emc2_dtype out_dtype, const int32_t* d_nbr,
                             const int32_t* d_n_out, int64_t capacity_out, int64_t n_in_rows, int32_t cin, int32_t cout,
                             void* d_out, void* stream);

typedef enum { EMC2_EXPERT_LPE = 0, EMC2_EXPERT_VEE = 1, EMC2_EXPERT_APE = 2 } emc2_expert;

/*
 * Scenario-Adaptive Dispatcher (paper Sec. 3.2): the expert of every scene of a batch, from the distance and the
 * confidence of its proposal regions, and the scenes grouped by expert.
 *   d_props [n_props][4] fp32 (x, y, z, confidence) of each proposal region; d_scene [n_props] int32 its scene,
 *   or NULL (all in scene 0); ids outside [0, n_scenes) are ignored.
 *   A proposal is "far" unless fl(fl(x*x) + fl(y*y)) < fl(dist*dist) (range in the ground plane, fp32), "unclear"
 *   unless confidence >= conf; a NaN therefore counts as far / unclear.
 *     EMC2_EXPERT_APE (accuracy-prioritised): some proposal of the scene is far and unclear;
 *     EMC2_EXPERT_VEE (versatile efficiency): otherwise, some proposal is near and unclear, or far and clear;
 *     EMC2_EXPERT_LPE (latency-prioritised):  otherwise (all near and clear; also a scene without proposals).
 *   d_expert [n_scenes] int32; d_counts [3] int32 scenes per expert; d_order [n_scenes] int32: scene indices grouped
 *   by expert (LPE, VEE, APE), ascending within a group: expert e runs on d_order[sum(counts[:e]) ...][counts[e]].
 *   dist >= 0 (the paper uses 23.5 m and 35 m); 1 <= n_scenes <= 2^20.  Integer results, exact.
 */
emc2_status emc2_dispatch(emc2_ctx* ctx, const float* d_props, const int32_t* d_scene, int64_t n_props,
                          int32_t n_scenes, float dist, float conf, int32_t* d_expert, int32_t* d_counts,
                          int32_t* d_order, void* stream);

/*
 * Expert-grouped batching (paper Sec. 3.2: the dispatcher routes every scene to one expert, so each expert's
 * network runs on the scenes routed to it).  From emc2_dispatch's outputs, the batch ids that make emc2_voxelize
 * build expert `expert`'s batch out of a mixed batch of points:
 *   d_slot [n_scenes] int32 (written for every scene): the scene's position inside its own expert's group, i.e. its
 *          index in d_order minus the sizes of the groups before its expert's;
 *   d_group_batch [n_points] int32: d_slot[scene] for a point whose scene runs on `expert`, else -1 (a batch id
 *          emc2_voxelize drops), also for a scene id outside [0, n_scenes).
 *   d_scene [n_points] int32 scene of each point, or NULL (all in scene 0); d_expert, d_order, d_counts as written
 *   by emc2_dispatch for the same n_scenes.  Voxelizing with d_batch = d_group_batch and n_batch = n_scenes (or
 *   the group's size, if the host knows it) yields the group's scenes as frames 0 .. count-1 in ascending scene
 *   order.  Integer results, exact.
 */
emc2_status emc2_group_points(emc2_ctx* ctx, const int32_t* d_scene, int64_t n_points, const int32_t* d_expert,
                              const int32_t* d_order, const int32_t* d_counts, int32_t n_scenes, int32_t expert,
                              int32_t* d_slot, int32_t* d_group_batch, void* stream);

/*
 * Point -> image projection with bilinear feature gather (paper Sec. 3.1: image features are
 * aligned with 3D positions for fusion; Fig. 5 caption: sites without a match get zero-filled
 * features).
 *   (U, V, w) = P (x, y, z, 1) in fp64, u = U/w, v = V/w; valid iff w > 0, 0 <= u <= W-1,
 *   0 <= v <= H-1.  Pixel (row j, col i) sits at (u, v) = (i, j).  The four neighbours
 *   (floor and floor+1, clamped to the last row/col) are blended in fp32 and rounded once to fp16.
 *   Invalid points get an all-zero row and valid = 0.
 *   d_points [n][stride_f] fp32; P host float[12] row-major 3x4; d_img [H][W][C] fp16, C even and
 *   <= 1024; d_out [n][C] fp16; d_valid [n] uint8; d_uv [n][2] fp32 or NULL.
 */
emc2_status emc2_project_gather(emc2_ctx* ctx, const float* d_points, int32_t stride_f,
                                int64_t n_points, const float P[12], const void* d_img, int32_t H,
                                int32_t W, int32_t C, void* d_out, uint8_t* d_valid, float* d_uv,
                                void* stream);

#ifdef __cplusplus
}
#endif
#endif /* EMC2_H_ */
