// Output-stationary implicit gather-GEMM sparse convolution on the CDNA4 matrix cores
// (paper Sec. 3.5: 3D sparse convolution over non-empty voxels is where inference time goes;
// Sec. 3.6: segment-wise overlap of data movement with compute, and operator fusion).
//
// GEMM view per tap k:  out[M = output voxels][N = Cout] += X_k[M][K = Cin] * W_k[K][N],
// where row m of X_k is the feature row of the input voxel nbr[k][o_m] (zero if absent).
//
// Tiling (64-wide wavefronts, v_mfma_f32_32x32x16_{f16,bf16}):
//   - a block is 4 waves; each wave owns MT*32 consecutive output rows and ALL Cout columns, so the
//     fp32 accumulators never leave registers and no output atomics are needed;
//   - gather: CIN/8 consecutive lanes fetch one whole feature row with 16-byte loads, so a load
//     instruction asks for full cache lines (8 rows of 128 B at Cin = 64) instead of 32 partial ones;
//     the rows of a tap go registers -> a wave-private, padded LDS tile, and the A operand (lane =
//     row, 8 consecutive input channels) is one ds_read_b128 from that tile.  Loads run several taps ahead
//     of the MFMAs that consume them; the 27 kernel-map entries of a row are fetched up front;
//   - B operand: weights are pre-packed in fragment order (one 16-byte piece per lane and fragment),
//     copied to LDS once per block and tap with 16-byte accesses, double buffered so the copy of
//     tap k+1 overlaps the MFMAs of tap k; a fragment read is one conflict-free ds_read_b128;
//   - absent neighbours contribute zero rows (masked when the A operand is read); the whole tap loop
//     is branch-free so that the compiler can count the loads in flight exactly;
//   - epilogue: acc*scale+shift, ReLU, convert, store.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "common.h"
#include "spconv_mfma.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
// Native 16-byte vector: values staged in registers must be real loads and stores.  (Copies of the HIP
// struct type uint4 become memcpy calls that the optimizer forwards from global memory to the later
// LDS store, which silently turns a prefetch into a late load.)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <int DT> struct Mma;
template <> struct Mma<EMC2_F16> {
  static __device__ __forceinline__ floatx16 run(u32x4 a, u32x4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float v) { return __half_as_ushort(__float2half_rn(v)); }
};
template <> struct Mma<EMC2_BF16> {
  static __device__ __forceinline__ floatx16 run(u32x4 a, u32x4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float v) {
    return __builtin_bit_cast(uint16_t, __float2bfloat16(v));
  }
};

constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;

// Packed weight layout: piece index ((k*KS + t)*NT + j)*64 + lane, lane = 32*h + n, holds the 8 values
// W[k][16t + 8h + e][32j + n], e = 0..7 -- exactly the B operand of k-step t, column tile j.
__global__ void __launch_bounds__(256) k_pack_weights(const uint16_t* __restrict__ w, int cin, int cout,
                                                      uint4* __restrict__ packed) {
  const int ks = cin / 16, nt = cout / 32;
  const int total = 27 * ks * nt * 64;
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= total) return;
  const int lane = p & 63;
  int f = p >> 6;
  const int j = f % nt; f /= nt;
  const int t = f % ks; f /= ks;
  const int k = f;
  const int n = 32 * j + (lane & 31);
  const int c0 = 16 * t + 8 * (lane >> 5);
  const uint16_t* src = w + ((int64_t)k * cin + c0) * cout + n;
  uint32_t v[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
    v[e] = (uint32_t)src[(2 * e) * cout] | ((uint32_t)src[(2 * e + 1) * cout] << 16);
  packed[p] = make_uint4(v[0], v[1], v[2], v[3]);
}

// Pipeline depths.  Global-memory latency on this part is of the order of a microsecond while one
// tap of MFMA work for a wave is a few hundred cycles, so everything a tap needs is requested
// well ahead: D taps of gathered rows and WD taps of weights are in flight per wave, kernel-map
// entries are fetched two (dz,dy) groups (six taps) ahead.  The 27 taps run as 9 groups of 3 so
// that every register set is named by a compile-time constant (tap % 3) inside the unrolled group.
template <int CIN, int COUT> struct Pipe {
  static constexpr int D = CIN <= 64 ? 3 : 1;                     // 1 or 3
  static constexpr int WD = (CIN * COUT <= 64 * 64) ? 3 : 1;      // 1 or 3
  static constexpr int NB = WD == 3 ? 3 : 2;                      // weight buffers in LDS
  // waves per SIMD the register allocator must leave room for (2 where LDS also lets two blocks share a CU)
  static constexpr int MINW = (CIN <= 64 && COUT <= 64) ? 2 : 1;
  // skip the LDS and matrix work of a tap at which none of the wave's 64 rows has a neighbour: measured to
  // pay only where a tap is expensive (Cin = 64) and the accumulators live in ordinary VGPRs (MINW = 2)
  static constexpr bool SKIP = (CIN == 64 && COUT <= 64);
};

template <int DT, int CIN, int COUT, int MT>
__global__ void __launch_bounds__(kThreads, (Pipe<CIN, COUT>::MINW)) k_spconv_mfma(const uint16_t* __restrict__ in, const u32x4* __restrict__ wp,
                                                          const float* __restrict__ scale, const float* __restrict__ shift,
                                                          int epilogue, const int32_t* __restrict__ nbr,
                                                          const int32_t* __restrict__ d_n_out, int64_t capacity_out,
                                                          int32_t n_in, int32_t* __restrict__ dev_flags,
                                                          uint16_t* __restrict__ out) {
  static_assert(MT == 2, "a wave owns 64 rows: one kernel-map entry per lane and tap");
  constexpr int KS = CIN / 16;                // k-steps per tap
  constexpr int NT = COUT / 32;               // 32-column tiles
  constexpr int W16 = KS * NT * 64;           // 16-byte weight pieces per tap
  constexpr int WPT = (W16 + kThreads - 1) / kThreads;
  // a tap with fewer pieces than threads (W16 = 64 or 128) is copied redundantly by the surplus threads
  // (same values to the same place) rather than under a branch
  constexpr int WMASK = (W16 >= kThreads) ? 0x7fffffff : (W16 - 1);
  static_assert(W16 % kThreads == 0 || (W16 & (W16 - 1)) == 0, "piece count must tile the block or be a power of two");
  constexpr int R = 32 * MT;                  // rows per wave
  constexpr int CH = CIN / 8;                 // 16-byte chunks per feature row
  constexpr int RPI = 64 / CH;                // rows covered by one staging load instruction
  constexpr int NI = R / RPI;                 // staging load instructions per tap
  // LDS tile layout, in 16-byte units.  The LDS serves a 16-byte write instruction 8 lanes at a time over
  // 32 banks and a 16-byte read 16 lanes at a time over 64 banks.  Rows of 128 bytes or more get one unit
  // of padding (8 lanes write half a row or more; 16 lanes read one piece of 16 consecutive rows: distinct
  // banks).  Shorter rows are stored unpadded with their pieces XOR-swizzled by the row number: padding
  // would make the 2 or 4 rows that 8 lanes write overlap modulo 32 banks.
  constexpr bool SWZ = CH <= 4;
  constexpr int ROW16 = SWZ ? CH : CH + 1;
  constexpr int SWSH = CH == 4 ? 2 : 3;       // swizzle key of row r: (r >> SWSH) & (CH - 1)
  constexpr int D = Pipe<CIN, COUT>::D;
  constexpr int WD = Pipe<CIN, COUT>::WD;
  constexpr int NB = Pipe<CIN, COUT>::NB;
  __shared__ u32x4 wl[NB][W16];
  // wave-private tiles: gathered rows of a tap; at the end, 32 output rows at a time on their way to memory
  constexpr int TILE16 = (R * ROW16 > 32 * (COUT / 8 + 1)) ? R * ROW16 : 32 * (COUT / 8 + 1);
  __shared__ u32x4 tile[kWaves][TILE16];

  int64_t n_out = *d_n_out;
  if (n_out > capacity_out) n_out = capacity_out;
  // XCD-aware tile assignment: workgroups are dealt round-robin to the 8 XCDs (each with its own L2), so
  // workgroup b runs on XCD b % 8.  Giving XCD x the contiguous tile range [x*chunk, (x+1)*chunk) keeps
  // spatially adjacent tiles -- which gather largely the same input rows -- behind one L2.
  const int64_t n_tiles = (n_out + kWaves * R - 1) / (kWaves * R);
  const int64_t chunk = (n_tiles + 7) / 8;
  const int64_t slot_in_xcd = blockIdx.x / 8;
  const int64_t tile_id = (int64_t)(blockIdx.x % 8) * chunk + slot_in_xcd;
  if (slot_in_xcd >= chunk || tile_id >= n_tiles) return;  // uniform for the block
  const int64_t block_row0 = tile_id * (kWaves * R);

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int m = lane & 31, h = lane >> 5;
  const int64_t wave_row0 = block_row0 + (int64_t)wave * R;
  u32x4* my_tile = tile[wave];

  // lane l holds the kernel-map entries of row l of this wave's 64 rows
  const bool live = wave_row0 + lane < n_out;
  const int32_t* nrow = nbr + (live ? wave_row0 + lane : 0);
  const int32_t dead = live ? 0 : -1;   // OR-ed into kernel-map entries: rows past n_out have no neighbours
  unsigned long long oob = 0ull;        // lanes that saw an entry outside [0, n_in)
  const int srow = lane / CH, schunk = lane % CH;   // staging role: row within an instruction, 16-byte chunk

  floatx16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mt][j][e] = 0.f;

  int32_t jq[3][3];         // kernel-map entries of groups g, g+1, g+2
  u32x4 sreg[D][NI];        // gathered rows in flight; tap x lives in set x % D
  u32x4 wq[WD][WPT];        // weights in flight;       tap x lives in set x % WD

  // Every load below is issued unconditionally (addresses are clamped, results are masked afterwards):
  // a load under a branch may or may not have been issued, so the compiler could no longer count the
  // loads in flight and would wait for all of them (vmcnt(0)) at the first use, undoing the pipeline.
#define EMC2_IDX_LOAD(GROUP, DST)                                                                        \
  _Pragma("unroll") for (int kx_ = 0; kx_ < 3; ++kx_) {                                                  \
    /* raw value; rows past n_out and groups past the last one are masked where the entry is used */  \
    jq[DST][kx_] = nrow[(int64_t)(3 * ((GROUP) < 9 ? (GROUP) : 8) + kx_) * capacity_out];                \
  }
#define EMC2_STAGE_LOAD(JROW, SET)                                                                       \
  _Pragma("unroll") for (int i_ = 0; i_ < NI; ++i_) {                                                    \
    const int32_t j_ = __shfl((JROW), i_ * RPI + srow, 64);                                              \
    sreg[SET][i_] = *(reinterpret_cast<const u32x4*>(in + (int64_t)(j_ >= 0 ? j_ : 0) * CIN) + schunk);  \
  }
#define EMC2_W_LOAD(TAP, SET)                                                                            \
  {                                                                                                      \
    const u32x4* wsrc_ = wp + (int64_t)(TAP) * W16;                                                      \
    _Pragma("unroll") for (int i_ = 0; i_ < WPT; ++i_) {                                                 \
      const int p_ = (threadIdx.x + i_ * kThreads) & WMASK;                                              \
      wq[SET][i_] = wsrc_[p_];                                                                           \
    }                                                                                                    \
  }
#define EMC2_W_STORE(BUF, SET)                                                                           \
  _Pragma("unroll") for (int i_ = 0; i_ < WPT; ++i_) {                                                   \
    const int p_ = (threadIdx.x + i_ * kThreads) & WMASK;                                                \
    wl[BUF][p_] = wq[SET][i_];                                                                           \
  }

  // prologue: map entries of groups 0..2; weights of tap 0 to LDS, of taps 1..WD-1 to registers;
  // gathers of taps 0..D-1
  EMC2_IDX_LOAD(0, 0)
  EMC2_IDX_LOAD(1, 1)
  EMC2_IDX_LOAD(2, 2)
  EMC2_W_LOAD(0, 0)
  EMC2_W_STORE(0, 0)
  if constexpr (WD == 3) {
    EMC2_W_LOAD(1, 1)
    EMC2_W_LOAD(2, 2)
  }
  EMC2_STAGE_LOAD(emc2_entry(jq[0][0], dead, n_in, oob), 0)
  if constexpr (D == 3) {
    EMC2_STAGE_LOAD(emc2_entry(jq[0][1], dead, n_in, oob), 1)
    EMC2_STAGE_LOAD(emc2_entry(jq[0][2], dead, n_in, oob), 2)
  }
  __syncthreads();

  for (int g = 0; g < 9; ++g) {
    // kernel-map entries of group g + 3, requested a whole group before anything (even the queue rotation
    // below) touches them
    int32_t jn[3];
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) jn[kx] = nrow[(int64_t)(3 * (g + 3 < 9 ? g + 3 : 8) + kx) * capacity_out];
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
      const int tap = 3 * g + kx;
      const unsigned long long mask = __ballot(emc2_entry(jq[0][kx], dead, n_in, oob) >= 0);
      // weights of tap + WD: global -> registers (the set was emptied at the end of the previous tap)
      EMC2_W_LOAD(tap + WD < 27 ? tap + WD : 26, kx % WD)
      // gathered rows of this tap: registers -> wave-private LDS tile
      // a tap at which none of the wave's 64 rows has a neighbour does no LDS or matrix work at all; the
      // loads stay unconditional (see above), only their use is skipped (wave-uniform branch)
      if (!Pipe<CIN, COUT>::SKIP || mask != 0ull) {
#pragma unroll
        for (int i = 0; i < NI; ++i) my_tile[(i * RPI + srow) * ROW16 + (SWZ ? (schunk ^ (((i * RPI + srow) >> SWSH) & (CH - 1))) : schunk)] = sreg[kx % D][i];
      }
      // the freed register set takes the gather of tap + D (absent entries re-read row 0 and are masked)
      const int32_t past = g < 8 ? 0 : -1;   // entries of "group 9" do not exist
      if constexpr (D == 3) {
        EMC2_STAGE_LOAD(emc2_entry(jq[1][kx], dead | past, n_in, oob), kx)
      } else {
        if (kx < 2) { EMC2_STAGE_LOAD(emc2_entry(jq[0][kx < 2 ? kx + 1 : 0], dead, n_in, oob), 0) } else { EMC2_STAGE_LOAD(emc2_entry(jq[1][0], dead | past, n_in, oob), 0) }
      }
      __builtin_amdgcn_wave_barrier();
      const u32x4* wb = wl[tap % NB];
      if (!Pipe<CIN, COUT>::SKIP || mask != 0ull) {
        // no per-tile branches inside: with finer-grained conditions around the MFMAs the compiler starts
        // copying accumulators between register classes on every tap
        const bool v0 = (mask >> m) & 1ull, v1 = (mask >> (32 + m)) & 1ull;
#pragma unroll
        for (int t = 0; t < KS; ++t) {
          u32x4 b[NT];
#pragma unroll
          for (int j = 0; j < NT; ++j) b[j] = wb[(t * NT + j) * 64 + lane];
          const int ca = SWZ ? ((2 * t + h) ^ ((m >> SWSH) & (CH - 1))) : 2 * t + h;   // rows m and 32 + m share a key
          u32x4 a0 = my_tile[m * ROW16 + ca];
          u32x4 a1 = my_tile[(32 + m) * ROW16 + ca];
          a0 = v0 ? a0 : u32x4{0u, 0u, 0u, 0u};
          a1 = v1 ? a1 : u32x4{0u, 0u, 0u, 0u};
#pragma unroll
          for (int j = 0; j < NT; ++j) {
            acc[0][j] = Mma<DT>::run(a0, b[j], acc[0][j]);
            acc[1][j] = Mma<DT>::run(a1, b[j], acc[1][j]);
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
      // weights of tap + 1: registers -> LDS ring; one barrier per tap publishes them and retires
      // the buffer read NB - 1 taps ago
      EMC2_W_STORE((tap + 1) % NB, (kx + 1) % WD)  // after the last tap this rewrites a buffer nobody reads
      __syncthreads();
    }
    // rotate the kernel-map queue
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
      jq[0][kx] = jq[1][kx];
      jq[1][kx] = jq[2][kx];
      jq[2][kx] = jn[kx];
    }
  }
#undef EMC2_IDX_LOAD
#undef EMC2_STAGE_LOAD
#undef EMC2_W_LOAD
#undef EMC2_W_STORE
  emc2_report_oob(oob, dev_flags);

  // epilogue: lane holds column n = 32*j + m; acc element e <-> row 8*(e/4) + 4*h + (e%4).
  // Scale/shift/ReLU/convert in registers, then each 32-row tile goes through the wave's LDS tile so that
  // the global stores are whole 16-byte pieces of consecutive rows (a lane-per-column store would write 2
  // bytes per lane and take as long as several taps).
  float sc[NT], sh[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    sc[j] = (epilogue != EMC2_EPI_NONE) ? scale[32 * j + m] : 1.f;
    sh[j] = (epilogue != EMC2_EPI_NONE) ? shift[32 * j + m] : 0.f;
  }
  uint16_t* otile = reinterpret_cast<uint16_t*>(my_tile);
  constexpr int OCH = COUT / 8;               // 16-byte pieces per output row
  constexpr int OPITCH = (OCH + 1) * 8;       // LDS row pitch in 16-bit units (one piece of padding)
  constexpr int ORPI = 64 / OCH;              // rows one store instruction covers
  const int orow = lane / OCH, ochunk = lane % OCH;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float v = acc[mt][j][e];
        if (epilogue != EMC2_EPI_NONE) v = fmaf(v, sc[j], sh[j]);
        if (epilogue == EMC2_EPI_AFFINE_RELU) v = v > 0.f ? v : 0.f;
        otile[(8 * (e / 4) + 4 * h + (e % 4)) * OPITCH + 32 * j + m] = Mma<DT>::cvt(v);
      }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < 32 / ORPI; ++i) {
      const int r = i * ORPI + orow;
      const u32x4 piece = *reinterpret_cast<const u32x4*>(otile + r * OPITCH + ochunk * 8);
      const int64_t o = wave_row0 + mt * 32 + r;
      if (o < n_out) *reinterpret_cast<u32x4*>(out + o * COUT + ochunk * 8) = piece;
    }
    __builtin_amdgcn_wave_barrier();
  }
}

template <int DT, int CIN, int COUT>
void launch(const void* d_in, const void* d_wp, const float* d_scale, const float* d_shift, int epilogue,
            const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int32_t n_in, int32_t* dev_flags,
            void* d_out, hipStream_t s) {
  constexpr int MT = 2;
  const int64_t rows_per_block = kWaves * MT * 32;
  hipLaunchKernelGGL((k_spconv_mfma<DT, CIN, COUT, MT>), dim3((unsigned)(emc2_div_up(capacity_out, rows_per_block) + 8)),  // + 8: the per-XCD ranges round up
                     dim3(kThreads), 0, s, (const uint16_t*)d_in, (const u32x4*)d_wp, d_scale, d_shift, epilogue, d_nbr,
                     d_n_out, capacity_out, n_in, dev_flags, (uint16_t*)d_out);
}

template <int DT>
void dispatch(const void* d_in, const void* d_wp, const float* d_scale, const float* d_shift, int epilogue,
              const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int32_t n_in, int32_t* dev_flags, int cin,
              int cout, void* d_out, hipStream_t s) {
#define CASE(CI, CO)                                                                                              \
  if (cin == CI && cout == CO) {                                                                                  \
    launch<DT, CI, CO>(d_in, d_wp, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, n_in, dev_flags,     \
                       d_out, s);                                                                                 \
    return;                                                                                                       \
  }
  CASE(16, 32) CASE(32, 32) CASE(32, 64) CASE(64, 64) CASE(64, 128) CASE(128, 128)
  CASE(16, 64) CASE(32, 128) CASE(64, 32) CASE(128, 64) CASE(128, 32) CASE(16, 128)
#undef CASE
}

}  // namespace

bool emc2_spconv_mfma_supported(int cin, int cout) {
  const bool ci = cin == 16 || cin == 32 || cin == 64 || cin == 128;
  const bool co = cout == 32 || cout == 64 || cout == 128;
  return ci && co;
}

void emc2_spconv_mfma_pack(const void* d_w, int cin, int cout, void* d_packed, hipStream_t stream) {
  const int total = 27 * (cin / 16) * (cout / 32) * 64;
  hipLaunchKernelGGL(k_pack_weights, dim3((unsigned)emc2_div_up(total, 256)), dim3(256), 0, stream, (const uint16_t*)d_w, cin,
                     cout, (uint4*)d_packed);
}

void emc2_spconv_mfma_launch(emc2_dtype dtype, const void* d_in, const void* d_wp, const float* d_scale,
                             const float* d_shift, int epilogue, const int32_t* d_nbr, const int32_t* d_n_out,
                             int64_t capacity_out, int32_t n_in, int32_t* dev_flags, int cin, int cout, void* d_out,
                             hipStream_t stream) {
  if (dtype == EMC2_F16)
    dispatch<EMC2_F16>(d_in, d_wp, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, n_in, dev_flags, cin, cout,
                       d_out, stream);
  else
    dispatch<EMC2_BF16>(d_in, d_wp, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, n_in, dev_flags, cin, cout,
                        d_out, stream);
}
