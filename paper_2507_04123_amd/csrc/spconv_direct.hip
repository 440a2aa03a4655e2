// Register-direct MFMA sparse convolution (paper Sec. 3.5 sparse convolution over the non-empty voxels;
// Sec. 3.6 operator fusion).
//
// Measured on this part, the local data share serves a wave's 16-byte read in ~8 cycles and a 16-byte
// write in ~15, per CU, whatever the occupancy.  A gather-GEMM that stages the gathered rows in LDS
// (write the tile, read it back as the A operand, read the weights as the B operand) then spends more
// LDS cycles per tap than matrix-core cycles, and that -- not memory latency, not the matrix cores --
// bounds it.  This kernel keeps the gathered rows out of LDS altogether:
//
//   v_mfma_f32_16x16x32_{f16,bf16}: the A operand of lane (m = lane % 16, q = lane / 16) is the 8
//   consecutive input channels 8q .. 8q+7 of row m of the tile, i.e. 16 contiguous bytes of the feature
//   row nbr[k][o_m].  Four lanes cover 64 contiguous bytes of one row, so a single global_load_dwordx4
//   per (16-row tile, 32 channels) IS the A operand: global -> VGPR -> matrix core, nothing in between.
//   Absent neighbours read a zeroed row instead (an address select, no masking of data).
//
// LDS holds only the weights of the current and the next tap (packed in B-fragment order, copied once
// per block and tap, requested three taps ahead) and a small tile for the epilogue's transposition.
//
// A block is 4 waves; a wave owns 32 consecutive output rows (2 tiles of 16; 64 rows = 4 tiles at 32 -> 32, where
// the accumulators are few) and all Cout columns, so the fp32 accumulators never leave registers.  Gathers run 3
// taps ahead of their use; kernel-map entries two (dz,dy) groups ahead.  Every load is unconditional so the
// compiler can count the loads in flight.  Shapes: Cin, Cout in {32, 64}, and 64 -> 128 / 128 -> 128, where a
// tap's matrix work per gathered byte doubles and the kernel leaves the staged per-tap kernel behind by a third.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "common.h"
#include "spconv_mfma.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vector: real loads and stores
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <int DT> struct MmaD;
template <> struct MmaD<EMC2_F16> {
  static __device__ __forceinline__ floatx4 run(u32x4 a, u32x4 b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float v) { return __half_as_ushort(__float2half_rn(v)); }
};
template <> struct MmaD<EMC2_BF16> {
  static __device__ __forceinline__ floatx4 run(u32x4 a, u32x4 b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float v) { return __builtin_bit_cast(uint16_t, __float2bfloat16(v)); }
};

constexpr int kDWaves = 4;
constexpr int kDThreads = kDWaves * 64;

// Packed weight layout of this kernel: piece index ((k*KS + t)*NT + j)*64 + lane, lane = 16*q + n, holds the
// 8 values W[k][32t + 8q + e][16j + n], e = 0..7 -- the B operand of k-step t, column tile j.
__global__ void __launch_bounds__(256) k_pack_weights_direct(const uint16_t* __restrict__ w, int cin, int cout,
                                                             uint4* __restrict__ packed) {
  const int ks = cin / 32, nt = cout / 16;
  const int total = 27 * ks * nt * 64;
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= total) return;
  const int lane = p & 63;
  int f = p >> 6;
  const int j = f % nt; f /= nt;
  const int t = f % ks; f /= ks;
  const int k = f;
  const int n = 16 * j + (lane & 15);
  const int c0 = 32 * t + 8 * (lane >> 4);
  const uint16_t* src = w + ((int64_t)k * cin + c0) * cout + n;
  uint32_t v[4];
#pragma unroll
  for (int e = 0; e < 4; ++e)
    v[e] = (uint32_t)src[(2 * e) * cout] | ((uint32_t)src[(2 * e + 1) * cout] << 16);
  packed[p] = make_uint4(v[0], v[1], v[2], v[3]);
}

template <int CIN, int COUT> struct DirectCfg {
  // 16-row tiles per wave (2 or 4): fewer rows per wave mean fewer accumulators and operands in flight, so more
  // waves fit a SIMD and cover each other's stalls; more rows per wave reuse a weight fragment read more often
  static constexpr int MT = (CIN <= 32 && COUT <= 32) ? 4 : 2;
  // waves per SIMD the register allocator must leave room for (the 128-channel shapes keep 64-128 accumulators
  // and as many operands in flight)
  // (128 -> 128 ends up at one wave per SIMD whatever is asked for here -- 83 KB of LDS, 360 registers -- and the
  // compiler says so in a warning; asking for one outright, or forcing two with a shorter weight prefetch, were
  // both measured slower)
  static constexpr int MINW = (CIN >= 128 || COUT >= 128) ? 2 : 3;
};

template <int DT, int CIN, int COUT>
__global__ void __launch_bounds__(kDThreads, (DirectCfg<CIN, COUT>::MINW))
k_spconv_direct(const uint16_t* __restrict__ in, const u32x4* __restrict__ wp, const float* __restrict__ scale,
                const float* __restrict__ shift, int epilogue, const int32_t* __restrict__ nbr,
                const int32_t* __restrict__ d_n_out, int64_t capacity_out, int32_t n_in, int32_t* __restrict__ dev_flags,
                const uint16_t* __restrict__ zrow, uint16_t* __restrict__ out) {
  constexpr int KS = CIN / 32;                // k-steps per tap
  constexpr int NT = COUT / 16;               // 16-column tiles
  constexpr int MT = DirectCfg<CIN, COUT>::MT;   // 16-row tiles per wave
  constexpr int R = 16 * MT;                  // rows per wave
  static_assert(MT == 2 || MT == 4, "the lane-swap broadcast below handles 2 or 4 tiles");
  constexpr int W16 = KS * NT * 64;           // 16-byte weight pieces per tap
  constexpr int WPT = (W16 + kDThreads - 1) / kDThreads;
  static_assert((W16 & (W16 - 1)) == 0, "piece count is a power of two");
  // a tap with fewer pieces than threads is copied redundantly by the surplus threads (same values to the
  // same place) rather than under a branch
  constexpr int WMASK = W16 - 1;
  constexpr int NA = MT * KS;                 // A-operand loads per tap
  constexpr int OCH = COUT / 8;               // 16-byte pieces per output row
  constexpr int OPITCH = (OCH + 1) * 8;       // epilogue tile row pitch in 16-bit units
  __shared__ u32x4 wl[2][W16];
  __shared__ u32x4 otile_s[kDWaves][16 * (OCH + 1)];

  int64_t n_out = *d_n_out;
  if (n_out > capacity_out) n_out = capacity_out;
  // XCD-aware tile assignment: workgroup b runs on XCD b % 8; XCD x takes a contiguous range of tiles
  const int64_t n_tiles = (n_out + kDWaves * R - 1) / (kDWaves * R);
  const int64_t chunk = (n_tiles + 7) / 8;
  const int64_t slot_in_xcd = blockIdx.x / 8;
  const int64_t tile_id = (int64_t)(blockIdx.x % 8) * chunk + slot_in_xcd;
  if (slot_in_xcd >= chunk || tile_id >= n_tiles) return;  // uniform for the block

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int m = lane & 15, q = lane >> 4;
  const int64_t wave_row0 = tile_id * (kDWaves * R) + (int64_t)wave * R;

  // lane l holds the kernel-map entries of row l % R of this wave's R rows
  const bool live = wave_row0 + (lane % R) < n_out;
  const int32_t* nrow = nbr + (live ? wave_row0 + (lane % R) : 0);
  const int32_t dead = live ? 0 : -1;   // OR-ed into kernel-map entries: rows past n_out have no neighbours
  unsigned long long oob = 0ull;        // lanes that saw an entry outside [0, n_in)

  floatx4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[mt][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  int32_t jq[3][3];         // kernel-map entries of groups g, g+1, g+2 (as loaded; masked where used)
  u32x4 areg[3][NA];        // A operands in flight; tap x lives in set x % 3
  u32x4 wq[3][WPT];         // weights in flight; tap x lives in set x % 3

#define EMC2_IDX_LOAD(GROUP, DST)                                                                        \
  _Pragma("unroll") for (int kx_ = 0; kx_ < 3; ++kx_)                                                    \
      jq[DST][kx_] = nrow[(int64_t)(3 * ((GROUP) < 9 ? (GROUP) : 8) + kx_) * capacity_out];
  // A operands of one tap: tile mt, k-step ks <- 16 bytes at channel 32*ks + 8*q of row JROW[16*mt + m]
  // The entries of rows 16*mt .. 16*mt+15 sit in lanes 16*mt .. 16*mt+15; every lane needs the one of its
  // column m for each mt.  Three lane-swap instructions broadcast each 16-lane row to all four rows (no LDS
  // round trip: a ds_bpermute per tile costs a serialized ~120-cycle wait each).
#define EMC2_A_LOAD(JROW, SET)                                                                           \
  {                                                                                                      \
    const uint32_t jr_ = (uint32_t)(JROW);                                                               \
    /* R = 64: lane rows are 0123 -> 0101 | 2323;  R = 32: they already are 0101 */                      \
    u32x2 h_ = {jr_, jr_};                                                                               \
    if constexpr (MT == 4) h_ = __builtin_amdgcn_permlane32_swap(jr_, jr_, false, false);                \
    const u32x2 lo_ = __builtin_amdgcn_permlane16_swap(h_[0], h_[0], false, false);  /* 0000 | 1111 */   \
    const u32x2 hi_ = __builtin_amdgcn_permlane16_swap(h_[1], h_[1], false, false);  /* 2222 | 3333 */   \
    const int32_t jm_[4] = {(int32_t)lo_[0], (int32_t)lo_[1], (int32_t)hi_[0], (int32_t)hi_[1]};         \
  _Pragma("unroll") for (int mt_ = 0; mt_ < MT; ++mt_) {                                                 \
    const int32_t j_ = jm_[mt_];                                                                         \
    const uint16_t* src_ = (j_ >= 0 ? in + (int64_t)j_ * CIN : zrow) + 8 * q;                            \
    _Pragma("unroll") for (int ks_ = 0; ks_ < KS; ++ks_)                                                 \
        areg[SET][mt_ * KS + ks_] = *reinterpret_cast<const u32x4*>(src_ + 32 * ks_);                    \
  }                                                                                                      \
  }
#define EMC2_W_LOAD(TAP, SET)                                                                            \
  {                                                                                                      \
    const u32x4* wsrc_ = wp + (int64_t)(TAP) * W16;                                                      \
    _Pragma("unroll") for (int i_ = 0; i_ < WPT; ++i_)                                                   \
        wq[SET][i_] = wsrc_[(threadIdx.x + i_ * kDThreads) & WMASK];                                     \
  }
#define EMC2_W_STORE(BUF, SET)                                                                           \
  _Pragma("unroll") for (int i_ = 0; i_ < WPT; ++i_)                                                     \
      wl[BUF][(threadIdx.x + i_ * kDThreads) & WMASK] = wq[SET][i_];

  // prologue: map entries of groups 0..2; weights of tap 0 to LDS; A operands of taps 0..2
  EMC2_IDX_LOAD(0, 0)
  EMC2_IDX_LOAD(1, 1)
  EMC2_IDX_LOAD(2, 2)
  EMC2_W_LOAD(0, 0)
  EMC2_W_STORE(0, 0)
  EMC2_W_LOAD(1, 1)
  EMC2_W_LOAD(2, 2)
  EMC2_A_LOAD(emc2_entry(jq[0][0], dead, n_in, oob), 0)
  EMC2_A_LOAD(emc2_entry(jq[0][1], dead, n_in, oob), 1)
  EMC2_A_LOAD(emc2_entry(jq[0][2], dead, n_in, oob), 2)
  __syncthreads();

  for (int g = 0; g < 9; ++g) {
    // kernel-map entries of group g + 3, requested a whole group before anything touches them
    int32_t jn[3];
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) jn[kx] = nrow[(int64_t)(3 * (g + 3 < 9 ? g + 3 : 8) + kx) * capacity_out];
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
      const int tap = 3 * g + kx;
      // weights of tap + 3: global -> registers (the set was emptied at the end of the previous tap)
      EMC2_W_LOAD(tap + 3 < 27 ? tap + 3 : 26, kx)
      const u32x4* wb = wl[tap & 1];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        u32x4 b[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) b[j] = wb[(ks * NT + j) * 64 + lane];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int j = 0; j < NT; ++j) acc[mt][j] = MmaD<DT>::run(areg[kx][mt * KS + ks], b[j], acc[mt][j]);
      }
      // the freed register set takes the A operands of tap + 3 (entries of "group 9" do not exist)
      const int32_t past = g < 8 ? 0 : -1;
      EMC2_A_LOAD(emc2_entry(jq[1][kx], dead | past, n_in, oob), kx)
      __builtin_amdgcn_wave_barrier();
      // weights of tap + 1: registers -> the other LDS buffer; the barrier publishes them and retires the
      // buffer just read
      EMC2_W_STORE((tap + 1) & 1, (kx + 1) % 3)
      __syncthreads();
    }
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
      jq[0][kx] = jq[1][kx];
      jq[1][kx] = jq[2][kx];
      jq[2][kx] = jn[kx];
    }
  }
#undef EMC2_IDX_LOAD
#undef EMC2_A_LOAD
#undef EMC2_W_LOAD
#undef EMC2_W_STORE
  emc2_report_oob(oob, dev_flags);

  // epilogue: lane (m, q) holds column 16*j + m of rows 16*mt + 4*q + e.  Scale/shift/ReLU/convert in
  // registers, then each 16-row tile goes through LDS so that the global stores are whole 16-byte pieces.
  float sc[NT], sh[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    sc[j] = (epilogue != EMC2_EPI_NONE) ? scale[16 * j + m] : 1.f;
    sh[j] = (epilogue != EMC2_EPI_NONE) ? shift[16 * j + m] : 0.f;
  }
  uint16_t* otile = reinterpret_cast<uint16_t*>(otile_s[wave]);
  constexpr int OPI = 64 / OCH;               // rows one store instruction covers
  constexpr int ONI = (16 + OPI - 1) / OPI;   // store instructions per 16-row tile
  const int orow = lane / OCH, ochunk = lane % OCH;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float v = acc[mt][j][e];
        if (epilogue != EMC2_EPI_NONE) v = fmaf(v, sc[j], sh[j]);
        if (epilogue == EMC2_EPI_AFFINE_RELU) v = v > 0.f ? v : 0.f;
        otile[(4 * q + e) * OPITCH + 16 * j + m] = MmaD<DT>::cvt(v);
      }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < ONI; ++i) {
      const int r = i * OPI + orow;
      if (r < 16) {
        const u32x4 piece = *reinterpret_cast<const u32x4*>(otile + r * OPITCH + ochunk * 8);
        const int64_t o = wave_row0 + mt * 16 + r;
        if (o < n_out) *reinterpret_cast<u32x4*>(out + o * COUT + ochunk * 8) = piece;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

template <int DT, int CIN, int COUT>
void launch_direct(const void* d_in, const void* d_wp, const float* d_scale, const float* d_shift, int epilogue,
                   const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int32_t n_in, int32_t* dev_flags,
                   const void* d_zero_row, void* d_out, hipStream_t s) {
  const int64_t rows_per_block = kDWaves * 16 * DirectCfg<CIN, COUT>::MT;
  hipLaunchKernelGGL((k_spconv_direct<DT, CIN, COUT>), dim3((unsigned)(emc2_div_up(capacity_out, rows_per_block) + 8)),
                     dim3(kDThreads), 0, s, (const uint16_t*)d_in, (const u32x4*)d_wp, d_scale, d_shift, epilogue, d_nbr,
                     d_n_out, capacity_out, n_in, dev_flags, (const uint16_t*)d_zero_row, (uint16_t*)d_out);
}

}  // namespace

bool emc2_spconv_direct_supported(int cin, int cout) {
  return ((cin == 32 || cin == 64) && (cout == 32 || cout == 64)) || (cin == 128 && cout == 128) || (cin == 64 && cout == 128);
}

void emc2_spconv_direct_pack(const void* d_w, int cin, int cout, void* d_packed, hipStream_t stream) {
  const int total = 27 * (cin / 32) * (cout / 16) * 64;
  hipLaunchKernelGGL(k_pack_weights_direct, dim3((unsigned)emc2_div_up(total, 256)), dim3(256), 0, stream,
                     (const uint16_t*)d_w, cin, cout, (uint4*)d_packed);
}

void emc2_spconv_direct_launch(emc2_dtype dtype, const void* d_in, const void* d_wp, const float* d_scale,
                               const float* d_shift, int epilogue, const int32_t* d_nbr, const int32_t* d_n_out,
                               int64_t capacity_out, int32_t n_in, int32_t* dev_flags, int cin, int cout,
                               const void* d_zero_row, void* d_out, hipStream_t stream) {
#define CASE(DTV, CI, CO)                                                                                              \
  if (dtype == DTV && cin == CI && cout == CO) {                                                                       \
    launch_direct<DTV, CI, CO>(d_in, d_wp, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, n_in, dev_flags,  \
                               d_zero_row, d_out, stream);                                                             \
    return;                                                                                                            \
  }
  CASE(EMC2_F16, 32, 32) CASE(EMC2_F16, 32, 64) CASE(EMC2_F16, 64, 32) CASE(EMC2_F16, 64, 64)
  CASE(EMC2_BF16, 32, 32) CASE(EMC2_BF16, 32, 64) CASE(EMC2_BF16, 64, 32) CASE(EMC2_BF16, 64, 64)
  CASE(EMC2_F16, 128, 128) CASE(EMC2_F16, 64, 128) CASE(EMC2_BF16, 128, 128) CASE(EMC2_BF16, 64, 128)
#undef CASE
}
