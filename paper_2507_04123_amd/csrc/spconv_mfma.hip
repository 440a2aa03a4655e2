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
//   - A operand: lane (m = lane%32, h = lane/32) holds 8 consecutive input channels of row m, which
//     is one 16-byte load straight from the gathered feature row -- the gather goes global->VGPR;
//   - B operand: W_k is staged through LDS once per block and tap, transposed on the way in so that
//     lane (n, h) reads its 8 consecutive K values with one 16-byte LDS load;
//   - taps for which a 32-row tile has no neighbour at all are skipped by a wave ballot;
//   - epilogue: acc*scale+shift, ReLU, convert, store.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "common.h"
#include "spconv_mfma.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int DT> struct Mma;
template <> struct Mma<EMC2_F16> {
  static __device__ __forceinline__ floatx16 run(uint4 a, uint4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float v) { return __half_as_ushort(__float2half_rn(v)); }
};
template <> struct Mma<EMC2_BF16> {
  static __device__ __forceinline__ floatx16 run(uint4 a, uint4 b, floatx16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float v) {
    return __builtin_bit_cast(uint16_t, __float2bfloat16(v));
  }
};

constexpr int kWaves = 4;

// LDS image of one tap's weights, transposed: wt[n][K + pad] 16-bit, so that 8 consecutive K of a
// column are contiguous.  The pad of 8 elements (16 B) staggers rows across banks.
template <int CIN> struct LdsW { static constexpr int kRow = CIN + 8; };

template <int DT, int CIN, int COUT, int MT>
__global__ void __launch_bounds__(256) k_spconv_mfma(const uint16_t* __restrict__ in, const uint16_t* __restrict__ w,
                                                     const float* __restrict__ scale, const float* __restrict__ shift,
                                                     int epilogue, const int32_t* __restrict__ nbr,
                                                     const int32_t* __restrict__ d_n_out, int64_t capacity_out,
                                                     uint16_t* __restrict__ out) {
  constexpr int KS = CIN / 16;   // k-steps per tap
  constexpr int NT = COUT / 32;  // 32-column tiles
  constexpr int ROW = LdsW<CIN>::kRow;
  __shared__ __attribute__((aligned(16))) uint16_t wt[COUT * ROW];

  int64_t n_out = *d_n_out;
  if (n_out > capacity_out) n_out = capacity_out;
  const int64_t block_row0 = (int64_t)blockIdx.x * (kWaves * MT * 32);
  if (block_row0 >= n_out) return;  // whole block past the end (uniform)

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int m = lane & 31, h = lane >> 5;
  const int64_t wave_row0 = block_row0 + (int64_t)wave * (MT * 32);

  floatx16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[mt][j][e] = 0.f;

  for (int tap = 0; tap < 27; ++tap) {
    // gather this tap's A fragments (global -> VGPR)
    uint4 a[MT][KS];
    bool any[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int64_t o = wave_row0 + mt * 32 + m;
      const int32_t j = (o < n_out) ? nbr[(int64_t)tap * capacity_out + o] : -1;
      any[mt] = __ballot(j >= 0) != 0ull;
      const uint4* src = reinterpret_cast<const uint4*>(in + (int64_t)(j >= 0 ? j : 0) * CIN + 8 * h);
#pragma unroll
      for (int t = 0; t < KS; ++t) a[mt][t] = (j >= 0) ? src[2 * t] : make_uint4(0u, 0u, 0u, 0u);
    }
    // stage W[tap] into LDS, transposed to [n][K]
    __syncthreads();  // previous tap's B reads are done
    {
      const uint16_t* wk = w + (int64_t)tap * CIN * COUT;
      // each thread moves pairs of K for one column: coalesced 2-byte reads along n, 4-byte LDS writes
      for (int idx = threadIdx.x; idx < (CIN / 2) * COUT; idx += 256) {
        const int n = idx % COUT;
        const int c2 = idx / COUT;
        const uint32_t lo = wk[(2 * c2) * COUT + n];
        const uint32_t hi = wk[(2 * c2 + 1) * COUT + n];
        *reinterpret_cast<uint32_t*>(&wt[n * ROW + 2 * c2]) = lo | (hi << 16);
      }
    }
    __syncthreads();
    bool wave_any = false;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) wave_any |= any[mt];
    if (wave_any) {
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        uint4 b[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j)
          b[j] = *reinterpret_cast<const uint4*>(&wt[(32 * j + m) * ROW + 16 * t + 8 * h]);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          if (!any[mt]) continue;
#pragma unroll
          for (int j = 0; j < NT; ++j) acc[mt][j] = Mma<DT>::run(a[mt][t], b[j], acc[mt][j]);
        }
      }
    }
  }

  // epilogue: lane holds column n = 32*j + m; acc element e <-> row 8*(e/4) + 4*h + (e%4)
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int n = 32 * j + m;
    const float sc = (epilogue != EMC2_EPI_NONE) ? scale[n] : 1.f;
    const float sh = (epilogue != EMC2_EPI_NONE) ? shift[n] : 0.f;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int64_t o = wave_row0 + mt * 32 + 8 * (e / 4) + 4 * h + (e % 4);
        if (o < n_out) {
          float v = acc[mt][j][e];
          if (epilogue != EMC2_EPI_NONE) v = fmaf(v, sc, sh);
          if (epilogue == EMC2_EPI_AFFINE_RELU) v = v > 0.f ? v : 0.f;
          out[o * COUT + n] = Mma<DT>::cvt(v);
        }
      }
    }
  }
}

template <int DT, int CIN, int COUT>
void launch(const void* d_in, const void* d_w, const float* d_scale, const float* d_shift, int epilogue,
            const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, void* d_out, hipStream_t s) {
  constexpr int MT = 2;
  const int64_t rows_per_block = kWaves * MT * 32;
  hipLaunchKernelGGL((k_spconv_mfma<DT, CIN, COUT, MT>), dim3((unsigned)emc2_div_up(capacity_out, rows_per_block)), dim3(256),
                     0, s, (const uint16_t*)d_in, (const uint16_t*)d_w, d_scale, d_shift, epilogue, d_nbr, d_n_out,
                     capacity_out, (uint16_t*)d_out);
}

template <int DT>
void dispatch(const void* d_in, const void* d_w, const float* d_scale, const float* d_shift, int epilogue,
              const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int cin, int cout, void* d_out,
              hipStream_t s) {
#define CASE(CI, CO)                                                                                              \
  if (cin == CI && cout == CO) {                                                                                  \
    launch<DT, CI, CO>(d_in, d_w, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, d_out, s);            \
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

void emc2_spconv_mfma_launch(emc2_dtype dtype, const void* d_in, const void* d_w, const float* d_scale,
                             const float* d_shift, int epilogue, const int32_t* d_nbr, const int32_t* d_n_out,
                             int64_t capacity_out, int cin, int cout, void* d_out, hipStream_t stream) {
  if (dtype == EMC2_F16)
    dispatch<EMC2_F16>(d_in, d_w, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, cin, cout, d_out, stream);
  else
    dispatch<EMC2_BF16>(d_in, d_w, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, cin, cout, d_out, stream);
}
