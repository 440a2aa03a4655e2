// Sparse convolution over a kernel map (paper Sec. 3.5: customised 3D sparse convolution over the
// non-empty voxels; Sec. 3.6: graph fusion -> affine + ReLU fused into the epilogue).
// This file: argument checks, dispatch, and the vector-ALU kernel (fp32 path and channel counts
// the MFMA kernels do not cover).  The MFMA gather-GEMM lives in spconv_mfma.hip.
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>

#include "common.h"
#include "spconv_mfma.h"

namespace {

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(__half v) { return __half2float(v); }
__device__ __forceinline__ float to_f32(__hip_bfloat16 v) { return __bfloat162float(v); }
__device__ __forceinline__ void from_f32(float* p, float v) { *p = v; }
__device__ __forceinline__ void from_f32(__half* p, float v) { *p = __float2half_rn(v); }
__device__ __forceinline__ void from_f32(__hip_bfloat16* p, float v) { *p = __float2bfloat16(v); }

// Output-stationary: `cout` consecutive threads own one output row; taps outer, input channels inner.
template <typename T>
__global__ void __launch_bounds__(256) k_spconv_alu(const T* __restrict__ in, const T* __restrict__ w,
                                                    const float* __restrict__ scale, const float* __restrict__ shift,
                                                    int epilogue, const int32_t* __restrict__ nbr,
                                                    const int32_t* __restrict__ d_n_out, int64_t capacity_out,
                                                    int32_t n_in, int32_t* __restrict__ dev_flags, int cin, int cout,
                                                    int rows_per_block, T* __restrict__ out) {
  int64_t n = *d_n_out;
  if (n > capacity_out) n = capacity_out;
  const int row = threadIdx.x / cout;
  const int d = threadIdx.x - row * cout;
  const int64_t o = (int64_t)blockIdx.x * rows_per_block + row;
  if (row >= rows_per_block || o >= n) return;
  float acc = 0.f;
  for (int k = 0; k < 27; ++k) {
    const int32_t j = nbr[(int64_t)k * capacity_out + o];
    if (j < 0) continue;
    if (j >= n_in) {   // names a row the input does not hold: absent, and reported
      if (d == 0) atomicOr(dev_flags, EMC2_DEVFLAG_MAP);
      continue;
    }
    const T* xr = in + (int64_t)j * cin;
    const T* wk = w + (int64_t)k * cin * cout + d;
    for (int c = 0; c < cin; ++c) acc = fmaf(to_f32(xr[c]), to_f32(wk[(int64_t)c * cout]), acc);
  }
  if (epilogue != EMC2_EPI_NONE) acc = fmaf(acc, scale[d], shift[d]);
  if (epilogue == EMC2_EPI_AFFINE_RELU) acc = acc > 0.f ? acc : 0.f;
  from_f32(out + o * cout + d, acc);
}

// Small-channel kernel (Cin in {4, 16}, Cout in {16, 32}: the input layers that sit below the matrix-core
// tile sizes).  One thread owns one output row and all of its Cout accumulators; a tap's weights are LDS
// broadcasts and a tap nobody in the wave has is skipped.  These layers have few rows (one wave per 64 of
// them, a handful of waves per CU), so latency, not bandwidth, is what they can lose time to: all 27
// kernel-map entries of a row are requested at once, and the feature rows of a whole batch of taps (27 at
// Cin = 4, 9 at Cin = 16) are requested together, unconditionally (absent entries re-read row 0), before
// the first of them is used -- two memory round trips per batch instead of two per tap.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

template <typename T, int CIN, int COUT>
__global__ void __launch_bounds__(256) k_spconv_small(const T* __restrict__ in, const T* __restrict__ w,
                                                      const float* __restrict__ scale, const float* __restrict__ shift,
                                                      int epilogue, const int32_t* __restrict__ nbr,
                                                      const int32_t* __restrict__ d_n_out, int64_t capacity_out,
                                                      int32_t n_in, int32_t* __restrict__ dev_flags, T* __restrict__ out) {
  __shared__ float wl[27 * CIN * COUT];
  for (int i = threadIdx.x; i < 27 * CIN * COUT; i += 256) wl[i] = to_f32(w[i]);
  int64_t n = *d_n_out;
  if (n > capacity_out) n = capacity_out;
  const int64_t o = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const bool live = o < n;
  const int32_t* nrow = nbr + (live ? o : 0);
  const int32_t dead = live ? 0 : -1;
  constexpr int ROW_BYTES = CIN * (int)sizeof(T);
  static_assert(ROW_BYTES == 8 || ROW_BYTES % 16 == 0, "feature rows are read with 8- or 16-byte loads");
  constexpr int RW = ROW_BYTES / 4;               // 32-bit words per feature row
  constexpr int TB = ROW_BYTES <= 8 ? 27 : 9;     // taps whose rows are in flight together
  int32_t j[27];
  unsigned long long oob = 0ull;   // lanes that saw an entry outside [0, n_in)
#pragma unroll
  for (int k = 0; k < 27; ++k) j[k] = nrow[(int64_t)k * capacity_out];
  float acc[COUT];
#pragma unroll
  for (int d = 0; d < COUT; ++d) acc[d] = 0.f;
  __syncthreads();   // weights in LDS
#pragma unroll
  for (int k0 = 0; k0 < 27; k0 += TB) {
    uint32_t xr[TB][RW];
#pragma unroll
    for (int t = 0; t < TB; ++t) {
      const int32_t jj = j[k0 + t] = emc2_entry(j[k0 + t], dead, n_in, oob);   // masked once, used twice
      const char* src = reinterpret_cast<const char*>(in + (int64_t)(jj >= 0 ? jj : 0) * CIN);
      if constexpr (ROW_BYTES == 8) {
        const u32x2_t v = *reinterpret_cast<const u32x2_t*>(src);
        xr[t][0] = v.x; xr[t][1] = v.y;
      } else {
#pragma unroll
        for (int q = 0; q < ROW_BYTES / 16; ++q) {
          const u32x4_t v = reinterpret_cast<const u32x4_t*>(src)[q];
          xr[t][4 * q] = v.x; xr[t][4 * q + 1] = v.y; xr[t][4 * q + 2] = v.z; xr[t][4 * q + 3] = v.w;
        }
      }
    }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
      const int k = k0 + t;
      const bool have = j[k] >= 0;
      if (__ballot(have) == 0ull) continue;  // wave-uniform
      if (have) {
        const float* wk = wl + k * CIN * COUT;
#pragma unroll
        for (int c = 0; c < CIN; ++c) {
          T xe;
          if constexpr (sizeof(T) == 2) {
            const uint16_t bits = (uint16_t)(xr[t][c / 2] >> (16 * (c % 2)));
            xe = __builtin_bit_cast(T, bits);
          } else {
            xe = __builtin_bit_cast(T, xr[t][c]);
          }
          const float xv = to_f32(xe);
#pragma unroll
          for (int d = 0; d < COUT; ++d) acc[d] = fmaf(xv, wk[c * COUT + d], acc[d]);
        }
      }
    }
  }
  emc2_report_oob(oob, dev_flags);
  if (!live) return;
  alignas(16) T yr[COUT];
#pragma unroll
  for (int d = 0; d < COUT; ++d) {
    float v = acc[d];
    if (epilogue != EMC2_EPI_NONE) v = fmaf(v, scale[d], shift[d]);
    if (epilogue == EMC2_EPI_AFFINE_RELU) v = v > 0.f ? v : 0.f;
    from_f32(&yr[d], v);
  }
  constexpr int OUT_BYTES = COUT * (int)sizeof(T);
  static_assert(OUT_BYTES % 16 == 0, "output rows are written with 16-byte stores");
  char* dst = reinterpret_cast<char*>(out + o * COUT);
#pragma unroll
  for (int q = 0; q < OUT_BYTES / 16; ++q) reinterpret_cast<u32x4_t*>(dst)[q] = reinterpret_cast<const u32x4_t*>(yr)[q];
}

// Small-channel 16-bit kernel on the matrix cores (Cin in {4, 16}, Cout in {16, 32}).  Memory access as in
// k_spconv_small -- lane = output row, every kernel-map entry and feature row requested with whole-wave loads that
// touch a few cache lines each -- but the contraction runs on v_mfma_f32_4x4x4 (16 blocks of 4x4x4 per instruction):
// as the B operand, lane l supplies 4 input channels of ITS row (8 bytes, exactly what it loaded); as the A
// operand it supplies W[tap][4 channels][4g + l % 4], the same 4x4 weight block for every block of rows; the result
// leaves 4 consecutive output channels of row l in lane l's four accumulator registers, so the epilogue is
// per-lane and the stores are whole 16-byte pieces of the lane's own row.  The vector-ALU kernel spends its time
// re-reading weights from LDS for every multiply-add (one LDS read per 4 of them); here a weight block is read
// once per tap and 4 channels for two groups of 64 rows, and a tap none of the 128 rows has costs nothing.
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));

template <int DT> struct Mma4;
template <> struct Mma4<EMC2_F16> {
  static __device__ __forceinline__ float4_t run(u32x2_t a, u32x2_t b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_4x4x4f16(__builtin_bit_cast(half4_t, a), __builtin_bit_cast(half4_t, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t cvt2(float lo, float hi) {
    return (uint32_t)__half_as_ushort(__float2half_rn(lo)) | ((uint32_t)__half_as_ushort(__float2half_rn(hi)) << 16);
  }
};
template <> struct Mma4<EMC2_BF16> {
  static __device__ __forceinline__ float4_t run(u32x2_t a, u32x2_t b, float4_t c) {
    return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(__builtin_bit_cast(short4_t, a), __builtin_bit_cast(short4_t, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t cvt2(float lo, float hi) {
    return (uint32_t)__builtin_bit_cast(uint16_t, __float2bfloat16(lo)) |
           ((uint32_t)__builtin_bit_cast(uint16_t, __float2bfloat16(hi)) << 16);
  }
};

template <int DT, int CIN, int COUT>
__global__ void __launch_bounds__(256, 4) k_spconv_rows(const uint16_t* __restrict__ in, const uint16_t* __restrict__ w,
                                                     const float* __restrict__ scale, const float* __restrict__ shift,
                                                     int epilogue, const int32_t* __restrict__ nbr,
                                                     const int32_t* __restrict__ d_n_out, int64_t capacity_out,
                                                     int32_t n_in, int32_t* __restrict__ dev_flags,
                                                     uint16_t* __restrict__ out) {
  constexpr int KB = CIN / 4;                 // 4-channel blocks of an input row
  constexpr int G = COUT / 4;                 // 4-channel groups of an output row
  constexpr int RG = 2;                       // groups of 64 rows per wave (a weight block read serves both)
  constexpr int TB = CIN == 4 ? 9 : 3;        // taps whose rows are in flight together
  constexpr int RW = CIN / 2;                 // 32-bit words per input row
  static_assert(27 % TB == 0 && CIN % 4 == 0 && COUT % 8 == 0, "shapes this kernel covers");
  // weights as A operands: wl[((tap * KB + kb) * G + g) * 4 + j] = W[tap][4kb + 0..3][4g + j], 8 bytes
  __shared__ u32x2_t wl[27 * KB * G * 4];
  for (int e = threadIdx.x; e < 27 * KB * G * 4; e += 256) {
    const int j = e & 3;
    int f = e >> 2;
    const int g = f % G; f /= G;
    const int kb = f % KB;
    const int tap = f / KB;
    const uint16_t* src = w + ((int64_t)tap * CIN + 4 * kb) * COUT + 4 * g + j;
    wl[e] = u32x2_t{(uint32_t)src[0] | ((uint32_t)src[COUT] << 16), (uint32_t)src[2 * COUT] | ((uint32_t)src[3 * COUT] << 16)};
  }
  int64_t n = *d_n_out;
  if (n > capacity_out) n = capacity_out;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int64_t row0 = (int64_t)blockIdx.x * (4 * RG * 64) + (int64_t)wave * (RG * 64) + lane;
  bool live[RG];
  const int32_t* nrow[RG];
  int32_t dead[RG];
#pragma unroll
  for (int r = 0; r < RG; ++r) {
    live[r] = row0 + 64 * r < n;
    nrow[r] = nbr + (live[r] ? row0 + 64 * r : 0);
    dead[r] = live[r] ? 0 : -1;
  }
  unsigned long long oob = 0ull;
  float4_t acc[RG][G];
#pragma unroll
  for (int r = 0; r < RG; ++r)
#pragma unroll
    for (int g = 0; g < G; ++g) acc[r][g] = float4_t{0.f, 0.f, 0.f, 0.f};
  __syncthreads();   // weights in LDS
  const int jq = lane & 3;
#pragma unroll 1
  for (int k0 = 0; k0 < 27; k0 += TB) {
    int32_t j[RG][TB];
#pragma unroll
    for (int r = 0; r < RG; ++r)
#pragma unroll
      for (int t = 0; t < TB; ++t) j[r][t] = nrow[r][(int64_t)(k0 + t) * capacity_out];
    uint32_t x[RG][TB][RW];
#pragma unroll
    for (int r = 0; r < RG; ++r)
#pragma unroll
      for (int t = 0; t < TB; ++t) {
        j[r][t] = emc2_entry(j[r][t], dead[r], n_in, oob);
        const char* src = reinterpret_cast<const char*>(in + (int64_t)(j[r][t] >= 0 ? j[r][t] : 0) * CIN);
        if constexpr (RW == 2) {
          const u32x2_t v = *reinterpret_cast<const u32x2_t*>(src);
          x[r][t][0] = v.x; x[r][t][1] = v.y;
        } else {
#pragma unroll
          for (int q = 0; q < RW / 4; ++q) {
            const u32x4_t v = reinterpret_cast<const u32x4_t*>(src)[q];
            x[r][t][4 * q] = v.x; x[r][t][4 * q + 1] = v.y; x[r][t][4 * q + 2] = v.z; x[r][t][4 * q + 3] = v.w;
          }
        }
      }
#pragma unroll
    for (int t = 0; t < TB; ++t) {
      bool have[RG];
      unsigned long long any = 0ull;
#pragma unroll
      for (int r = 0; r < RG; ++r) {
        have[r] = j[r][t] >= 0;
        any |= __ballot(have[r]);
      }
      if (any == 0ull) continue;   // wave-uniform: nobody has this tap
      const u32x2_t* wt = wl + (k0 + t) * KB * G * 4 + jq;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        u32x2_t b[RG];
#pragma unroll
        for (int r = 0; r < RG; ++r)
          b[r] = have[r] ? u32x2_t{x[r][t][2 * kb], x[r][t][2 * kb + 1]} : u32x2_t{0u, 0u};   // an absent neighbour adds zero
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const u32x2_t a = wt[(kb * G + g) * 4];
#pragma unroll
          for (int r = 0; r < RG; ++r) acc[r][g] = Mma4<DT>::run(a, b[r], acc[r][g]);
        }
      }
    }
  }
  emc2_report_oob(oob, dev_flags);
  // lane l holds output channels 4g .. 4g+3 of its row in acc[r][g]
#pragma unroll
  for (int r = 0; r < RG; ++r) {
    if (!live[r]) continue;
    uint32_t y[COUT / 2];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float v[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        v[i] = acc[r][g][i];
        if (epilogue != EMC2_EPI_NONE) v[i] = fmaf(v[i], scale[4 * g + i], shift[4 * g + i]);
        if (epilogue == EMC2_EPI_AFFINE_RELU) v[i] = v[i] > 0.f ? v[i] : 0.f;
      }
      y[2 * g] = Mma4<DT>::cvt2(v[0], v[1]);
      y[2 * g + 1] = Mma4<DT>::cvt2(v[2], v[3]);
    }
    u32x4_t* dst = reinterpret_cast<u32x4_t*>(out + (row0 + 64 * r) * COUT);
#pragma unroll
    for (int q = 0; q < COUT / 8; ++q) dst[q] = u32x4_t{y[4 * q], y[4 * q + 1], y[4 * q + 2], y[4 * q + 3]};
  }
}

template <int DT>
bool launch_rows(const void* d_in, const void* d_w, const float* d_scale, const float* d_shift, int epilogue,
                 const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int32_t n_in, int32_t* dev_flags,
                 int cin, int cout, void* d_out, hipStream_t s) {
#define EMC2_ROWS(CI, CO)                                                                                             \
  if (cin == CI && cout == CO) {                                                                                      \
    hipLaunchKernelGGL((k_spconv_rows<DT, CI, CO>), dim3((unsigned)emc2_div_up(capacity_out, 512)), dim3(256), 0, s,  \
                       (const uint16_t*)d_in, (const uint16_t*)d_w, d_scale, d_shift, epilogue, d_nbr, d_n_out,       \
                       capacity_out, n_in, dev_flags, (uint16_t*)d_out);                                              \
    return true;                                                                                                      \
  }
  EMC2_ROWS(4, 16) EMC2_ROWS(4, 32) EMC2_ROWS(16, 16)
#undef EMC2_ROWS
  return false;
}

template <typename T>
bool launch_small(const void* d_in, const void* d_w, const float* d_scale, const float* d_shift, int epilogue,
                  const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int32_t n_in, int32_t* dev_flags,
                  int cin, int cout, void* d_out, hipStream_t s) {
#define EMC2_SMALL(CI, CO)                                                                                            \
  if (cin == CI && cout == CO) {                                                                                      \
    hipLaunchKernelGGL((k_spconv_small<T, CI, CO>), dim3((unsigned)emc2_div_up(capacity_out, 256)), dim3(256), 0, s,  \
                       (const T*)d_in, (const T*)d_w, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out,       \
                       n_in, dev_flags, (T*)d_out);                                                                   \
    return true;                                                                                                      \
  }
  EMC2_SMALL(4, 16) EMC2_SMALL(4, 32) EMC2_SMALL(16, 16)
#undef EMC2_SMALL
  return false;
}

template <typename T>
void launch_alu(const void* d_in, const void* d_w, const float* d_scale, const float* d_shift, int epilogue,
                const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int32_t n_in, int32_t* dev_flags,
                int cin, int cout, void* d_out, hipStream_t s) {
  if (launch_small<T>(d_in, d_w, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, n_in, dev_flags, cin, cout, d_out, s))
    return;
  const int rows = 256 / cout;
  hipLaunchKernelGGL(k_spconv_alu<T>, dim3((unsigned)emc2_div_up(capacity_out, rows)), dim3(256), 0, s, (const T*)d_in,
                     (const T*)d_w, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, n_in, dev_flags, cin, cout, rows,
                     (T*)d_out);
}

}  // namespace

extern "C" int32_t emc2_spconv_uses_mfma(emc2_dtype dtype, int32_t cin, int32_t cout) {
  return (dtype == EMC2_F16 || dtype == EMC2_BF16) && emc2_spconv_mfma_supported(cin, cout) ? 1 : 0;
}

// shapes of the thread-per-row vector-ALU kernel (fp32) and of the small-channel matrix-core kernel (16-bit); 16 -> 32
// was tried on the latter and is three times slower there than on the staged MFMA kernel
static bool small_covers(int cin, int cout) { return (cin == 4 && (cout == 16 || cout == 32)) || (cin == 16 && cout == 16); }
static bool rows_covers(int cin, int cout) { return small_covers(cin, cout); }

extern "C" const char* emc2_spconv_kernel(emc2_dtype dtype, int32_t cin, int32_t cout, int32_t map_hint) {
  if (dtype != EMC2_F32 && dtype != EMC2_F16 && dtype != EMC2_BF16) return nullptr;
  if (emc2_spconv_uses_mfma(dtype, cin, cout)) {
    if (!emc2_spconv_direct_supported(cin, cout)) return "k_spconv_mfma";
    return (map_hint == EMC2_CONV_SUBM && emc2_spconv_span_supported(cin, cout)) ? "k_spconv_span" : "k_spconv_direct";
  }
  if (dtype == EMC2_F32) return small_covers(cin, cout) ? "k_spconv_small" : "k_spconv_alu";
  return rows_covers(cin, cout) ? "k_spconv_rows" : "k_spconv_alu";
}

extern "C" emc2_status emc2_pack_weights(emc2_ctx* ctx, emc2_dtype dtype, const void* d_w, int32_t cin, int32_t cout,
                                         void* d_packed, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_w || !d_packed || d_w == d_packed) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pack_weights: bad pointers");
  if (!emc2_spconv_uses_mfma(dtype, cin, cout))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_pack_weights: (dtype, Cin=%d, Cout=%d) does not use the MFMA path", cin,
                     cout);
  // the fragment order is a function of (Cin, Cout) alone: whichever kernel a call later selects for this
  // shape reads the same packed weights
  if (emc2_spconv_direct_supported(cin, cout))
    emc2_spconv_direct_pack(d_w, cin, cout, d_packed, (hipStream_t)stream);
  else
    emc2_spconv_mfma_pack(d_w, cin, cout, d_packed, (hipStream_t)stream);
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_pack_weights launch");
}

extern "C" emc2_status emc2_spconv(emc2_ctx* ctx, emc2_dtype dtype, const void* d_in, const void* d_w,
                                   emc2_wlayout w_layout, const float* d_scale, const float* d_shift,
                                   emc2_epilogue epilogue, const int32_t* d_nbr, int32_t map_hint,
                                   const int32_t* d_n_out, int64_t capacity_out, int64_t n_in_rows, int32_t cin,
                                   int32_t cout, void* d_out, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_in || !d_w || !d_nbr || !d_n_out || !d_out)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv: null argument");
  if (epilogue != EMC2_EPI_NONE && epilogue != EMC2_EPI_AFFINE && epilogue != EMC2_EPI_AFFINE_RELU)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv: bad epilogue");
  if ((epilogue == EMC2_EPI_NONE) != (d_scale == nullptr) || (d_scale == nullptr) != (d_shift == nullptr))
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv: scale/shift must be given iff the epilogue is affine");
  if (capacity_out < 1) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv: capacity_out < 1");
  if (n_in_rows < 0) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv: n_in_rows < 0");
  const int32_t n_in = n_in_rows > 0x7fffffff ? 0x7fffffff : (int32_t)n_in_rows;
  if (cin < 1 || cout < 1 || cin > 1024 || cout > 256)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_spconv: channels outside Cin<=1024, Cout<=256");
  if (dtype != EMC2_F32 && dtype != EMC2_F16 && dtype != EMC2_BF16)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_spconv: bad dtype");
  if (w_layout != EMC2_W_PLAIN && w_layout != EMC2_W_PACKED)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv: bad weight layout");
  if (map_hint != EMC2_MAP_ANY && map_hint != EMC2_CONV_SUBM && map_hint != EMC2_CONV_STRIDED)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv: bad map_hint");
  const bool mfma = emc2_spconv_uses_mfma(dtype, cin, cout) != 0;
  if (w_layout == EMC2_W_PACKED && !mfma)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_spconv: packed weights need an MFMA-covered (dtype, Cin, Cout)");
  // the matrix-core and small-channel kernels move rows as 8- or 16-byte pieces
  if (dtype != EMC2_F32 && (((uintptr_t)d_in | (uintptr_t)d_out | (uintptr_t)d_w) & 15u))
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv: 16-bit d_in, d_w and d_out must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  int32_t* flags = ctx->dev_words;
  if (mfma) {
    const bool direct = emc2_spconv_direct_supported(cin, cout);
    const void* wp = d_w;
    if (w_layout == EMC2_W_PLAIN) {
      // stream order protects the shared scratch
      if (direct) emc2_spconv_direct_pack(d_w, cin, cout, ctx->wpack, s);
      else emc2_spconv_mfma_pack(d_w, cin, cout, ctx->wpack, s);
      wp = ctx->wpack;
    }
    if (!direct)
      emc2_spconv_mfma_launch(dtype, d_in, wp, d_scale, d_shift, (int)epilogue, d_nbr, d_n_out, capacity_out, n_in, flags,
                              cin, cout, d_out, s);
    else if (map_hint == EMC2_CONV_SUBM && emc2_spconv_span_supported(cin, cout))
      // pays where the three kx taps of a group name nearly the same rows
      emc2_spconv_span_launch(dtype, d_in, wp, d_scale, d_shift, (int)epilogue, d_nbr, d_n_out, capacity_out, n_in, flags,
                              cin, cout, d_out, s);
    else
      emc2_spconv_direct_launch(dtype, d_in, wp, d_scale, d_shift, (int)epilogue, d_nbr, d_n_out, capacity_out, n_in, flags,
                                cin, cout, ctx->zero_row, d_out, s);
  } else if (dtype == EMC2_F32) {
    launch_alu<float>(d_in, d_w, d_scale, d_shift, (int)epilogue, d_nbr, d_n_out, capacity_out, n_in, flags, cin, cout, d_out, s);
  } else if (dtype == EMC2_F16 && launch_rows<EMC2_F16>(d_in, d_w, d_scale, d_shift, (int)epilogue, d_nbr, d_n_out, capacity_out,
                                                        n_in, flags, cin, cout, d_out, s)) {
  } else if (dtype == EMC2_BF16 && launch_rows<EMC2_BF16>(d_in, d_w, d_scale, d_shift, (int)epilogue, d_nbr, d_n_out,
                                                          capacity_out, n_in, flags, cin, cout, d_out, s)) {
  } else if (dtype == EMC2_F16) {
    launch_alu<__half>(d_in, d_w, d_scale, d_shift, (int)epilogue, d_nbr, d_n_out, capacity_out, n_in, flags, cin, cout, d_out, s);
  } else {
    launch_alu<__hip_bfloat16>(d_in, d_w, d_scale, d_shift, (int)epilogue, d_nbr, d_n_out, capacity_out, n_in, flags, cin, cout,
                               d_out, s);
  }
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_spconv launch");
}
