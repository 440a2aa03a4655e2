// Quantised sparse convolution on the int8 matrix cores (paper Sec. 3.6 (2): model quantisation is one of the
// deployment optimisations; the paper gives no scheme, the one here is stated in emc2.h).
//
// Same shape as the register-direct 16-bit kernel: v_mfma_i32_16x16x64_i8 takes, in lane (m = lane % 16,
// q = lane / 16), the 16 consecutive input channels 16q .. 16q+15 of row m of the tile, i.e. 16 contiguous bytes
// of the feature row nbr[k][o_m]; a 64-channel int8 row is exactly the four lanes' 64 bytes, so ONE
// global_load_dwordx4 per 16-row tile and tap is the A operand (half the bytes and half the cache lines of the
// fp16 kernel, twice the multiply-accumulates per matrix instruction).  Absent neighbours read a zeroed row.
// LDS holds the weights of the current and the next tap in B-fragment order and a small tile that turns the
// accumulator layout into whole 16-byte pieces of output rows.  Accumulation is exact (int32); the epilogue is
// a fixed sequence of individually rounded fp32 operations, so results are bit-reproducible.
#include <hip/hip_fp16.h>

#include "common.h"

#pragma clang fp contract(off)

namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kQWaves = 4;
constexpr int kQThreads = kQWaves * 64;

__device__ __forceinline__ int quant_i8(float v, float inv_scale) {
  float r = rintf(v * inv_scale);  // to nearest, ties to even
  if (!(r == r)) r = 0.f;
  r = r > 127.f ? 127.f : r;
  r = r < -127.f ? -127.f : r;
  return (int)r;
}

// E4M3 (bias 7, no infinities, largest value 448): nearest finite value of t, ties to the even code, saturating,
// NaN -> 0, a result of zero always +0.  Integer arithmetic on the fp32 bits, so that no conversion mode of the
// hardware enters: above the subnormal range the 20 low mantissa bits are rounded away (the carry runs into the
// exponent by itself); below 2^-6 the value is a multiple of 2^-9.
__device__ __forceinline__ uint32_t quant_e4m3(float t) {
  if (!(t == t)) return 0u;
  const float a = fabsf(t);
  uint32_t code;
  if (a >= 448.0f) {
    code = 0x7Eu;
  } else if (a < 0.015625f) {
    code = (uint32_t)rintf(a * 512.0f);          // exact product; ties to even; 8 is the first normal code
  } else {
    const uint32_t bits = __float_as_uint(a);
    const uint32_t r = (bits + 0x7FFFFu + ((bits >> 20) & 1u)) >> 20;   // (exponent << 3 | mantissa), rounded to nearest even
    code = r - (120u << 3);
    code = code > 0x7Eu ? 0x7Eu : code;          // 464 .. 448 rounds up to a code that is not a number: saturate
  }
  return (code != 0u && t < 0.0f) ? (code | 0x80u) : code;
}

template <typename T>
__global__ void __launch_bounds__(256) k_quantize_e4m3(const T* __restrict__ x, int64_t n, float inv_scale, uint8_t* __restrict__ q) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) q[i] = (uint8_t)quant_e4m3((float)x[i] * inv_scale);
}

template <typename T>
__global__ void __launch_bounds__(256) k_quantize_i8(const T* __restrict__ x, int64_t n, float inv_scale, int8_t* __restrict__ q) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) q[i] = (int8_t)quant_i8((float)x[i], inv_scale);
}

// Packed layout: 16-byte piece ((k*KS + t)*NT + j)*64 + lane, lane = 16*q + n, holds W[k][64t + 16q + e][16j + n],
// e = 0..15 -- the B operand of k-step t, column tile j.
__global__ void __launch_bounds__(256) k_pack_weights_i8(const int8_t* __restrict__ w, int cin, int cout, uint4* __restrict__ packed) {
  const int ks = cin / 64, nt = cout / 16;
  const int total = 27 * ks * nt * 64;
  const int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= total) return;
  const int lane = p & 63;
  int f = p >> 6;
  const int j = f % nt; f /= nt;
  const int t = f % ks; f /= ks;
  const int k = f;
  const int n = 16 * j + (lane & 15);
  const int c0 = 64 * t + 16 * (lane >> 4);
  const int8_t* src = w + ((int64_t)k * cin + c0) * cout + n;
  uint32_t v[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    uint32_t word = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) word |= (uint32_t)(uint8_t)src[(int64_t)(4 * e + b) * cout] << (8 * b);
    v[e] = word;
  }
  packed[p] = make_uint4(v[0], v[1], v[2], v[3]);
}

// F8: 0 = int8 operands, exact int32 accumulation (v_mfma_i32_16x16x64_i8); 1 = E4M3 operands, fp32 accumulation
//     (two v_mfma_f32_16x16x32_fp8_fp8 per 16-byte operand: its low and its high 8 bytes; features and packed weights
//     split the same way, so the contraction pairs the same channels).
// OUTQ: int8 operands: 1 = int8 output (re-quantised), 0 = fp16 output; E4M3 operands: 1 = fp32 output, 0 = fp16 output.
// waves per SIMD the register allocator must leave room for: three where the operands in flight are few
template <int CIN, int COUT> struct QCfg { static constexpr int MINW = (CIN == 64 && COUT == 32) ? 3 : 2; };

template <int F8> struct QAcc { typedef intx4 type; };
template <> struct QAcc<1> { typedef floatx4 type; };

template <int CIN, int COUT, int OUTQ, int F8>
__global__ void __launch_bounds__(kQThreads, (QCfg<CIN, COUT>::MINW))
k_spconv_i8(const int8_t* __restrict__ in, const u32x4* __restrict__ wp, const float* __restrict__ mul,
            const float* __restrict__ add, int relu, float inv_out_scale, const int32_t* __restrict__ nbr,
            const int32_t* __restrict__ d_n_out, int64_t capacity_out, int32_t n_in, int32_t* __restrict__ dev_flags,
            const int8_t* __restrict__ zrow, void* __restrict__ out) {
  constexpr int KS = CIN / 64;                // k-steps per tap
  constexpr int NT = COUT / 16;               // 16-column tiles
  constexpr int MT = 4;                       // 16-row tiles per wave
  constexpr int R = 16 * MT;                  // rows per wave
  constexpr int W16 = KS * NT * 64;           // 16-byte weight pieces per tap
  constexpr int WPT = (W16 + kQThreads - 1) / kQThreads;
  static_assert((W16 & (W16 - 1)) == 0, "piece count is a power of two");
  constexpr int WMASK = W16 - 1;              // surplus threads copy redundantly rather than under a branch
  constexpr int NA = MT * KS;                 // A-operand loads per tap
  constexpr int ES = F8 ? (OUTQ ? 4 : 2) : (OUTQ ? 1 : 2);   // bytes per output element
  constexpr int OCH = COUT * ES / 16;         // 16-byte pieces per output row
  constexpr int OPITCH = (OCH + 1) * 16;      // epilogue tile row pitch in bytes
  __shared__ u32x4 wl[2][W16];
  __shared__ u32x4 otile_s[kQWaves][16 * (OCH + 1)];

  int64_t n_out = *d_n_out;
  if (n_out > capacity_out) n_out = capacity_out;
  // XCD-aware tile assignment: workgroup b runs on XCD b % 8; XCD x takes a contiguous range of tiles
  const int64_t n_tiles = (n_out + kQWaves * R - 1) / (kQWaves * R);
  const int64_t chunk = (n_tiles + 7) / 8;
  const int64_t slot_in_xcd = blockIdx.x / 8;
  const int64_t tile_id = (int64_t)(blockIdx.x % 8) * chunk + slot_in_xcd;
  if (slot_in_xcd >= chunk || tile_id >= n_tiles) return;  // uniform for the block

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int m = lane & 15, q = lane >> 4;
  const int64_t wave_row0 = tile_id * (kQWaves * R) + (int64_t)wave * R;

  // lane l holds the kernel-map entries of row l of this wave's 64 rows
  const bool live = wave_row0 + lane < n_out;
  const int32_t* nrow = nbr + (live ? wave_row0 + lane : 0);
  const int32_t dead = live ? 0 : -1;   // OR-ed into kernel-map entries: rows past n_out have no neighbours
  unsigned long long oob = 0ull;        // lanes that saw an entry outside [0, n_in)

  typedef typename QAcc<F8>::type acc_t;
  acc_t acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[mt][j] = acc_t{0, 0, 0, 0};

  int32_t jq[3][3];         // kernel-map entries of groups g, g+1, g+2 (as loaded; masked where used)
  u32x4 areg[3][NA];        // A operands in flight; tap x lives in set x % 3
  u32x4 wq[3][WPT];         // weights in flight; tap x lives in set x % 3

#define EMC2_IDX_LOAD(GROUP, DST)                                                                        \
  _Pragma("unroll") for (int kx_ = 0; kx_ < 3; ++kx_)                                                    \
      jq[DST][kx_] = nrow[(int64_t)(3 * ((GROUP) < 9 ? (GROUP) : 8) + kx_) * capacity_out];
  // A operands of one tap: tile mt, k-step ks <- 16 bytes at channel 64*ks + 16*q of row JROW[16*mt + m].  Three
  // lane-swap instructions broadcast each 16-lane row of the entries to all four rows.
#define EMC2_A_LOAD(JROW, SET)                                                                           \
  {                                                                                                      \
    const uint32_t jr_ = (uint32_t)(JROW);                                                               \
    const u32x2 h_ = __builtin_amdgcn_permlane32_swap(jr_, jr_, false, false);       /* 0101 | 2323 */   \
    const u32x2 lo_ = __builtin_amdgcn_permlane16_swap(h_[0], h_[0], false, false);  /* 0000 | 1111 */   \
    const u32x2 hi_ = __builtin_amdgcn_permlane16_swap(h_[1], h_[1], false, false);  /* 2222 | 3333 */   \
    const int32_t jm_[4] = {(int32_t)lo_[0], (int32_t)lo_[1], (int32_t)hi_[0], (int32_t)hi_[1]};         \
  _Pragma("unroll") for (int mt_ = 0; mt_ < MT; ++mt_) {                                                 \
    const int32_t j_ = jm_[mt_];                                                                         \
    const int8_t* src_ = (j_ >= 0 ? in + (int64_t)j_ * CIN : zrow) + 16 * q;                             \
    _Pragma("unroll") for (int ks_ = 0; ks_ < KS; ++ks_)                                                 \
        areg[SET][mt_ * KS + ks_] = *reinterpret_cast<const u32x4*>(src_ + 64 * ks_);                    \
  }                                                                                                      \
  }
#define EMC2_W_LOAD(TAP, SET)                                                                            \
  {                                                                                                      \
    const u32x4* wsrc_ = wp + (int64_t)(TAP) * W16;                                                      \
    _Pragma("unroll") for (int i_ = 0; i_ < WPT; ++i_)                                                   \
        wq[SET][i_] = wsrc_[(threadIdx.x + i_ * kQThreads) & WMASK];                                     \
  }
#define EMC2_W_STORE(BUF, SET)                                                                           \
  _Pragma("unroll") for (int i_ = 0; i_ < WPT; ++i_)                                                     \
      wl[BUF][(threadIdx.x + i_ * kQThreads) & WMASK] = wq[SET][i_];

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
      EMC2_W_LOAD(tap + 3 < 27 ? tap + 3 : 26, kx)   // weights of tap + 3: global -> registers
      const u32x4* wb = wl[tap & 1];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        u32x4 b[NT];
#pragma unroll
        for (int j = 0; j < NT; ++j) b[j] = wb[(ks * NT + j) * 64 + lane];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int j = 0; j < NT; ++j) {
            if constexpr (F8) {
              const u32x4 av = areg[kx][mt * KS + ks], bv = b[j];
              const long a_lo = (long)(((unsigned long)av.y << 32) | av.x), a_hi = (long)(((unsigned long)av.w << 32) | av.z);
              const long b_lo = (long)(((unsigned long)bv.y << 32) | bv.x), b_hi = (long)(((unsigned long)bv.w << 32) | bv.z);
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a_lo, b_lo, acc[mt][j], 0, 0, 0);
              acc[mt][j] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a_hi, b_hi, acc[mt][j], 0, 0, 0);
            } else {
              acc[mt][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(intx4, areg[kx][mt * KS + ks]),
                                                                 __builtin_bit_cast(intx4, b[j]), acc[mt][j], 0, 0, 0);
            }
          }
      }
      // the freed register set takes the A operands of tap + 3 (entries of "group 9" do not exist)
      const int32_t past = g < 8 ? 0 : -1;
      EMC2_A_LOAD(emc2_entry(jq[1][kx], dead | past, n_in, oob), kx)
      __builtin_amdgcn_wave_barrier();
      // weights of tap + 1: registers -> the other LDS buffer; the barrier publishes them and retires the one just read
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

  // epilogue: lane (m, q) holds column 16*j + m of rows 16*mt + 4*q + e.  int -> fp32, multiply, add (each rounded
  // on its own), ReLU, convert; each 16-row tile goes through LDS so that global stores are whole 16-byte pieces.
  float ml[NT], ad[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    ml[j] = mul[16 * j + m];
    ad[j] = add[16 * j + m];
  }
  uint8_t* otile = reinterpret_cast<uint8_t*>(otile_s[wave]);
  constexpr int OPI = 64 / OCH;               // rows one store instruction covers
  constexpr int ONI = (16 + OPI - 1) / OPI;   // store instructions per 16-row tile
  const int orow = lane / OCH, ochunk = lane % OCH;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float v = (float)acc[mt][j][e];
        v = v * ml[j];
        v = v + ad[j];
        if (relu) v = v > 0.f ? v : 0.f;
        uint8_t* dst = otile + (4 * q + e) * OPITCH + (16 * j + m) * ES;
        if (F8 && OUTQ) *reinterpret_cast<float*>(dst) = v;
        else if (OUTQ) *reinterpret_cast<int8_t*>(dst) = (int8_t)quant_i8(v, inv_out_scale);
        else *reinterpret_cast<uint16_t*>(dst) = __half_as_ushort(__float2half_rn(v));
      }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < ONI; ++i) {
      const int r = i * OPI + orow;
      if (r < 16) {
        const u32x4 piece = *reinterpret_cast<const u32x4*>(otile + r * OPITCH + ochunk * 16);
        const int64_t o = wave_row0 + mt * 16 + r;
        if (o < n_out) *reinterpret_cast<u32x4*>(reinterpret_cast<uint8_t*>(out) + o * (COUT * ES) + ochunk * 16) = piece;
      }
    }
    __builtin_amdgcn_wave_barrier();
  }
}

template <int CIN, int COUT, int OUTQ, int F8 = 0>
void launch_i8(const void* d_in, const void* d_wp, const float* d_mul, const float* d_add, int relu, float inv_out_scale,
               const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int32_t n_in, int32_t* dev_flags,
               const void* d_zero_row, void* d_out, hipStream_t s) {
  const int64_t rows_per_block = kQWaves * 64;
  hipLaunchKernelGGL((k_spconv_i8<CIN, COUT, OUTQ, F8>), dim3((unsigned)(emc2_div_up(capacity_out, rows_per_block) + 8)),
                     dim3(kQThreads), 0, s, (const int8_t*)d_in, (const u32x4*)d_wp, d_mul, d_add, relu, inv_out_scale, d_nbr,
                     d_n_out, capacity_out, n_in, dev_flags, (const int8_t*)d_zero_row, d_out);
}

bool i8_shape_ok(int cin, int cout) { return (cin == 64 || cin == 128) && (cout == 32 || cout == 64); }

}  // namespace

extern "C" int32_t emc2_spconv_i8_supported(int32_t cin, int32_t cout) { return i8_shape_ok(cin, cout) ? 1 : 0; }

extern "C" emc2_status emc2_quantize_i8(emc2_ctx* ctx, emc2_dtype dtype, const void* d_x, int64_t n, float inv_scale,
                                        int8_t* d_q, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (n < 0 || (n > 0 && (!d_x || !d_q))) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_quantize_i8: bad argument");
  if (!(inv_scale == inv_scale)) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_quantize_i8: inv_scale is not a number");
  if (n == 0) return EMC2_OK;
  const dim3 grid((unsigned)emc2_div_up(n, 256)), blk(256);
  hipStream_t s = (hipStream_t)stream;
  if (dtype == EMC2_F32) hipLaunchKernelGGL(k_quantize_i8<float>, grid, blk, 0, s, (const float*)d_x, n, inv_scale, d_q);
  else if (dtype == EMC2_F16) hipLaunchKernelGGL(k_quantize_i8<__half>, grid, blk, 0, s, (const __half*)d_x, n, inv_scale, d_q);
  else return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_quantize_i8: input must be F32 or F16");
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_quantize_i8 launch");
}

extern "C" emc2_status emc2_pack_weights_i8(emc2_ctx* ctx, const int8_t* d_w, int32_t cin, int32_t cout, void* d_packed,
                                            void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_w || !d_packed) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_pack_weights_i8: null argument");
  if (!i8_shape_ok(cin, cout))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_pack_weights_i8: Cin must be 64 or 128 and Cout 32 or 64");
  const int total = 27 * (cin / 64) * (cout / 16) * 64;
  hipLaunchKernelGGL(k_pack_weights_i8, dim3((unsigned)emc2_div_up(total, 256)), dim3(256), 0, (hipStream_t)stream, d_w, cin,
                     cout, (uint4*)d_packed);
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_pack_weights_i8 launch");
}

extern "C" emc2_status emc2_spconv_i8(emc2_ctx* ctx, const int8_t* d_in, const void* d_w_packed, const float* d_mul,
                                      const float* d_add, int32_t relu, emc2_dtype out_dtype, float inv_out_scale,
                                      const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int64_t n_in_rows,
                                      int32_t cin, int32_t cout, void* d_out, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_in || !d_w_packed || !d_mul || !d_add || !d_nbr || !d_n_out || !d_out)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_i8: null argument");
  if (capacity_out < 1) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_i8: capacity_out < 1");
  if (n_in_rows < 0) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_i8: n_in_rows < 0");
  if (((uintptr_t)d_in | (uintptr_t)d_w_packed | (uintptr_t)d_out) & 15u)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_i8: d_in, d_w_packed and d_out must be 16-byte aligned");
  const int32_t n_in = n_in_rows > 0x7fffffff ? 0x7fffffff : (int32_t)n_in_rows;
  if (!i8_shape_ok(cin, cout))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_spconv_i8: Cin must be 64 or 128 and Cout 32 or 64");
  if (out_dtype != EMC2_I8 && out_dtype != EMC2_F16)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_spconv_i8: output must be I8 or F16");
  if (out_dtype == EMC2_I8 && !(inv_out_scale == inv_out_scale))
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_i8: inv_out_scale is not a number");
  hipStream_t s = (hipStream_t)stream;
  const int rl = relu ? 1 : 0;
#define CASE(CI, CO)                                                                                                        \
  if (cin == CI && cout == CO) {                                                                                            \
    if (out_dtype == EMC2_I8)                                                                                               \
      launch_i8<CI, CO, 1>(d_in, d_w_packed, d_mul, d_add, rl, inv_out_scale, d_nbr, d_n_out, capacity_out, n_in,           \
                           ctx->dev_words, ctx->zero_row, d_out, s);                                                        \
    else                                                                                                                    \
      launch_i8<CI, CO, 0>(d_in, d_w_packed, d_mul, d_add, rl, inv_out_scale, d_nbr, d_n_out, capacity_out, n_in,           \
                           ctx->dev_words, ctx->zero_row, d_out, s);                                                        \
  }
  CASE(64, 32) CASE(64, 64) CASE(128, 32) CASE(128, 64)
#undef CASE
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_spconv_i8 launch");
}

// ---------------------------------------------------------------------------------------------------------
// E4M3 variant: same kernel, same packed-weight byte order (emc2_pack_weights_i8 permutes bytes, whatever they encode)
// ---------------------------------------------------------------------------------------------------------
extern "C" emc2_status emc2_quantize_e4m3(emc2_ctx* ctx, emc2_dtype dtype, const void* d_x, int64_t n, float inv_scale,
                                          uint8_t* d_q, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (n < 0 || (n > 0 && (!d_x || !d_q))) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_quantize_e4m3: bad argument");
  if (!(inv_scale == inv_scale)) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_quantize_e4m3: inv_scale is not a number");
  if (n == 0) return EMC2_OK;
  const dim3 grid((unsigned)emc2_div_up(n, 256)), blk(256);
  hipStream_t s = (hipStream_t)stream;
  if (dtype == EMC2_F32) hipLaunchKernelGGL(k_quantize_e4m3<float>, grid, blk, 0, s, (const float*)d_x, n, inv_scale, d_q);
  else if (dtype == EMC2_F16) hipLaunchKernelGGL(k_quantize_e4m3<__half>, grid, blk, 0, s, (const __half*)d_x, n, inv_scale, d_q);
  else return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_quantize_e4m3: input must be F32 or F16");
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_quantize_e4m3 launch");
}

extern "C" emc2_status emc2_spconv_e4m3(emc2_ctx* ctx, const uint8_t* d_in, const void* d_w_packed, const float* d_mul,
                                        const float* d_add, int32_t relu, emc2_dtype out_dtype, const int32_t* d_nbr,
                                        const int32_t* d_n_out, int64_t capacity_out, int64_t n_in_rows, int32_t cin,
                                        int32_t cout, void* d_out, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!d_in || !d_w_packed || !d_mul || !d_add || !d_nbr || !d_n_out || !d_out)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_e4m3: null argument");
  if (capacity_out < 1) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_e4m3: capacity_out < 1");
  if (n_in_rows < 0) return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_e4m3: n_in_rows < 0");
  if (((uintptr_t)d_in | (uintptr_t)d_w_packed | (uintptr_t)d_out) & 15u)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_spconv_e4m3: d_in, d_w_packed and d_out must be 16-byte aligned");
  if (!i8_shape_ok(cin, cout))
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_spconv_e4m3: Cin must be 64 or 128 and Cout 32 or 64");
  if (out_dtype != EMC2_F32 && out_dtype != EMC2_F16)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_spconv_e4m3: output must be F32 or F16");
  const int32_t n_in = n_in_rows > 0x7fffffff ? 0x7fffffff : (int32_t)n_in_rows;
  hipStream_t s = (hipStream_t)stream;
  const int rl = relu ? 1 : 0;
#define CASE(CI, CO)                                                                                                         \
  if (cin == CI && cout == CO) {                                                                                             \
    if (out_dtype == EMC2_F32)                                                                                               \
      launch_i8<CI, CO, 1, 1>(d_in, d_w_packed, d_mul, d_add, rl, 0.f, d_nbr, d_n_out, capacity_out, n_in, ctx->dev_words,   \
                              ctx->zero_row, d_out, s);                                                                      \
    else                                                                                                                     \
      launch_i8<CI, CO, 0, 1>(d_in, d_w_packed, d_mul, d_add, rl, 0.f, d_nbr, d_n_out, capacity_out, n_in, ctx->dev_words,   \
                              ctx->zero_row, d_out, s);                                                                      \
  }
  CASE(64, 32) CASE(64, 64) CASE(128, 32) CASE(128, 64)
#undef CASE
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_spconv_e4m3 launch");
}
