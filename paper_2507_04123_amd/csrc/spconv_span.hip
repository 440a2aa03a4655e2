// Span-gather variant of the MFMA sparse convolution (paper Sec. 3.5 sparse convolution over the
// non-empty voxels; Sec. 3.6 keeping data on chip between dependent steps).
//
// Voxels are indexed in ascending order of their linear cell key (x fastest).  The three taps of one
// (dz, dy) pair -- kx = 0, 1, 2 -- therefore read input rows that differ by one position along x: for a
// run of 64 consecutive output rows they touch nearly the same short interval [lo, hi] of input rows
// (in a submanifold layer 66 rows at the median).  This kernel fetches that interval ONCE per group of
// three taps, as one contiguous block of feature rows, into a wave-private LDS tile; each tap then
// reads its A operand from the tile through a per-lane row index (kernel-map entry minus lo).  Absent
// neighbours point at a zeroed row of the tile.  Compared with one gather per tap this moves ~2.5x
// fewer bytes through the vector L1 / L2 and writes the LDS tile once instead of three times.
//
// When the interval does not fit the tile (kernel maps of strided layers; a few percent of the
// groups elsewhere) the group falls back to three passes, one per tap, each gathering exactly the 64
// rows its tap names.  Results never depend on which mode a group took: the mode is chosen from the
// table entries themselves, and every entry is range-checked against the tile before use.
//
// Block = 8 waves (one per 64 output rows) sharing the weights of a group (3 taps) in a double-buffered
// LDS area: one block-wide barrier per group.  All global loads of a group are issued in one burst
// right after the tile has been written, a whole group (thousands of cycles) before their first use.
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

template <int DT> struct MmaS;
template <> struct MmaS<EMC2_F16> {
  static __device__ __forceinline__ floatx4 run(u32x4 a, u32x4 b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float v) { return __half_as_ushort(__float2half_rn(v)); }
};
template <> struct MmaS<EMC2_BF16> {
  static __device__ __forceinline__ floatx4 run(u32x4 a, u32x4 b, floatx4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t cvt(float v) { return __builtin_bit_cast(uint16_t, __float2bfloat16(v)); }
};

constexpr int kSpanWaves = 8;
constexpr int kSpanThreads = kSpanWaves * 64;

template <int CIN> struct SpanCfg {
  // rows of the LDS tile (a multiple of the rows one load instruction covers); sized so that 8 tiles and
  // two weight buffers fit the 160 KB of LDS
  static constexpr int SMAX = 80;
  // waves per SIMD the register allocator must leave room for
  static constexpr int MINW = 2;
};

// What a group of three taps needs from the input: the interval [lo, hi] of rows its valid entries name
// (wave-uniform), and whether every valid entry lies inside [lo, lo + SMAX).
struct GroupInfo {
  int32_t lo, hi;
  bool span;
  uint32_t rows;   // span mode: rows of the interval that hold data (0 for a group without a valid entry)
  unsigned long long valid[3];
};

template <int SMAX>
__device__ __forceinline__ GroupInfo analyze(const int32_t j[3]) {
  GroupInfo gi;
  int32_t lo = 0x7fffffff, hi = 0;
#pragma unroll
  for (int kx = 0; kx < 3; ++kx) {
    const unsigned long long mk = __ballot(j[kx] >= 0);
    gi.valid[kx] = mk;
    // a table from emc2_build_kmap is ascending in the row index wherever it is valid, so the first and last
    // valid lanes hold the extremes; in any other table some entry falls outside [lo, hi], fails the range
    // check below, and the group takes the three-pass route
    const int first = mk ? __builtin_ctzll(mk) : 0;
    const int last = mk ? 63 - __builtin_clzll(mk) : 0;
    const int32_t vf = __builtin_amdgcn_readlane(j[kx], first);
    const int32_t vl = __builtin_amdgcn_readlane(j[kx], last);
    if (mk) {
      lo = vf < lo ? vf : lo;
      hi = vl > hi ? vl : hi;
    }
  }
  if (lo == 0x7fffffff) lo = 0;
  if (hi < lo) hi = lo;
  // rows past hi are not fetched (the gather clamps to hi), so an entry is usable in span mode only inside
  // [lo, hi], and the interval must fit the tile
  const uint32_t width = (uint32_t)(hi - lo);
  unsigned long long bad = width >= (uint32_t)SMAX ? ~0ull : 0ull;
#pragma unroll
  for (int kx = 0; kx < 3; ++kx) bad |= __ballot(j[kx] >= 0 && (uint32_t)(j[kx] - lo) > width);
  gi.lo = lo;
  gi.hi = hi;
  gi.span = bad == 0ull;
  gi.rows = (gi.valid[0] | gi.valid[1] | gi.valid[2]) != 0ull ? width + 1u : 0u;
  return gi;
}

// The main loop of one wave.  LATE = false: a group's interval is  [tile write, request loads] -> compute;
// LATE = true:  compute -> [tile write for the next group, request loads for the one after].  Both kinds
// meet at the same block-wide barrier once per group, but between two barriers they do their memory
// phase and their matrix phase in opposite order, so the two waves that share a SIMD (wave w and w + 4)
// do not both want the LDS / the load path / the matrix core at the same time.
template <int DT, int CIN, int COUT, bool LATE>
__device__ __forceinline__ void span_wave(const uint16_t* __restrict__ in, const u32x4* __restrict__ wp,
                                          const float* __restrict__ scale, const float* __restrict__ shift, int epilogue,
                                          const int32_t* __restrict__ nbr, int64_t n_out, int64_t capacity_out,
                                          int32_t n_in, int32_t* __restrict__ dev_flags,
                                          uint16_t* __restrict__ out, u32x4* __restrict__ wl, u32x4* __restrict__ my_tile,
                                          int64_t wave_row0) {
  constexpr int KS = CIN / 32;                // k-steps per tap (v_mfma_f32_16x16x32)
  constexpr int NT = COUT / 16;               // 16-column tiles
  constexpr int MT = 4;                       // 16-row tiles per wave
  constexpr int W16 = KS * NT * 64;           // 16-byte weight pieces per tap
  constexpr int G16 = 3 * W16;                // ... per group of three taps
  constexpr int WPT = (G16 + kSpanThreads - 1) / kSpanThreads;
  constexpr int CH = CIN / 8;                 // 16-byte chunks per feature row
  constexpr int RPI = 64 / CH;                // rows covered by one load instruction
  constexpr int SMAX = SpanCfg<CIN>::SMAX;
  constexpr int NI = SMAX / RPI;              // load instructions per gather
  constexpr int ROW16 = CH + 1;               // LDS row pitch in 16-byte units (one unit of padding)
  constexpr int ZROW = SMAX;                  // the zeroed row absent neighbours read

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int m = lane & 15, q = lane >> 4;
  if (lane < ROW16) my_tile[ZROW * ROW16 + lane] = u32x4{0u, 0u, 0u, 0u};

  const bool live = wave_row0 + lane < n_out;
  const int32_t* nrow = nbr + (live ? wave_row0 + lane : 0);
  const int32_t dead = live ? 0 : -1;               // rows past n_out have no neighbours
  unsigned long long oob = 0ull;                    // lanes that saw an entry outside [0, n_in)
  const int srow = lane / CH, schunk = lane % CH;   // gather role: row within an instruction, 16-byte chunk

  floatx4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int j = 0; j < NT; ++j) acc[mt][j] = floatx4{0.f, 0.f, 0.f, 0.f};

  // kernel-map entries (lane = row) of the group being computed, the next, and (LATE) the one after, as
  // loaded: rows past n_out are masked where the entries are used, never right after the load (that would
  // wait for the load at once)
  int32_t jq0[3], jq1[3], jq2[3];
  u32x4 sreg[NI];           // gathered rows in flight (an instruction that is skipped leaves its slot as it was)
#pragma unroll
  for (int i = 0; i < NI; ++i) sreg[i] = u32x4{0u, 0u, 0u, 0u};
  u32x4 wq[WPT];            // weights in flight

#define EMC2_IDX_LOAD(GROUP, DST)                                                                          \
  _Pragma("unroll") for (int kx_ = 0; kx_ < 3; ++kx_)                                                      \
      DST[kx_] = nrow[(int64_t)(3 * ((GROUP) < 9 ? (GROUP) : 8) + kx_) * capacity_out];
#define EMC2_MASKED(C, J)                                                                                  \
  const int32_t C[3] = {emc2_entry(J[0], dead, n_in, oob), emc2_entry(J[1], dead, n_in, oob),              \
                        emc2_entry(J[2], dead, n_in, oob)};
#define EMC2_W_LOAD(GROUP)                                                                                 \
  {                                                                                                        \
    const u32x4* wsrc_ = wp + (int64_t)((GROUP) < 9 ? (GROUP) : 8) * G16;                                  \
    _Pragma("unroll") for (int i_ = 0; i_ < WPT; ++i_) {                                                   \
      const int p_ = tid + i_ * kSpanThreads;                                                              \
      wq[i_] = wsrc_[p_ < G16 ? p_ : G16 - 1];                                                             \
    }                                                                                                      \
  }
#define EMC2_W_STORE(BUF)                                                                                  \
  _Pragma("unroll") for (int i_ = 0; i_ < WPT; ++i_) {                                                     \
    const int p_ = tid + i_ * kSpanThreads;                                                                \
    wl[(BUF) * G16 + (p_ < G16 ? p_ : G16 - 1)] = wq[i_]; /* surplus threads rewrite the last piece */     \
  }
  // gather of the interval [lo, hi] (rows past hi re-read row hi and are never referenced)
#define EMC2_GATHER_SPAN(GI)                                                                               \
  {                                                                                                        \
    /* wave-uniform base (scalar registers) + a small per-lane byte offset */                              \
    const char* base_ = reinterpret_cast<const char*>(in) + (int64_t)(GI).lo * (CIN * 2);                  \
    const uint32_t last_ = (uint32_t)((GI).hi - (GI).lo);                                                  \
    _Pragma("unroll") for (int i_ = 0; i_ < NI; ++i_) {                                                    \
      /* wave-uniform: an instruction none of whose rows holds data is not issued (its tile rows are never read) */ \
      if ((uint32_t)(i_ * RPI) < (GI).rows) {                                                              \
        const uint32_t p_ = (uint32_t)(i_ * RPI + srow);                                                   \
        const uint32_t off_ = (p_ < last_ ? p_ : last_) * (uint32_t)(CIN * 2) + (uint32_t)(schunk * 16);   \
        sreg[i_] = *reinterpret_cast<const u32x4*>(base_ + off_);                                          \
      }                                                                                                    \
    }                                                                                                      \
  }
  // gather of exactly the rows one tap names: tile row p <- input row JROW[p] (absent entries re-read row 0)
#define EMC2_GATHER_TAP(JROW)                                                                              \
  _Pragma("unroll") for (int i_ = 0; i_ < NI; ++i_) {                                                      \
    if (i_ * RPI < 64) { /* compile time: a tap names 64 rows */                                           \
      const int p_ = i_ * RPI + srow;                                                                      \
      const int32_t j_ = __shfl((JROW), p_, 64);                                                           \
      sreg[i_] = *(reinterpret_cast<const u32x4*>(in + (int64_t)(j_ >= 0 ? j_ : 0) * CIN) + schunk);       \
    }                                                                                                      \
  }
#define EMC2_GATHER_MAIN(GI, J)                                                                            \
  if ((GI).span) { EMC2_GATHER_SPAN(GI) } else { EMC2_GATHER_TAP((J)[0]) }
  // registers -> tile, the first ROWS rows (wave-uniform; whole instructions)
#define EMC2_TILE_WRITE_N(ROWS)                                                                            \
  _Pragma("unroll") for (int i_ = 0; i_ < NI; ++i_)                                                        \
    if ((uint32_t)(i_ * RPI) < (uint32_t)(ROWS)) my_tile[(i_ * RPI + srow) * ROW16 + schunk] = sreg[i_];
  // ... what the main gather of group GI left in the registers: its interval, or the 64 rows of its first tap
#define EMC2_TILE_WRITE(GI) EMC2_TILE_WRITE_N((GI).span ? (GI).rows : 64u)
  // Issue order inside a tap (KS = 2, MT = NT = 4: 16 operand reads, 32 matrix instructions): operands are read one
  // to two row tiles ahead of the matrix instructions that use them, so that after the first six reads of a tap a
  // read's latency falls under the four matrix instructions before its use.
#define EMC2_TAP_ORDER()                                                                                   \
  if (KS == 2 && MT == 4 && NT == 4) {                                                                     \
    __builtin_amdgcn_sched_group_barrier(0x100, 6, 0); /* b0..b3, a0, a1 of the first k-step */            \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0); __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);  \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0); __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  \
    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0); __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  \
    __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);                                                     \
  }
  // one tap: lane l's LROW is the tile row that output row l of the wave reads.  The A operand of lane
  // (m, q) for tile mt is 16 bytes at piece 4*ks + q of tile row LROW[16*mt + m]: three lane-swap
  // instructions broadcast each 16-lane row of LROW to all four rows (no LDS round trip).
#define EMC2_TAP(KX, LROW, WB)                                                                             \
  {                                                                                                        \
    const uint32_t lr_ = (uint32_t)(LROW);                                                                 \
    const u32x2 h_ = __builtin_amdgcn_permlane32_swap(lr_, lr_, false, false);        /* rows 0101 | 2323 */ \
    const u32x2 lo_ = __builtin_amdgcn_permlane16_swap(h_[0], h_[0], false, false);   /* 0000 | 1111 */    \
    const u32x2 hi_ = __builtin_amdgcn_permlane16_swap(h_[1], h_[1], false, false);   /* 2222 | 3333 */    \
    const u32x4* ap_[MT] = {my_tile + lo_[0] * ROW16 + q, my_tile + lo_[1] * ROW16 + q,                    \
                            my_tile + hi_[0] * ROW16 + q, my_tile + hi_[1] * ROW16 + q};                   \
    _Pragma("unroll") for (int t = 0; t < KS; ++t) {                                                       \
      u32x4 b[NT], a[MT];                                                                                  \
      _Pragma("unroll") for (int j = 0; j < NT; ++j) b[j] = (WB)[(((KX) * KS + t) * NT + j) * 64 + lane];  \
      _Pragma("unroll") for (int mt = 0; mt < MT; ++mt) a[mt] = ap_[mt][4 * t];                            \
      _Pragma("unroll") for (int mt = 0; mt < MT; ++mt)                                                    \
        _Pragma("unroll") for (int j = 0; j < NT; ++j) acc[mt][j] = MmaS<DT>::run(a[mt], b[j], acc[mt][j]); \
    }                                                                                                      \
    EMC2_TAP_ORDER()                                                                                       \
  }
  // Tile row that output row `lane` reads at tap KX.  Span mode: entry minus lo.  Three-pass mode: the
  // tile holds exactly the rows of the tap being computed, row p for output row p.
#define EMC2_LROW(KX, C, GI) ((C)[KX] >= 0 ? ((GI).span ? (C)[KX] - (GI).lo : lane) : ZROW)
  // The three taps are straight-line code: with branches between the matrix instructions of a group the
  // compiler keeps two copies of the accumulators and moves 64 registers back and forth at every join.
  // Only the memory operations of the (rare) three-pass mode are conditional inside a group.
#define EMC2_COMPUTE(C, GI, NXT, CNXT, WB)                                                                 \
  {                                                                                                        \
    __builtin_amdgcn_s_setprio(2);                                                                         \
    { const int32_t lrow_ = EMC2_LROW(0, C, GI); EMC2_TAP(0, lrow_, WB) }                                  \
    __builtin_amdgcn_wave_barrier();                                                                       \
    if (!(GI).span) { EMC2_TILE_WRITE_N(64) EMC2_GATHER_TAP((C)[2]) }                                          \
    __builtin_amdgcn_wave_barrier();                                                                       \
    { const int32_t lrow_ = EMC2_LROW(1, C, GI); EMC2_TAP(1, lrow_, WB) }                                  \
    __builtin_amdgcn_wave_barrier();                                                                       \
    if (!(GI).span) { EMC2_TILE_WRITE_N(64) EMC2_GATHER_MAIN(NXT, CNXT) }                                      \
    __builtin_amdgcn_wave_barrier();                                                                       \
    { const int32_t lrow_ = EMC2_LROW(2, C, GI); EMC2_TAP(2, lrow_, WB) }                                  \
    __builtin_amdgcn_s_setprio(0);                                                                         \
  }
  // prologue.  The analyses of the groups (wave-uniform, ~80 scalar instructions each) are carried from
  // iteration to iteration, one new analysis per group, always of entries loaded a whole group earlier.
  EMC2_IDX_LOAD(0, jq0)
  EMC2_IDX_LOAD(1, jq1)
  EMC2_W_LOAD(0)
  EMC2_W_STORE(0)
  GroupInfo cur, nxt, aft;
  {
    EMC2_MASKED(c0, jq0)
    EMC2_MASKED(c1, jq1)
    cur = analyze<SMAX>(c0);
    nxt = analyze<SMAX>(c1);
    aft = nxt;
    EMC2_GATHER_MAIN(cur, c0)
    if constexpr (LATE) {
      // one interval ahead on the memory side: first pass of group 0 in the tile, next pass requested
      EMC2_TILE_WRITE(cur)
      EMC2_IDX_LOAD(2, jq2)
      EMC2_W_LOAD(1)
      if (cur.span) { EMC2_GATHER_MAIN(nxt, c1) } else { EMC2_GATHER_TAP(c0[1]) }
    }
  }
  __syncthreads();

  for (int g = 0; g < 9; ++g) {
    const u32x4* wb = wl + (g & 1) * G16;
    EMC2_MASKED(c0, jq0)
    EMC2_MASKED(c1, jq1)
    if constexpr (!LATE) {
      EMC2_TILE_WRITE(cur)                    // rows of group g, requested during group g - 1
      // requests: entries of group g + 2, weights of group g + 1, and the rows of the next pass (group
      // g + 1, or the second pass of this group if it runs in three passes)
      EMC2_IDX_LOAD(g + 2, jq2)
      EMC2_W_LOAD(g + 1)
      if (cur.span) { EMC2_GATHER_MAIN(nxt, c1) } else { EMC2_GATHER_TAP(c0[1]) }
      __builtin_amdgcn_wave_barrier();
      // a group none of whose 192 entries is valid costs no LDS read and no matrix instruction
      if (((cur.valid[0] | cur.valid[1] | cur.valid[2]) != 0ull) || !cur.span) {
        EMC2_COMPUTE(c0, cur, nxt, c1, wb)
      }
      __builtin_amdgcn_wave_barrier();
      EMC2_W_STORE((g + 1) & 1)               // weights of group g + 1 -> the LDS buffer group g - 1 used
      {
        EMC2_MASKED(c2, jq2)                  // requested at the top of this group
        cur = nxt;
        nxt = analyze<SMAX>(c2);
      }
    } else {
      // tile holds group g (first pass); registers hold the rows of the next pass; wq holds W(g + 1)
      // a group none of whose 192 entries is valid costs no LDS read and no matrix instruction
      if (((cur.valid[0] | cur.valid[1] | cur.valid[2]) != 0ull) || !cur.span) {
        EMC2_COMPUTE(c0, cur, nxt, c1, wb)
      }
      __builtin_amdgcn_wave_barrier();
      EMC2_MASKED(c2, jq2)                    // requested at the end of the previous group
      aft = analyze<SMAX>(c2);
      EMC2_W_STORE((g + 1) & 1)
      EMC2_TILE_WRITE(nxt)                    // first pass of group g + 1
      int32_t jn[3];
      EMC2_IDX_LOAD(g + 3, jn)
      EMC2_W_LOAD(g + 2)
      // rows of the pass after that: second pass of group g + 1 if it runs in three passes, else group g + 2
      if (nxt.span) { EMC2_GATHER_MAIN(aft, c2) } else { EMC2_GATHER_TAP(c1[1]) }
      cur = nxt;
      nxt = aft;
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) {
        jq0[kx] = jq1[kx];
        jq1[kx] = jq2[kx];
        jq2[kx] = jn[kx];
      }
    }
    __syncthreads();                          // publishes W(g + 1), retires the buffer just read
    if constexpr (!LATE) {
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) {
        jq0[kx] = jq1[kx];
        jq1[kx] = jq2[kx];
      }
    }
  }
#undef EMC2_IDX_LOAD
#undef EMC2_MASKED
#undef EMC2_W_LOAD
#undef EMC2_W_STORE
#undef EMC2_GATHER_SPAN
#undef EMC2_GATHER_TAP
#undef EMC2_GATHER_MAIN
#undef EMC2_TILE_WRITE
#undef EMC2_TILE_WRITE_N
#undef EMC2_TAP
#undef EMC2_TAP_ORDER
#undef EMC2_LROW
#undef EMC2_COMPUTE
  emc2_report_oob(oob, dev_flags);

  // epilogue: lane (m, q) holds column 16*j + m of rows 16*mt + 4*q + e.  Scale/shift/ReLU/convert in
  // registers, then each 16-row tile goes through the wave's LDS tile so that the global stores are whole
  // 16-byte pieces of rows.
  float sc[NT], sh[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    sc[j] = (epilogue != EMC2_EPI_NONE) ? scale[16 * j + m] : 1.f;
    sh[j] = (epilogue != EMC2_EPI_NONE) ? shift[16 * j + m] : 0.f;
  }
  uint16_t* otile = reinterpret_cast<uint16_t*>(my_tile);
  constexpr int OCH = COUT / 8;               // 16-byte pieces per output row
  constexpr int OPITCH = (OCH + 1) * 8;       // LDS row pitch in 16-bit units
  constexpr int OPI = 64 / OCH;               // rows one store instruction covers
  constexpr int ONI = (16 + OPI - 1) / OPI;   // store instructions per 16-row tile
  static_assert(16 * (OCH + 1) <= (SMAX + 1) * ROW16, "a 16-row output tile fits the gather tile");
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
        otile[(4 * q + e) * OPITCH + 16 * j + m] = MmaS<DT>::cvt(v);
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
__global__ void __launch_bounds__(kSpanThreads, (SpanCfg<CIN>::MINW))
k_spconv_span(const uint16_t* __restrict__ in, const u32x4* __restrict__ wp, const float* __restrict__ scale,
              const float* __restrict__ shift, int epilogue, const int32_t* __restrict__ nbr,
              const int32_t* __restrict__ d_n_out, int64_t capacity_out, int32_t n_in, int32_t* __restrict__ dev_flags,
              uint16_t* __restrict__ out) {
  constexpr int G16 = 3 * (CIN / 32) * (COUT / 16) * 64;
  constexpr int SMAX = SpanCfg<CIN>::SMAX;
  constexpr int ROW16 = CIN / 8 + 1;
  static_assert(SMAX % (64 / (CIN / 8)) == 0 && SMAX >= 64, "the tile holds whole load instructions and at least the 64 rows of a pass");
  __shared__ u32x4 wl[2 * G16];
  __shared__ u32x4 tile[kSpanWaves][(SMAX + 1) * ROW16];

  int64_t n_out = *d_n_out;
  if (n_out > capacity_out) n_out = capacity_out;
  // XCD-aware tile assignment: workgroup b runs on XCD b % 8; XCD x takes a contiguous range of tiles
  const int64_t n_tiles = (n_out + kSpanWaves * 64 - 1) / (kSpanWaves * 64);
  const int64_t chunk = (n_tiles + 7) / 8;
  const int64_t slot_in_xcd = blockIdx.x / 8;
  const int64_t tile_id = (int64_t)(blockIdx.x % 8) * chunk + slot_in_xcd;
  if (slot_in_xcd >= chunk || tile_id >= n_tiles) return;  // uniform for the block
  const int wave = threadIdx.x >> 6;
  const int64_t wave_row0 = tile_id * (kSpanWaves * 64) + (int64_t)wave * 64;
  // waves w and w + 4 share a SIMD: one of each kind per SIMD
  if (wave < 4)
    span_wave<DT, CIN, COUT, false>(in, wp, scale, shift, epilogue, nbr, n_out, capacity_out, n_in, dev_flags, out, wl,
                                    tile[wave], wave_row0);
  else
    span_wave<DT, CIN, COUT, true>(in, wp, scale, shift, epilogue, nbr, n_out, capacity_out, n_in, dev_flags, out, wl,
                                    tile[wave], wave_row0);
}

template <int DT, int CIN, int COUT>
void launch_span(const void* d_in, const void* d_wp, const float* d_scale, const float* d_shift, int epilogue,
                 const int32_t* d_nbr, const int32_t* d_n_out, int64_t capacity_out, int32_t n_in, int32_t* dev_flags,
                 void* d_out, hipStream_t s) {
  const int64_t rows_per_block = kSpanWaves * 64;
  hipLaunchKernelGGL((k_spconv_span<DT, CIN, COUT>), dim3((unsigned)(emc2_div_up(capacity_out, rows_per_block) + 8)),
                     dim3(kSpanThreads), 0, s, (const uint16_t*)d_in, (const u32x4*)d_wp, d_scale, d_shift, epilogue, d_nbr,
                     d_n_out, capacity_out, n_in, dev_flags, (uint16_t*)d_out);
}

}  // namespace

// Only (64, 64) is instantiated: at 32 channels the gather is too small a part of a tap for the re-use to pay
// (measured slower than the register-direct kernel).
// Weights: the packed layout of the register-direct kernel (emc2_spconv_direct_pack).
bool emc2_spconv_span_supported(int cin, int cout) { return cin == 64 && cout == 64; }

void emc2_spconv_span_launch(emc2_dtype dtype, const void* d_in, const void* d_wp, const float* d_scale,
                             const float* d_shift, int epilogue, const int32_t* d_nbr, const int32_t* d_n_out,
                             int64_t capacity_out, int32_t n_in, int32_t* dev_flags, int cin, int cout, void* d_out,
                             hipStream_t stream) {
#define CASE(DTV, CI, CO)                                                                                           \
  if (dtype == DTV && cin == CI && cout == CO) {                                                                    \
    launch_span<DTV, CI, CO>(d_in, d_wp, d_scale, d_shift, epilogue, d_nbr, d_n_out, capacity_out, n_in, dev_flags, \
                             d_out, stream);                                                                        \
    return;                                                                                                         \
  }
  CASE(EMC2_F16, 64, 64) CASE(EMC2_BF16, 64, 64)
#undef CASE
}
