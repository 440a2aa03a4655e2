// Internal interface of the MFMA sparse-conv kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "emc2.h"

// true iff (cin, cout) is covered by an MFMA instantiation (16-bit dtypes only)
bool emc2_spconv_mfma_supported(int cin, int cout);

// Re-order W[27][Cin][Cout] (16-bit) into MFMA B-fragment order (same byte size).
void emc2_spconv_mfma_pack(const void* d_w, int cin, int cout, void* d_packed, hipStream_t stream);

// d_wp: weights already in fragment order.
// n_in: rows of d_in; a kernel-map entry outside [0, n_in) is treated as absent and raises EMC2_DEVFLAG_MAP in
// *dev_flags (the same two arguments on every launcher below).
void emc2_spconv_mfma_launch(emc2_dtype dtype, const void* d_in, const void* d_wp, const float* d_scale,
                             const float* d_shift, int epilogue, const int32_t* d_nbr, const int32_t* d_n_out,
                             int64_t capacity_out, int32_t n_in, int32_t* dev_flags, int cin, int cout, void* d_out,
                             hipStream_t stream);

// Span-gather variant (one contiguous fetch of input rows per group of three kx taps): profitable for
// kernel maps whose three kx taps name nearly the same rows (submanifold maps over voxels sorted by key).
// Same arguments and results as emc2_spconv_mfma_launch.
bool emc2_spconv_span_supported(int cin, int cout);
void emc2_spconv_span_launch(emc2_dtype dtype, const void* d_in, const void* d_wp, const float* d_scale,
                             const float* d_shift, int epilogue, const int32_t* d_nbr, const int32_t* d_n_out,
                             int64_t capacity_out, int32_t n_in, int32_t* dev_flags, int cin, int cout, void* d_out,
                             hipStream_t stream);

// Register-direct variant (A operands straight from global memory, 16x16x32 MFMA; LDS holds weights only).
// Its packed weight layout differs from the other kernels': shapes it supports are packed by
// emc2_spconv_direct_pack and always run on it.  d_zero_row: >= 256 zero bytes in device memory.
bool emc2_spconv_direct_supported(int cin, int cout);
void emc2_spconv_direct_pack(const void* d_w, int cin, int cout, void* d_packed, hipStream_t stream);
void emc2_spconv_direct_launch(emc2_dtype dtype, const void* d_in, const void* d_wp, const float* d_scale,
                               const float* d_shift, int epilogue, const int32_t* d_nbr, const int32_t* d_n_out,
                               int64_t capacity_out, int32_t n_in, int32_t* dev_flags, int cin, int cout,
                               const void* d_zero_row, void* d_out, hipStream_t stream);
