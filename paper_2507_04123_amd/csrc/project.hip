// Point -> image projection with bilinear feature gather (paper Sec. 3.1: image features aligned
// with 3D positions for fusion; Fig. 5 caption: zero fill where there is no match).
//
// Half a wavefront (32 lanes) serves one point: every lane repeats the 3x4 projection in fp64 (it
// decides validity and the pixel indices, so it is evaluated in the same precision and operation
// order as the definition, without fused multiply-add), then lane l blends channel pairs
// l, l+32, ... from the four neighbouring HWC pixels with 4-byte loads, so one pixel's C channels
// are read as contiguous 128-byte segments.
#include <hip/hip_fp16.h>

#include "common.h"

#pragma clang fp contract(off)

namespace {

struct ProjMat {
  double m[12];
};

__global__ void __launch_bounds__(256) k_project_gather(const float* __restrict__ points, int stride_f, int64_t n_points,
                                                        ProjMat pm, const __half2* __restrict__ img, int H, int W, int C2,
                                                        __half2* __restrict__ out, uint8_t* __restrict__ valid,
                                                        float2* __restrict__ uv_out) {
  const int64_t i = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);
  const int lane = threadIdx.x & 31;
  if (i >= n_points) return;
  const float* p = points + i * stride_f;
  const double x = (double)p[0], y = (double)p[1], z = (double)p[2];
  const double uu = pm.m[0] * x + pm.m[1] * y + pm.m[2] * z + pm.m[3];
  const double vv = pm.m[4] * x + pm.m[5] * y + pm.m[6] * z + pm.m[7];
  const double ww = pm.m[8] * x + pm.m[9] * y + pm.m[10] * z + pm.m[11];
  bool ok = false;
  double u = 0.0, v = 0.0;
  if (ww > 0.0) {
    u = uu / ww;
    v = vv / ww;
    ok = (u >= 0.0) && (u <= (double)(W - 1)) && (v >= 0.0) && (v <= (double)(H - 1));
  }
  if (lane == 0) {
    valid[i] = ok ? 1 : 0;
    if (uv_out) {
      const float nanf_ = __int_as_float(0x7fc00000);
      uv_out[i] = (ww != 0.0) ? make_float2((float)(uu / ww), (float)(vv / ww)) : make_float2(nanf_, nanf_);
    }
  }
  __half2* o = out + i * C2;
  if (!ok) {
    const __half2 zero = __floats2half2_rn(0.f, 0.f);
    for (int c = lane; c < C2; c += 32) o[c] = zero;
    return;
  }
  const int i0 = (int)floor(u), j0 = (int)floor(v);
  const int i1 = i0 + 1 < W ? i0 + 1 : W - 1;
  const int j1 = j0 + 1 < H ? j0 + 1 : H - 1;
  const float a = (float)(u - (double)i0), b = (float)(v - (double)j0);
  const float w00 = (1.f - a) * (1.f - b), w01 = a * (1.f - b), w10 = (1.f - a) * b, w11 = a * b;
  const __half2* p00 = img + ((int64_t)j0 * W + i0) * C2;
  const __half2* p01 = img + ((int64_t)j0 * W + i1) * C2;
  const __half2* p10 = img + ((int64_t)j1 * W + i0) * C2;
  const __half2* p11 = img + ((int64_t)j1 * W + i1) * C2;
  for (int c = lane; c < C2; c += 32) {
    const float2 f00 = __half22float2(p00[c]);
    const float2 f01 = __half22float2(p01[c]);
    const float2 f10 = __half22float2(p10[c]);
    const float2 f11 = __half22float2(p11[c]);
    const float gx = w00 * f00.x + w01 * f01.x + w10 * f10.x + w11 * f11.x;
    const float gy = w00 * f00.y + w01 * f01.y + w10 * f10.y + w11 * f11.y;
    o[c] = __floats2half2_rn(gx, gy);
  }
}

}  // namespace

extern "C" emc2_status emc2_project_gather(emc2_ctx* ctx, const float* d_points, int32_t stride_f, int64_t n_points,
                                           const float P[12], const void* d_img, int32_t H, int32_t W, int32_t C,
                                           void* d_out, uint8_t* d_valid, float* d_uv, void* stream) {
  if (!ctx) return EMC2_ERR_INVALID_ARG;
  if (!P || !d_img || (n_points > 0 && (!d_points || !d_out || !d_valid)))
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_project_gather: null argument");
  if (n_points < 0 || stride_f < 3 || H < 1 || W < 1)
    return emc2_fail(ctx, EMC2_ERR_INVALID_ARG, "emc2_project_gather: bad size");
  if (C < 2 || (C & 1) || C > 1024)
    return emc2_fail(ctx, EMC2_ERR_UNSUPPORTED, "emc2_project_gather: C must be even and in [2, 1024]");
  if (n_points == 0) return EMC2_OK;
  ProjMat pm;
  for (int k = 0; k < 12; ++k) pm.m[k] = (double)P[k];
  hipLaunchKernelGGL(k_project_gather, dim3((unsigned)emc2_div_up(n_points, 8)), dim3(256), 0, (hipStream_t)stream, d_points,
                     stride_f, n_points, pm, (const __half2*)d_img, H, W, C / 2, (__half2*)d_out, d_valid, (float2*)d_uv);
  return emc2_check_hip(ctx, hipGetLastError(), "emc2_project_gather launch");
}
