// Per-head q/k preparation of the rope kernel: split-K plane sum, optional per-head RMSNorm (Qwen3 qk-norm),
// rotary embedding in the half-split convention.  One wave per head; lane i < hd/2 owns the pair (i, i + hd/2), other lanes carry zeros.
#pragma once
#include "common.h"

namespace rlx {

// x0, x1 = sum over planes (ascending) of src[p * plane + i], src[p * plane + i + half]; all loads of a batch of
// eight planes are issued before the adds (long calls have one plane: one load per element, same sum)
__device__ __forceinline__ void sum_head_planes(const float* src, size_t plane, int n_planes, bool act, int li,
                                                int half, float& x0, float& x1) {
  x0 = 0.f; x1 = 0.f;
  if (n_planes == 1) {                           // uniform over the grid
    const float u0 = src[li], u1 = src[li + half];
    if (act) { x0 += u0; x1 += u1; }
    return;
  }
  for (int p0 = 0; p0 < n_planes; p0 += 8) {
    float u0[8], u1[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const bool ok = act && p0 + q < n_planes;
      const size_t off = ok ? (size_t)(p0 + q) * plane : 0;
      u0[q] = src[off + li];
      u1[q] = src[off + li + half];
      if (!ok) { u0[q] = 0.f; u1[q] = 0.f; }
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) { x0 += u0[q]; x1 += u1[q]; }
  }
}

// cos / sin of pos * theta^(-2 i / hd); the angle and its reduction are taken in double
__device__ __forceinline__ void rope_cos_sin(int pos, const double* inv_freq, bool act, int li, float& c, float& s) {
  c = 1.f; s = 0.f;
  if (act) {
    double ang = (double)pos * inv_freq[li];
    double sd, cd;
    sincos(ang, &sd, &cd);
    c = (float)cd; s = (float)sd;
  }
}

// optional RMSNorm over the head (gain != null), then the rotation; must be called by the whole wave.  The fused
// multiply-adds are written out so that the rounding does not depend on which product the compiler chooses to fuse.
__device__ __forceinline__ void head_norm_rope(float x0, float x1, const h16_t* gain, int dtype, int hd, float eps,
                                               bool act, int lane, float c, float s, float& y0, float& y1) {
  if (gain) {
    const int li = act ? lane : 0;             // the gains are loaded before the reduction, not after it
    const h16_t g0 = gain[li], g1 = gain[li + (hd >> 1)];
    float ss = wave_sum(__builtin_fmaf(x1, x1, x0 * x0));
    float rstd = 1.0f / sqrtf(ss / (float)hd + eps);
    if (act) {
      x0 = x0 * rstd * h16_to_f32(g0, dtype);
      x1 = x1 * rstd * h16_to_f32(g1, dtype);
    }
  }
  y0 = __builtin_fmaf(x0, c, -(x1 * s));
  y1 = __builtin_fmaf(x1, c, x0 * s);
}

}  // namespace rlx
