// Device-side arithmetic of the group quantizer, shared by kvp_quantize and by the
// configuration-evaluation kernels (which quantize and dequantize on the fly).
//
// Bit-exact codes without one full IEEE division per element.  The defined result is
// q = rint(fl32(x / scale)).  exact_code() forms y0 = x * rcp(scale) (relative error far below
// 2^-21), q0 = rint(y0), and accepts q0 whenever y0 is further than kTieMargin from the nearest
// half-integer: the correctly rounded quotient then lies in the same rounding interval.  Elements
// close to a half-integer are resolved exactly: if fma(-h, scale, x) == 0 the quotient IS the
// half-integer h (common with bf16 inputs) and rounds to the even neighbour; otherwise the element
// takes the full IEEE division.  Both slow steps sit behind wave-uniform branches.
#pragma once

#include "kvp_common.h"

namespace kvp {

template <int CTRL>
__device__ __forceinline__ float dpp_max(float v) {
  const int moved = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true);
  return fmaxf(v, __int_as_float(moved));
}

// max over the `lanes` adjacent lanes (4, 8 or 16, aligned) that share a quantization group;
// `lanes` must be uniform across the wave.
__device__ __forceinline__ float group_max(float v, int lanes) {
  v = dpp_max<0xB1>(v);                      // quad_perm [1,0,3,2]
  v = dpp_max<0x4E>(v);                      // quad_perm [2,3,0,1]
  if (lanes >= 8) v = dpp_max<0x141>(v);     // row_half_mirror: quads 0<->1, 2<->3
  if (lanes >= 16) v = dpp_max<0x140>(v);    // row_mirror: halves of the 16-lane row
  return v;
}

// Code of one element, bit-exact with rint(fl32(x / scale)).
template <int QMAX>
__device__ __forceinline__ int exact_code(float x, float scale, float inv, bool unsafe) {
  // |y0 - fl32(x/scale)| <= |x/scale| * (2^-22 + 2^-24 + 2^-24) < (QMAX + 1) * 2^-21
  constexpr float kTieMargin = static_cast<float>(QMAX + 1) * 0x1p-20f;
  const float y0 = x * inv;
  float q0 = rintf(y0);
  const float d = y0 - q0;  // exact
  const bool risky = unsafe || fabsf(d) > 0.5f - kTieMargin;
  if (__builtin_amdgcn_ballot_w64(risky)) {
    if (risky) {
      const float h = q0 + copysignf(0.5f, d);      // nearest half-integer, exact
      const float e = fmaf(-h, scale, x);           // zero exactly when x / scale == h
      const bool divide = unsafe || e != 0.0f;
      if (!divide) q0 = rintf(h);
      if (__builtin_amdgcn_ballot_w64(divide)) {
        if (divide) q0 = rintf(x / scale);
      }
    }
  }
  return static_cast<int>(q0);
}

// Scale of a group from its abs-max, and the helpers exact_code() needs.
template <int QMAX>
struct GroupScale {
  float scale, inv;
  bool unsafe;
  __device__ __forceinline__ explicit GroupScale(float amax) {
    scale = amax / static_cast<float>(QMAX);  // IEEE division
    // outside this range rcp or the products may leave the normal range: take the division path
    unsafe = !(scale >= 0x1p-100f && scale <= 0x1p100f) && scale != 0.0f;
    inv = (scale == 0.0f) ? 0.0f : __builtin_amdgcn_rcpf(scale);
  }
  __device__ __forceinline__ int code(float x) const {
    const int v = exact_code<QMAX>(x, scale, inv, unsafe);
    return min(QMAX, max(-QMAX, v));
  }
};

// int2: codes are -1, 0, +1 and scale = amax.  x / amax is a ratio of two 8-bit significands and
// cannot round across 1/2, so |code| = 1 exactly when 2|x| > amax (the doubling is exact).
__device__ __forceinline__ int ternary_code(float x, float amax) {
  return (2.0f * fabsf(x) > amax) ? (x < 0.0f ? -1 : 1) : 0;
}

__device__ __forceinline__ void unpack_bf16x8(const uint4 raw, float x[8]) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = bf16lo(w[i]);
    x[2 * i + 1] = bf16hi(w[i]);
  }
}

__device__ __forceinline__ float abs_max8(const float x[8]) {
  float m = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(x[i]));
  return m;
}

}  // namespace kvp
