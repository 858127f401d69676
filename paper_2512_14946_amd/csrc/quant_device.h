// Device-side arithmetic of the group quantizer, shared by kvp_quantize and by the
// configuration-evaluation kernels (which quantize and dequantize on the fly).
//
// Bit-exact codes without one full IEEE division per element: see GroupQuantizer below.
#pragma once

#include "kvp_common.h"

namespace kvp {

// Cross-lane max of non-negative floats, taken on their bit patterns as unsigned integers (the IEEE
// order of non-negative floats is the order of their patterns), so that no NaN canonicalization is
// emitted and the DPP operand folds into the max instruction.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_umax(uint32_t v) {
  const uint32_t moved = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, 0xf, 0xf, true));
  return max(v, moved);
}

// max over the `lanes` adjacent lanes (4, 8 or 16, aligned) that share a quantization group;
// `lanes` must be uniform across the wave and v must be non-negative.
__device__ __forceinline__ float group_max(float v, int lanes) {
  uint32_t u = __float_as_uint(v);
  u = dpp_umax<0xB1>(u);                     // quad_perm [1,0,3,2]
  u = dpp_umax<0x4E>(u);                     // quad_perm [2,3,0,1]
  if (lanes >= 8) u = dpp_umax<0x141>(u);    // row_half_mirror: quads 0<->1, 2<->3
  if (lanes >= 16) u = dpp_umax<0x140>(u);   // row_mirror: halves of the 16-lane row
  return __uint_as_float(u);
}

// scale = fl32(amax / QMAX) for QMAX in {7, 127} without the full division sequence:
// q0 = amax * c, r = fma(-QMAX, q0, amax), scale = fma(r, c, q0) with c = fl32(1 / QMAX).
// amax is always a bf16 value (the abs-max of bf16 inputs); the identity with IEEE division was
// checked exhaustively over all 32640 finite non-negative bf16 values, subnormals included.
template <int QMAX>
__device__ __forceinline__ float scale_of_bf16_amax(float amax) {
  constexpr float kQ = static_cast<float>(QMAX);
  constexpr float kC = 1.0f / kQ;
  const float q0 = amax * kC;
  const float r = fmaf(-kQ, q0, amax);
  return fmaf(r, kC, q0);
}

// fl32(1 / s) for 2^-60 <= s <= 2^60 without the division sequence: v_rcp_f32 (1 ulp) and one fma correction
// step.  On gfx950 the result equals the IEEE quotient 1.0f / s for EVERY binary32 s in that range:
// kvp_selftest_reciprocal runs the comparison over all 2^23 significands x 121 exponents on the device (0.3 s)
// and a GPU test asserts that it finds no mismatch.
__device__ __forceinline__ float reciprocal_in_range(float s) {
  const float y0 = __builtin_amdgcn_rcpf(s);
  return fmaf(fmaf(-s, y0, 1.0f), y0, y0);
}

// Group quantizer for QMAX in {7, 127}: scale and the codes (as integral floats) of one lane's
// 8 elements, bit-exact with rint(fl32(x / scale)), without a division per element and without a
// branch:
//   inv = fl32(1 / scale)   from v_rcp_f32 (1 ulp) and one correction step fma(fma(-scale, y0, 1), y0, y0),
//                           which lands on the correctly rounded reciprocal for every one of the
//                           2 x 32640 scales that exist (scale = fl32(bf16 / QMAX)), whatever the
//                           sign of the reciprocal estimate's last-place error;
//   q0 = x * inv,  r = fma(-scale, q0, x) (the exact remainder),  y = fma(r, inv, q0),  code = rint(y).
// y is the correctly rounded quotient (the classical remainder-correction division step), so exact
// ties k + 1/2 come out exactly and round to even.  The identity rint(y) == rint(fl32(x / scale)) was
// checked on the CPU for every bf16 amax in the exponent range below and every bf16 |x| <= amax
// (1.7e9 pairs, both QMAX).  Outside that range the quantizer divides.
template <int QMAX>
struct GroupQuantizer {
  float scale, inv;
  bool unsafe;
  __device__ __forceinline__ explicit GroupQuantizer(float amax) {
    scale = scale_of_bf16_amax<QMAX>(amax);
    // outside this range an intermediate may leave the normal range: take the division path
    unsafe = !(scale >= 0x1p-60f && scale <= 0x1p60f) && scale != 0.0f;
    const float y0 = __builtin_amdgcn_rcpf(scale);
    inv = (scale == 0.0f) ? 0.0f : fmaf(fmaf(-scale, y0, 1.0f), y0, y0);
  }
  // from parameters computed elsewhere (the same scale and reciprocal)
  __device__ __forceinline__ GroupQuantizer(float s, float i) : scale(s), inv(i) {
    unsafe = !(s >= 0x1p-60f && s <= 0x1p60f) && s != 0.0f;
  }

  __device__ __forceinline__ float code(float x) const {
    const float q0 = x * inv;
    const float r = fmaf(-scale, q0, x);
    return rintf(fmaf(r, inv, q0));
  }

  __device__ __forceinline__ void codes8(const float x[8], float q[8]) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = code(x[i]);
    if (__builtin_amdgcn_ballot_w64(unsafe)) {         // extreme magnitudes only
      if (unsafe) {
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = rintf(x[i] / scale);
      }
    }
  }
};

// Asymmetric codec: codes 0 .. LEVELS of d = fl32(x - mn) on the scale fl32(fl32(mx - mn) / LEVELS).
// The same remainder-correction step as GroupQuantizer, applied to d; the scale is an arbitrary
// binary32 value here, so the step needs the correctly rounded reciprocal fl32(1 / scale): that is what
// reciprocal_in_range returns for every operand of its range on this hardware (checked exhaustively on the device).
template <int LEVELS>
struct AsymQuantizer {
  float scale, inv, mn;
  bool unsafe;
  __device__ __forceinline__ AsymQuantizer(float gmin, float gmax) {
    mn = gmin + 0.0f;                                   // -0 -> +0, everything else unchanged
    const float range = (gmax + 0.0f) - mn;             // a zero maximum counts as +0 too
    // range / LEVELS, correctly rounded without a division: product with the rounded reciprocal,
    // exact remainder, one correction (checked against IEEE division for all 2^23 significands and
    // LEVELS = 3, 15, 255).  Outside the exponent range where no step under- or overflows: divide.
    constexpr float kLevels = static_cast<float>(LEVELS);
    constexpr float kInvLevels = 1.0f / kLevels;
    const float q0 = range * kInvLevels;
    scale = fmaf(fmaf(-kLevels, q0, range), kInvLevels, q0);
    unsafe = !(q0 >= 0x1p-60f && q0 <= 0x1p60f) && range != 0.0f;
    if (__builtin_amdgcn_ballot_w64(unsafe)) {
      if (unsafe) scale = range / kLevels;
    }
    unsafe = unsafe && scale != 0.0f;
    // inside the exponent range the corrected hardware reciprocal is the IEEE one (see reciprocal_in_range);
    // outside it codes8 divides and inv is not used
    inv = (scale == 0.0f) ? 0.0f : reciprocal_in_range(scale);
  }
  // from parameters computed elsewhere (the same scale, reciprocal and minimum)
  __device__ __forceinline__ AsymQuantizer(float s, float i, float m) : scale(s), inv(i), mn(m) {
    unsafe = !(s >= 0x1p-60f && s <= 0x1p60f) && s != 0.0f;
  }

  __device__ __forceinline__ float code(float x) const {
    const float d0 = x - mn;
    const float q0 = d0 * inv;
    const float r = fmaf(-scale, q0, d0);
    return rintf(fmaf(r, inv, q0));
  }
  __device__ __forceinline__ void codes8(const float x[8], float q[8]) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = code(x[i]);
    if (__builtin_amdgcn_ballot_w64(unsafe)) {
      if (unsafe) {
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = fminf(static_cast<float>(LEVELS), fmaxf(0.0f, rintf((x[i] - mn) / scale)));
      }
    }
  }
};

template <int CTRL>
__device__ __forceinline__ float dpp_peer(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xf, 0xf, false));
}
// min and max over the `lanes` adjacent lanes (4, 8 or 16, aligned) of a quantization group
__device__ __forceinline__ void group_min_max(float& lo, float& hi, int lanes) {
  lo = fminf(lo, dpp_peer<0xB1>(lo)); hi = fmaxf(hi, dpp_peer<0xB1>(hi));
  lo = fminf(lo, dpp_peer<0x4E>(lo)); hi = fmaxf(hi, dpp_peer<0x4E>(hi));
  if (lanes >= 8) { lo = fminf(lo, dpp_peer<0x141>(lo)); hi = fmaxf(hi, dpp_peer<0x141>(hi)); }
  if (lanes >= 16) { lo = fminf(lo, dpp_peer<0x140>(lo)); hi = fmaxf(hi, dpp_peer<0x140>(hi)); }
}

// int2: codes are -1, 0, +1 and scale = amax.  x / amax is a ratio of two 8-bit significands, so it
// is either exactly 1/2 (code 0: ties go to even) or at least 1/510 away from it.  Multiplying by a
// reciprocal shrunk by 2^-20 keeps exact ties below 1/2 and cannot move any other quotient across
// it, so rint(x * inv) is the exact code.  Extreme magnitudes compare 2|x| > amax instead.
struct TernaryQuantizer {
  float amax, inv;
  bool unsafe;
  __device__ __forceinline__ explicit TernaryQuantizer(float a) : amax(a) {
    unsafe = !(a >= 0x1p-60f && a <= 0x1p60f) && a != 0.0f;
    inv = (a == 0.0f) ? 0.0f : __builtin_amdgcn_rcpf(a) * (1.0f - 0x1p-20f);
  }
  __device__ __forceinline__ TernaryQuantizer(float a, float i) : amax(a), inv(i) {
    unsafe = !(a >= 0x1p-60f && a <= 0x1p60f) && a != 0.0f;
  }
  __device__ __forceinline__ void codes8(const float x[8], float q[8]) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) q[i] = rintf(x[i] * inv);
    if (__builtin_amdgcn_ballot_w64(unsafe)) {
      if (unsafe) {
#pragma unroll
        for (int i = 0; i < 8; ++i) q[i] = (2.0f * fabsf(x[i]) > amax) ? copysignf(1.0f, x[i]) : 0.0f;
      }
    }
  }
};

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

// Packing of integral-float codes, done in the float domain: with an offset of 2^(bits-1) every
// field is non-negative, the weighted sum of up to 16 bits is exact in binary32, and one XOR turns
// the offset fields into two's complement fields.
__device__ __forceinline__ uint32_t pack_int4x8(const float q[8]) {
  const float lo = fmaf(q[3], 4096.0f, fmaf(q[2], 256.0f, fmaf(q[1], 16.0f, q[0]))) + 34952.0f;  // 0x8888
  const float hi = fmaf(q[7], 4096.0f, fmaf(q[6], 256.0f, fmaf(q[5], 16.0f, q[4]))) + 34952.0f;
  return (static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16)) ^ 0x88888888u;
}
__device__ __forceinline__ uint32_t pack_int8x4(const float q[4]) {
  const float lo = fmaf(q[1], 256.0f, q[0]) + 32896.0f;  // 0x8080
  const float hi = fmaf(q[3], 256.0f, q[2]) + 32896.0f;
  return (static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16)) ^ 0x80808080u;
}
__device__ __forceinline__ uint32_t pack_int2x8(const float q[8]) {
  float s = q[7];
#pragma unroll
  for (int i = 6; i >= 0; --i) s = fmaf(s, 4.0f, q[i]);
  return static_cast<uint32_t>(s + 43690.0f) ^ 0xAAAAu;  // 0xAAAA
}

// Unsigned fields (asymmetric codec): plain exact weighted sums.
__device__ __forceinline__ uint32_t pack_uint4x8(const float q[8]) {
  const float lo = fmaf(q[3], 4096.0f, fmaf(q[2], 256.0f, fmaf(q[1], 16.0f, q[0])));
  const float hi = fmaf(q[7], 4096.0f, fmaf(q[6], 256.0f, fmaf(q[5], 16.0f, q[4])));
  return static_cast<uint32_t>(lo) | (static_cast<uint32_t>(hi) << 16);
}
__device__ __forceinline__ uint32_t pack_uint8x4(const float q[4]) {
  return static_cast<uint32_t>(fmaf(q[1], 256.0f, q[0])) | (static_cast<uint32_t>(fmaf(q[3], 256.0f, q[2])) << 16);
}
__device__ __forceinline__ uint32_t pack_uint2x8(const float q[8]) {
  float s = q[7];
#pragma unroll
  for (int i = 6; i >= 0; --i) s = fmaf(s, 4.0f, q[i]);
  return static_cast<uint32_t>(s);
}

// ---- packed codes of one lane (8 consecutive channels of a row) ----------------------------------
template <int BITS>
struct Packed;  // the 8 codes of one lane
template <> struct Packed<8> { uint32_t lo, hi; };
template <> struct Packed<4> { uint32_t w; };
template <> struct Packed<2> { uint32_t w; };

template <int BITS>
__device__ __forceinline__ void store_codes(uint8_t* row_codes, int lane_in_row, const Packed<BITS>& p);
template <>
__device__ __forceinline__ void store_codes<8>(uint8_t* row_codes, int lane_in_row, const Packed<8>& p) {
  store_stream8(row_codes + lane_in_row * 8, make_uint2(p.lo, p.hi));
}
template <>
__device__ __forceinline__ void store_codes<4>(uint8_t* row_codes, int lane_in_row, const Packed<4>& p) {
  store_stream4(row_codes + lane_in_row * 4, p.w);
}
template <>
__device__ __forceinline__ void store_codes<2>(uint8_t* row_codes, int lane_in_row, const Packed<2>& p) {
  store_stream2(row_codes + lane_in_row * 2, p.w);
}

template <int BITS>
__device__ __forceinline__ uint2 load_codes(const uint8_t* row_codes, int lane_in_row);
template <>
__device__ __forceinline__ uint2 load_codes<8>(const uint8_t* row_codes, int lane_in_row) {
  return load_stream8(row_codes + lane_in_row * 8);
}
template <>
__device__ __forceinline__ uint2 load_codes<4>(const uint8_t* row_codes, int lane_in_row) {
  return make_uint2(load_stream4(row_codes + lane_in_row * 4), 0);
}
template <>
__device__ __forceinline__ uint2 load_codes<2>(const uint8_t* row_codes, int lane_in_row) {
  return make_uint2(load_stream2(row_codes + lane_in_row * 2), 0);
}

// field i (of 8) of a lane's packed codes: signed (symmetric codec) or unsigned (asymmetric codec)
template <int BITS, bool ASYM>
__device__ __forceinline__ int field(const uint2 c, int i) {
  const uint32_t w = (BITS == 8 && i >= 4) ? c.y : c.x;
  const int off = BITS == 8 ? 8 * (i & 3) : BITS * i;
  if constexpr (ASYM)
    return static_cast<int>(__builtin_amdgcn_ubfe(w, off, BITS));
  else
    return __builtin_amdgcn_sbfe(static_cast<int>(w), off, BITS);
}

}  // namespace kvp
