// Shared host/device helpers of libkvp (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvp.h"

namespace kvp {

constexpr int kWave = 64;
constexpr int kHeadDim = 128;          // the only head_dim the kernels are tiled for
constexpr int kLanesPerRow = 16;       // 128 bf16 = 16 lanes x 16 bytes

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int32_t launch_status() { return hipGetLastError() == hipSuccess ? KVP_OK : KVP_ERR_LAUNCH; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Division of a non-negative n < 2^31 by a divisor fixed at launch: multiply-high and shift.
struct FastDiv {
  uint32_t mul, shift, d;
  FastDiv() : mul(1), shift(0), d(1) {}
  explicit FastDiv(uint32_t div) : d(div) {
    shift = 0;
    while ((1ull << shift) < div) ++shift;
    mul = static_cast<uint32_t>(((1ull << 32) * ((1ull << shift) - div)) / div + 1);
  }
  __device__ __forceinline__ uint32_t quot(uint32_t n) const { return (__umulhi(n, mul) + n) >> shift; }
};

// Validation of a strided bf16 view whose rows the kernels read with 16-byte loads.
inline int32_t check_view(const kvp_view* v) {
  if (!v || !v->ptr) return KVP_ERR_NULL;
  if (v->D != kHeadDim) return KVP_ERR_UNSUPPORTED;
  if (v->L <= 0 || v->T <= 0 || v->H <= 0) return KVP_ERR_SHAPE;
  if (v->stride_l < 0 || v->stride_t < 0 || v->stride_h < 0) return KVP_ERR_SHAPE;
  if (!aligned16(v->ptr) || v->stride_l % 8 || v->stride_t % 8 || v->stride_h % 8) return KVP_ERR_ALIGN;
  return KVP_OK;
}

inline int32_t check_paged(const kvp_paged* p) {
  if (!p || !p->pool || !p->block_table) return KVP_ERR_NULL;
  if (p->D != kHeadDim) return KVP_ERR_UNSUPPORTED;
  if (p->L <= 0 || p->T <= 0 || p->H <= 0 || p->bs <= 0 || p->num_blocks <= 0) return KVP_ERR_SHAPE;
  if (p->num_blocks < ceil_div(p->T, p->bs)) return KVP_ERR_SHAPE;
  if (p->stride_l < p->num_blocks * p->bs * p->H * p->D) return KVP_ERR_SHAPE;
  if (!aligned16(p->pool) || p->stride_l % 8 || (reinterpret_cast<uintptr_t>(p->block_table) & 3u))
    return KVP_ERR_ALIGN;
  return KVP_OK;
}

inline int32_t check_qplane(const kvp_qplane* q) {
  if (!q || !q->codes || !q->scales) return KVP_ERR_NULL;
  if (q->D != kHeadDim) return KVP_ERR_UNSUPPORTED;
  if (q->bits != 8 && q->bits != 4 && q->bits != 2) return KVP_ERR_UNSUPPORTED;
  if (q->group != 32 && q->group != 64 && q->group != 128) return KVP_ERR_UNSUPPORTED;
  if (q->group_axis != KVP_GROUP_CHANNELS && q->group_axis != KVP_GROUP_TOKENS) return KVP_ERR_UNSUPPORTED;
  if (q->L <= 0 || q->T <= 0 || q->H <= 0 || q->Tp < q->T) return KVP_ERR_SHAPE;
  if (!aligned16(q->codes) || !aligned16(q->scales) || !aligned16(q->mins)) return KVP_ERR_ALIGN;
  return KVP_OK;
}

// ---- streaming (non-temporal) global accesses ------------------------------------------------
// K/V planes are read once and written once per call; marking the accesses non-temporal keeps them
// from displacing each other in the caches and measurably raises the sustained HBM rate.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint4 load_stream16(const void* p) {
  const u32x4_t v = __builtin_nontemporal_load(static_cast<const u32x4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ uint2 load_stream8(const void* p) {
  const u32x2_t v = __builtin_nontemporal_load(static_cast<const u32x2_t*>(p));
  return make_uint2(v.x, v.y);
}
__device__ __forceinline__ uint32_t load_stream4(const void* p) {
  return __builtin_nontemporal_load(static_cast<const uint32_t*>(p));
}
__device__ __forceinline__ uint32_t load_stream2(const void* p) {
  return __builtin_nontemporal_load(static_cast<const uint16_t*>(p));
}
__device__ __forceinline__ void store_stream16(void* p, uint4 v) {
  const u32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, static_cast<u32x4_t*>(p));
}
__device__ __forceinline__ void store_stream8(void* p, uint2 v) {
  const u32x2_t w = {v.x, v.y};
  __builtin_nontemporal_store(w, static_cast<u32x2_t*>(p));
}
__device__ __forceinline__ void store_stream4(void* p, uint32_t v) {
  __builtin_nontemporal_store(v, static_cast<uint32_t*>(p));
}
__device__ __forceinline__ void store_stream2(void* p, uint32_t v) {
  __builtin_nontemporal_store(static_cast<uint16_t>(v), static_cast<uint16_t*>(p));
}
__device__ __forceinline__ void store_stream_f32(float* p, float v) { __builtin_nontemporal_store(v, p); }

// ---- device-side bf16 helpers ------------------------------------------------------------

// Two bf16 packed in one 32-bit word -> two floats (exact).
__device__ __forceinline__ float bf16lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// binary32 -> bf16, round to nearest even, done on the integer pattern so that the result does not
// depend on any floating-point mode (subnormal results included).  Finite inputs only.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
// Two floats -> two bf16 in one word with the gfx950 packed convert (v_cvt_pk_bf16_f32; the
// compiler emits it for this vector fptrunc, whose semantics are round-to-nearest-even).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const floatx2_t f = {lo, hi};
  union { bf16x2_t b; uint32_t u; } c;
  c.b = __builtin_convertvector(f, bf16x2_t);
  return c.u;
}

}  // namespace kvp
