// kvp_quantize: group-wise symmetric quantization of bf16 K/V rows to int8/int4/int2 codes with
// one fp32 scale per group (the quantization category of the paper's Background section,
// "KV cache compression"; the formula is this library's stated reading, see include/kvp.h).
//
// Mapping.  A row (one token of one head, 128 bf16 = 256 B) is read by 16 adjacent lanes with one
// 128-bit load each; a lane owns 8 consecutive channels.  A group of 128 / 64 / 32 channels is
// 16 / 8 / 4 adjacent lanes of one DPP row, so the group abs-max is 4 / 3 / 2 cross-lane max steps
// in registers.  A 256-thread block covers kRowsPerBlock consecutive rows of one layer; all loads of
// a thread are issued before any arithmetic so that several KiB per wave are in flight.
//
// The exact-code arithmetic (reciprocal fast path with an exact fallback) lives in quant_device.h.

#include "kvp_common.h"
#include "kvp_internal.h"
#include "quant_device.h"

namespace kvp {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerStep = kThreads / kLanesPerRow;  // 16 rows per load step
// Rows in flight per thread, chosen by measurement on the 8B-shaped plane: the int4 kernel sustains
// 76 % of the HBM peak with 4 (75 % with 2), int8 and int2 80 % and 82 % with 2 (77 % and 79 % with 4).
constexpr int steps_for(int bits) { return bits == 4 ? 4 : 2; }

template <int BITS, int GROUP, bool ASYM>
__device__ __forceinline__ void quantize_lane(const uint4 raw, Packed<BITS>& out, float& scale_out, float& min_out) {
  float x[8], q[8];
  unpack_bf16x8(raw, x);
  if constexpr (ASYM) {
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) {
      lo = fminf(lo, x[i]);
      hi = fmaxf(hi, x[i]);
    }
    group_min_max(lo, hi, GROUP / 8);
    const AsymQuantizer<(1 << BITS) - 1> aq(lo, hi);
    scale_out = aq.scale;
    min_out = aq.mn;
    aq.codes8(x, q);
    if constexpr (BITS == 2) {
      out.w = pack_uint2x8(q);
    } else if constexpr (BITS == 4) {
      out.w = pack_uint4x8(q);
    } else {
      out.lo = pack_uint8x4(q);
      out.hi = pack_uint8x4(q + 4);
    }
  } else {
    min_out = 0.0f;
    const float amax = group_max(abs_max8(x), GROUP / 8);
    if constexpr (BITS == 2) {
      const TernaryQuantizer tq(amax);
      scale_out = amax;  // qmax = 1
      tq.codes8(x, q);
      out.w = pack_int2x8(q);
    } else if constexpr (BITS == 4) {
      const GroupQuantizer<7> gq(amax);
      scale_out = gq.scale;
      gq.codes8(x, q);
      out.w = pack_int4x8(q);
    } else {
      const GroupQuantizer<127> gq(amax);
      scale_out = gq.scale;
      gq.codes8(x, q);
      out.lo = pack_int8x4(q);
      out.hi = pack_int8x4(q + 4);
    }
  }
}

template <int BITS, int GROUP, int MODE, bool ASYM>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const QuantArgs a) {
  constexpr int CB = kHeadDim * BITS / 8;      // code bytes per row
  constexpr int NS = kHeadDim / GROUP;         // scales per row
  constexpr int LANES_PER_GROUP = GROUP / 8;
  constexpr int kSteps = steps_for(BITS);
  constexpr int kRowsPerBlock = kRowsPerStep * kSteps;
  const uint32_t lane_in_row = threadIdx.x & (kLanesPerRow - 1);
  const uint32_t row_in_step = threadIdx.x / kLanesPerRow;
  const uint32_t l = blockIdx.y;
  const uint32_t block_row0 = blockIdx.x * kRowsPerBlock;
  const uint32_t valid_rows = a.n_slots * a.H;
  // block-uniform 64-bit bases, 32-bit per-thread offsets
  const uint16_t* base_l = a.src + static_cast<int64_t>(l) * a.stride_l;
  const uint16_t* base_blk = base_l + static_cast<int64_t>(block_row0) * a.stride_h;  // linear mode only
  const int64_t out_row0 = static_cast<int64_t>(l) * a.rows_per_layer + block_row0;
  uint8_t* codes_blk = a.codes + out_row0 * CB;
  float* scales_blk = a.scales + out_row0 * NS;

  uint4 raw[kSteps];
#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    const uint32_t rloc = row_in_step + s * kRowsPerStep;
    const uint32_t rr = block_row0 + rloc;
    raw[s] = make_uint4(0, 0, 0, 0);
    if (rr < valid_rows) {
      const uint16_t* row;
      if constexpr (MODE == kLinear) {
        row = base_blk + rloc * static_cast<uint32_t>(a.stride_h);
      } else {
        const uint32_t i = a.div_h.quot(rr);
        const uint32_t h = rr - i * a.H;
        uint32_t t = i;
        if (a.keep_idx) {
          // an out-of-contract index is clamped so that a bad keep list cannot fault the GPU
          t = static_cast<uint32_t>(a.keep_idx[(static_cast<int64_t>(l) * a.H + h) * a.k + i]);
          t = min(t, a.T - 1);
        }
        if constexpr (MODE == kStrided) {
          row = base_l + static_cast<int64_t>(t) * a.stride_t + static_cast<int64_t>(h) * a.stride_h;
        } else {
          const uint32_t pg = a.div_bs.quot(t);
          const uint32_t slot = t - pg * a.bs;
          const int64_t blk = min(static_cast<uint32_t>(a.block_table[pg]), a.num_blocks - 1);
          row = base_l + ((blk * a.bs + slot) * a.H + h) * kHeadDim;
        }
      }
      raw[s] = load_stream16(row + lane_in_row * 8);
    }
  }

#pragma unroll
  for (int s = 0; s < kSteps; ++s) {
    const uint32_t rloc = row_in_step + s * kRowsPerStep;
    if (block_row0 + rloc >= a.rows_per_layer) continue;
    Packed<BITS> p;
    float scale, gmin;
    quantize_lane<BITS, GROUP, ASYM>(raw[s], p, scale, gmin);  // zero rows (padding slots) give zero codes and scales
    store_codes<BITS>(codes_blk + rloc * CB, lane_in_row, p);
    if ((lane_in_row % LANES_PER_GROUP) == 0) {
      store_stream_f32(scales_blk + rloc * NS + lane_in_row / LANES_PER_GROUP, scale);
      if constexpr (ASYM) store_stream_f32(a.mins + out_row0 * NS + rloc * NS + lane_in_row / LANES_PER_GROUP, gmin);
    }
  }
}

template <int BITS, int GROUP, bool ASYM>
void launch_mode(int mode, dim3 grid, hipStream_t st, const QuantArgs& a) {
  switch (mode) {
    case kLinear: quantize_kernel<BITS, GROUP, kLinear, ASYM><<<grid, kThreads, 0, st>>>(a); break;
    case kStrided: quantize_kernel<BITS, GROUP, kStrided, ASYM><<<grid, kThreads, 0, st>>>(a); break;
    default: quantize_kernel<BITS, GROUP, kPaged, ASYM><<<grid, kThreads, 0, st>>>(a); break;
  }
}

template <int BITS, bool ASYM>
void launch_group2(int group, int mode, dim3 grid, hipStream_t st, const QuantArgs& a) {
  switch (group) {
    case 32: launch_mode<BITS, 32, ASYM>(mode, grid, st, a); break;
    case 64: launch_mode<BITS, 64, ASYM>(mode, grid, st, a); break;
    default: launch_mode<BITS, 128, ASYM>(mode, grid, st, a); break;
  }
}

template <int BITS>
void launch_group(int group, int mode, dim3 grid, hipStream_t st, const QuantArgs& a) {
  if (a.mins)
    launch_group2<BITS, true>(group, mode, grid, st, a);
  else
    launch_group2<BITS, false>(group, mode, grid, st, a);
}

}  // namespace
}  // namespace kvp

extern "C" int32_t kvp_quantize(const kvp_view* src, const kvp_paged* src_paged, const int32_t* keep_idx, int64_t k,
                                const kvp_qplane* dst, void* stream) {
  using namespace kvp;
  if ((src == nullptr) == (src_paged == nullptr)) return src ? KVP_ERR_SHAPE : KVP_ERR_NULL;
  int32_t rc = check_qplane(dst);
  if (rc != KVP_OK) return rc;
  QuantArgs a{};
  int64_t L, T, H;
  int mode;
  if (src) {
    rc = check_view(src);
    if (rc != KVP_OK) return rc;
    L = src->L; T = src->T; H = src->H;
    a.src = static_cast<const uint16_t*>(src->ptr);
    a.stride_l = src->stride_l; a.stride_t = src->stride_t; a.stride_h = src->stride_h;
    mode = (!keep_idx && src->stride_t == H * src->stride_h && src->stride_h < (1 << 20)) ? kLinear : kStrided;  // 32-bit row offsets inside a block
  } else {
    rc = check_paged(src_paged);
    if (rc != KVP_OK) return rc;
    L = src_paged->L; T = src_paged->T; H = src_paged->H;
    a.src = static_cast<const uint16_t*>(src_paged->pool);
    a.stride_l = src_paged->stride_l;
    a.block_table = src_paged->block_table;
    a.bs = static_cast<uint32_t>(src_paged->bs);
    a.num_blocks = static_cast<uint32_t>(src_paged->num_blocks);
    a.div_bs = FastDiv(a.bs);
    mode = kPaged;
  }
  if (dst->L != L || dst->H != H) return KVP_ERR_SHAPE;
  int64_t n_slots = T;
  if (keep_idx) {
    if (k <= 0 || k > T) return KVP_ERR_SHAPE;
    if (reinterpret_cast<uintptr_t>(keep_idx) & 3u) return KVP_ERR_ALIGN;
    n_slots = k;
  }
  if (dst->T != n_slots) return KVP_ERR_SHAPE;
  if (dst->Tp * H >= (1ll << 31) || T >= (1ll << 31) || L > 65535) return KVP_ERR_SHAPE;
  if (src_paged && src_paged->num_blocks >= (1ll << 31)) return KVP_ERR_SHAPE;
  a.keep_idx = keep_idx;
  a.k = k;
  a.n_slots = static_cast<uint32_t>(n_slots);
  a.T = static_cast<uint32_t>(T);
  a.rows_per_layer = static_cast<uint32_t>(dst->Tp * H);
  a.H = static_cast<uint32_t>(H);
  a.div_h = FastDiv(a.H);
  a.codes = dst->codes;
  a.scales = dst->scales;
  a.mins = dst->mins;
  const hipStream_t st = as_stream(stream);
  if (dst->group_axis == KVP_GROUP_TOKENS) {
    quantize_channel_launch(a, dst->bits, dst->group, mode, L, st);
    return launch_status();
  }
  const int rows_per_block = kRowsPerStep * steps_for(dst->bits);
  const dim3 grid(static_cast<unsigned>(ceil_div(a.rows_per_layer, rows_per_block)), static_cast<unsigned>(L));
  switch (dst->bits) {
    case 8: launch_group<8>(dst->group, mode, grid, st, a); break;
    case 4: launch_group<4>(dst->group, mode, grid, st, a); break;
    default: launch_group<2>(dst->group, mode, grid, st, a); break;
  }
  return launch_status();
}

// ---- self-test of the arithmetic identity the asymmetric quantizer leans on ----
namespace kvp {
namespace {
// one thread per significand; every exponent of the range in turn
__global__ __launch_bounds__(256) void reciprocal_selftest_kernel(unsigned long long* mismatches) {
  const uint32_t sig = blockIdx.x * 256u + threadIdx.x;   // 0 .. 2^23 - 1
  uint32_t bad = 0;
  for (uint32_t e = 127 - 60; e <= 127 + 60; ++e) {
    const float s = __uint_as_float((e << 23) | sig);
    if (__float_as_uint(reciprocal_in_range(s)) != __float_as_uint(1.0f / s)) ++bad;
  }
  if (bad != 0) atomicAdd(mismatches, static_cast<unsigned long long>(bad));
}
}  // namespace
}  // namespace kvp

extern "C" int32_t kvp_selftest_reciprocal(uint64_t* mismatches, void* stream) {
  using namespace kvp;
  if (!mismatches) return KVP_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(mismatches) & 7u) return KVP_ERR_ALIGN;
  reciprocal_selftest_kernel<<<dim3((1u << 23) / 256u), 256, 0, as_stream(stream)>>>(
      reinterpret_cast<unsigned long long*>(mismatches));
  return launch_status();
}

