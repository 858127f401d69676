// kvp_dequantize_paged: packed int8/int4/int2 codes x fp32 group scales -> bf16 rows scattered into
// the serving engine's page pool (the decompression step the paper's Background attributes to
// quantization methods, landing in the paged GPU memory that retrieve() fills).
//
// Mapping.  One 256-thread block restores one page of one layer: bs tokens x H heads = bs*H rows
// that are contiguous both in the compressed plane ([Tp][H][...], tokens t0 .. t0+bs-1) and in the
// destination page, so a block reads one contiguous run of codes and scales and writes one
// contiguous 32 KiB run (H = 8) with 128-bit stores; the block-table entry is read once per block.
// A lane owns 8 consecutive channels of a row: it loads 8 / 4 / 2 bytes of codes and its group's
// scale, and stores 16 bytes.  y = (float)code * scale is one binary32 multiply, rounded to bf16
// (nearest even) on the integer pattern, so the output is bit-identical to the definition.

#include <type_traits>

#include "kvp_common.h"
#include "kvp_internal.h"
#include "quant_device.h"

namespace kvp {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerStep = kThreads / kLanesPerRow;  // 16
constexpr int kUnroll = 8;                             // a 16-token x 8-head page in one sweep

template <int BITS, int GROUP, bool ASYM, bool SCATTER>
__global__ __launch_bounds__(kThreads) void dequantize_paged_kernel(const DequantArgs a) {
  constexpr int CB = kHeadDim * BITS / 8;
  constexpr int NS = kHeadDim / GROUP;
  constexpr int LANES_PER_GROUP = GROUP / 8;
  const int lane_in_row = threadIdx.x & (kLanesPerRow - 1);
  const uint32_t row_in_step = threadIdx.x / kLanesPerRow;
  const uint32_t page = blockIdx.x;
  const uint32_t l = blockIdx.y;
  const uint32_t t0 = page * a.bs;
  const uint32_t tokens = min(a.bs, a.T - t0);
  const uint32_t rows = tokens * a.H;  // rows of this page that hold tokens < T
  // an out-of-contract table entry is clamped so that it cannot fault the GPU
  const int64_t blk = SCATTER ? 0 : min(static_cast<uint32_t>(a.block_table[page]), a.num_blocks - 1);
  const int64_t src_row0 = (static_cast<int64_t>(l) * a.Tp + t0) * a.H;
  const uint8_t* codes = a.codes + src_row0 * CB;
  const float* scales = a.scales + src_row0 * NS;
  const float* mins = ASYM ? a.mins + src_row0 * NS : nullptr;
  uint16_t* dst = a.pool + static_cast<int64_t>(l) * a.pool_stride_l + blk * a.bs * a.H * kHeadDim;

  // One sweep: kUnroll rows per thread, all loads first.  FULL: every row of the sweep exists (the
  // common case: a whole page of 16 tokens x 8 heads is exactly one sweep), so the code carries no
  // per-row guards and no branches.
  auto sweep = [&](auto full_tag, uint32_t r0) {
    constexpr bool FULL = decltype(full_tag)::value;
    uint2 c[kUnroll];
    float s[kUnroll], m[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t r = r0 + u * kRowsPerStep;
      c[u] = make_uint2(0, 0);
      s[u] = 0.0f;
      m[u] = 0.0f;
      if (FULL || r < rows) {
        if constexpr (ASYM) m[u] = __builtin_nontemporal_load(mins + static_cast<int64_t>(r) * NS + lane_in_row / LANES_PER_GROUP);
        c[u] = load_codes<BITS>(codes + static_cast<int64_t>(r) * CB, lane_in_row);
        s[u] = __builtin_nontemporal_load(scales + static_cast<int64_t>(r) * NS + lane_in_row / LANES_PER_GROUP);
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t r = r0 + u * kRowsPerStep;
      if (!FULL && r >= rows) continue;
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float lo = static_cast<float>(field<BITS, ASYM>(c[u], 2 * i)) * s[u];
        float hi = static_cast<float>(field<BITS, ASYM>(c[u], 2 * i + 1)) * s[u];
        if constexpr (ASYM) {   // a separate binary32 add (contraction is off for this library)
          lo = lo + m[u];
          hi = hi + m[u];
        }
        w[i] = pack_bf16x2(lo, hi);
      }
      uint16_t* out_row = SCATTER ? scatter_row(a, l, t0, r) : dst + static_cast<int64_t>(r) * kHeadDim;
      store_stream16(out_row + lane_in_row * 8, make_uint4(w[0], w[1], w[2], w[3]));
    }
  };
  if (rows == kRowsPerStep * kUnroll) {
    sweep(std::true_type{}, row_in_step);
  } else {
    for (uint32_t r0 = row_in_step; r0 < rows; r0 += kRowsPerStep * kUnroll) sweep(std::false_type{}, r0);
  }
}

template <int BITS, bool ASYM, bool SCATTER>
void launch_group3(int group, dim3 grid, hipStream_t st, const DequantArgs& a) {
  switch (group) {
    case 32: dequantize_paged_kernel<BITS, 32, ASYM, SCATTER><<<grid, kThreads, 0, st>>>(a); break;
    case 64: dequantize_paged_kernel<BITS, 64, ASYM, SCATTER><<<grid, kThreads, 0, st>>>(a); break;
    default: dequantize_paged_kernel<BITS, 128, ASYM, SCATTER><<<grid, kThreads, 0, st>>>(a); break;
  }
}

template <int BITS, bool ASYM>
void launch_group2(int group, dim3 grid, hipStream_t st, const DequantArgs& a) {
  if (a.keep_idx)
    launch_group3<BITS, ASYM, true>(group, grid, st, a);
  else
    launch_group3<BITS, ASYM, false>(group, grid, st, a);
}

template <int BITS>
void launch_group(int group, dim3 grid, hipStream_t st, const DequantArgs& a) {
  if (a.mins)
    launch_group2<BITS, true>(group, grid, st, a);
  else
    launch_group2<BITS, false>(group, grid, st, a);
}

__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  // one 16-byte streaming load and store per thread: the shape that sustained the highest rate on this part
  const size_t idx = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  if (idx < n16) store_stream16(dst + idx, load_stream16(src + idx));
}

}  // namespace
}  // namespace kvp

namespace kvp {
namespace {

// Common body of kvp_dequantize_paged (keep_idx == nullptr) and kvp_dequantize_paged_scatter.
int32_t dequantize_impl(const kvp_qplane* src, const int32_t* keep_idx, const kvp_paged* dst, void* stream) {
  int32_t rc = check_qplane(src);
  if (rc != KVP_OK) return rc;
  rc = check_paged(dst);
  if (rc != KVP_OK) return rc;
  if (src->L != dst->L || src->H != dst->H) return KVP_ERR_SHAPE;
  if (keep_idx ? src->T > dst->T : src->T != dst->T) return KVP_ERR_SHAPE;
  if (keep_idx && (reinterpret_cast<uintptr_t>(keep_idx) & 3u)) return KVP_ERR_ALIGN;
  if (dst->T >= (1ll << 31) || dst->bs * dst->H >= (1ll << 31) || dst->num_blocks >= (1ll << 31) || dst->L > 65535)
    return KVP_ERR_SHAPE;
  DequantArgs a{};
  a.codes = src->codes;
  a.scales = src->scales;
  a.mins = src->mins;
  a.pool = static_cast<uint16_t*>(dst->pool);
  a.block_table = dst->block_table;
  a.pool_stride_l = dst->stride_l;
  a.Tp = src->Tp;
  a.T = static_cast<uint32_t>(src->T);
  a.H = static_cast<uint32_t>(dst->H);
  a.bs = static_cast<uint32_t>(dst->bs);
  a.num_blocks = static_cast<uint32_t>(dst->num_blocks);
  a.keep_idx = keep_idx;
  a.k = src->T;
  a.T_full = static_cast<uint32_t>(dst->T);
  a.div_h = FastDiv(a.H);
  a.div_bs = FastDiv(a.bs);
  const dim3 grid(static_cast<unsigned>(ceil_div(src->T, dst->bs)), static_cast<unsigned>(dst->L));
  const hipStream_t st = as_stream(stream);
  if (src->group_axis == KVP_GROUP_TOKENS) {
    if (src->group % dst->bs != 0) return KVP_ERR_UNSUPPORTED;
    dequantize_channel_launch(a, src->bits, src->group, dst->L, st);
    return launch_status();
  }
  switch (src->bits) {
    case 8: launch_group<8>(src->group, grid, st, a); break;
    case 4: launch_group<4>(src->group, grid, st, a); break;
    default: launch_group<2>(src->group, grid, st, a); break;
  }
  return launch_status();
}

}  // namespace
}  // namespace kvp

extern "C" int32_t kvp_dequantize_paged(const kvp_qplane* src, const kvp_paged* dst, void* stream) {
  return kvp::dequantize_impl(src, nullptr, dst, stream);
}

extern "C" int32_t kvp_dequantize_paged_scatter(const kvp_qplane* src, const int32_t* keep_idx, const kvp_paged* dst,
                                                void* stream) {
  if (!keep_idx) return KVP_ERR_NULL;
  return kvp::dequantize_impl(src, keep_idx, dst, stream);
}

extern "C" int32_t kvp_copy_bytes(void* dst, const void* src, size_t nbytes, void* stream) {
  using namespace kvp;
  if (!dst || !src) return KVP_ERR_NULL;
  if (!aligned16(dst) || !aligned16(src) || nbytes % 16) return KVP_ERR_ALIGN;
  if (nbytes == 0) return KVP_OK;
  const size_t n16 = nbytes / 16;
  const size_t blocks = (n16 + 255) / 256;
  if (blocks >= (1ull << 31)) return KVP_ERR_SHAPE;
  copy_kernel<<<dim3(static_cast<unsigned>(blocks)), 256, 0, as_stream(stream)>>>(static_cast<uint4*>(dst),
                                                                                   static_cast<const uint4*>(src), n16);
  return launch_status();
}

extern "C" int64_t kvp_keep_count(double ratio, int64_t T) {
  // ceil(ratio * T) evaluated in double, clamped to [1, T]
  const double x = ratio * static_cast<double>(T);
  int64_t k = static_cast<int64_t>(x);
  if (static_cast<double>(k) < x) ++k;
  if (k < 1) k = 1;
  if (k > T) k = T;
  return k;
}

extern "C" const char* kvp_strerror(int32_t code) {
  switch (code) {
    case KVP_OK: return "ok";
    case KVP_ERR_NULL: return "a required pointer is NULL";
    case KVP_ERR_ALIGN: return "pointer or stride breaks the 16-byte row alignment";
    case KVP_ERR_SHAPE: return "inconsistent sizes";
    case KVP_ERR_UNSUPPORTED: return "unsupported bits / group / head_dim";
    case KVP_ERR_WORKSPACE: return "workspace missing or too small";
    case KVP_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown kvp error code";
  }
}

// major.minor.patch as 0x00MMmmpp; the minor number moves whenever the ABI gains a field or an entry point
extern "C" uint32_t kvp_version(void) { return 0x00010500u; }

extern "C" size_t kvp_workspace_bytes(int32_t op, const kvp_dims* d) {
  if (!d) return 0;
  switch (op) {
    case KVP_WS_SCORE_TOKENS: return kvp_score_workspace_bytes(d->L, d->Hkv, d->Hq, d->W, d->T);
    case KVP_WS_SCORE_KEYS: return kvp_score_keys_workspace_bytes(d->L, d->Hkv, d->T, d->method);
    case KVP_WS_SELECT_TOPK: return kvp_select_workspace_bytes(d->n_rows, d->T, d->k);
    case KVP_WS_EVAL_CONFIGS: return kvp_eval_workspace_bytes(d->L, d->Hkv, d->Hq, d->W, d->T, d->n_cfgs);
    default: return 0;
  }
}
