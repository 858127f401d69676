// Quantization groups that run along the TOKEN axis inside one channel ("per-channel" key
// quantization of the KIVI / KVQuant family that the paper's Related work and Limitations name as
// members of a richer compression pool).  The per-element arithmetic is that of the per-token codecs
// in quant_device.h; only the set of elements that share a scale differs: `group` consecutive slots
// of one channel of one head.
//
// Quantize.  A 256-thread block (512 for groups of 128 slots) owns one (token group, 2 heads, layer).  A
// thread owns one (head, 8-channel chunk) column and the token slots  slot, slot + S, ...  of the
// group (S = threads / 32 slots per load step).  All G / S rows of a thread (4 or 8) are loaded up
// front and stay in registers, so the plane is read once.  The per-channel extremes of the S slots
// meet in LDS; one thread per channel then reduces them and builds that channel's quantizer (scale,
// reciprocal, minimum) once, publishes it to LDS and to the scales / mins planes; after the second
// barrier every thread encodes its own rows with the 8 quantizers of its channels.  Blocks are small
// on purpose: several are resident per CU, so one block's load phase overlaps another's encode.
//
// Dequantize.  One 256-thread block per (page, layer) as in the per-token kernel; a page lies inside
// one token group, so a lane keeps the 8 scales (and minima) of its channels in registers.

#include "kvp_common.h"
#include "kvp_internal.h"
#include "quant_device.h"

namespace kvp {
namespace {

// Quantizer of one channel's group, built from the group's extremes (parameter phase) or rebuilt
// from the published (scale, reciprocal, minimum) in the encode phase.
template <int BITS, bool ASYM>
struct ChannelQuantizer;
template <int BITS>
struct ChannelQuantizer<BITS, true> {
  AsymQuantizer<(1 << BITS) - 1> q;
  __device__ __forceinline__ ChannelQuantizer(float lo, float hi) : q(lo, hi) {}
  __device__ __forceinline__ ChannelQuantizer(float scale, float inv, float mn) : q(scale, inv, mn) {}
  __device__ __forceinline__ float scale() const { return q.scale; }
  __device__ __forceinline__ float inv() const { return q.inv; }
  __device__ __forceinline__ float minimum() const { return q.mn; }
  __device__ __forceinline__ bool unsafe() const { return q.unsafe; }
  __device__ __forceinline__ float fast(float x) const { return q.code(x); }
  __device__ __forceinline__ float slow(float x) const {
    return fminf(static_cast<float>((1 << BITS) - 1), fmaxf(0.0f, rintf((x - q.mn) / q.scale)));
  }
};
template <int BITS>
struct ChannelQuantizer<BITS, false> {
  GroupQuantizer<(1 << (BITS - 1)) - 1> q;
  __device__ __forceinline__ ChannelQuantizer(float, float amax) : q(amax) {}
  __device__ __forceinline__ ChannelQuantizer(float scale, float inv, float) : q(scale, inv) {}
  __device__ __forceinline__ float scale() const { return q.scale; }
  __device__ __forceinline__ float inv() const { return q.inv; }
  __device__ __forceinline__ float minimum() const { return 0.0f; }
  __device__ __forceinline__ bool unsafe() const { return q.unsafe; }
  __device__ __forceinline__ float fast(float x) const { return q.code(x); }
  __device__ __forceinline__ float slow(float x) const { return rintf(x / q.scale); }
};
template <>
struct ChannelQuantizer<2, false> {
  TernaryQuantizer q;
  __device__ __forceinline__ ChannelQuantizer(float, float amax) : q(amax) {}
  __device__ __forceinline__ ChannelQuantizer(float scale, float inv, float) : q(scale, inv) {}
  __device__ __forceinline__ float scale() const { return q.amax; }
  __device__ __forceinline__ float inv() const { return q.inv; }
  __device__ __forceinline__ float minimum() const { return 0.0f; }
  __device__ __forceinline__ bool unsafe() const { return q.unsafe; }
  __device__ __forceinline__ float fast(float x) const { return rintf(x * q.inv); }
  __device__ __forceinline__ float slow(float x) const { return (2.0f * fabsf(x) > q.amax) ? copysignf(1.0f, x) : 0.0f; }
};

template <int BITS, bool ASYM>
__device__ __forceinline__ Packed<BITS> pack_codes(const float q[8]) {
  Packed<BITS> p;
  if constexpr (BITS == 8) {
    p.lo = ASYM ? pack_uint8x4(q) : pack_int8x4(q);
    p.hi = ASYM ? pack_uint8x4(q + 4) : pack_int8x4(q + 4);
  } else if constexpr (BITS == 4) {
    p.w = ASYM ? pack_uint4x8(q) : pack_int4x8(q);
  } else {
    p.w = ASYM ? pack_uint2x8(q) : pack_int2x8(q);
  }
  return p;
}
template <int BITS>
__device__ __forceinline__ Packed<BITS> zero_codes() {
  Packed<BITS> p;
  if constexpr (BITS == 8) {
    p.lo = p.hi = 0;
  } else {
    p.w = 0;
  }
  return p;
}

// Block shape for a group of G slots: threads and heads per block; a thread keeps
// G * 16 * HB / threads rows in registers.
#ifndef KVP_QC_SHAPES
#define KVP_QC_SHAPES {256, 2}, {256, 2}, {512, 2}
#endif
struct BlockShape { int threads, heads; };
constexpr BlockShape kShapes[3] = {KVP_QC_SHAPES};   // G = 32, 64, 128
constexpr BlockShape shape_for(int G) { return kShapes[G == 32 ? 0 : (G == 64 ? 1 : 2)]; }

// LDS position of channel `ch` (0 .. 8*COLS-1, ch = col * 8 + c) in an array that the encode phase
// reads back as two float4 per column with consecutive columns adjacent: [half][col][4].
template <int COLS>
__device__ __forceinline__ int param_slot(int ch) {
  const int col = ch >> 3, c = ch & 7;
  return ((c >> 2) * COLS + col) * 4 + (c & 3);
}

template <int BITS, int G, int HB, int kThreadsQ, bool ASYM>
__global__ __launch_bounds__(kThreadsQ) void quantize_channel_kernel(const QuantArgs a, const int mode,
                                                                     const uint32_t n_groups, const uint32_t n_tiles,
                                                                     const FastDiv div_tiles) {
  constexpr int COLS = kLanesPerRow * HB;   // (head, 8-channel chunk) columns of the block
  constexpr int S = kThreadsQ / COLS;       // token slots per load step
  constexpr int NL = G / S;                 // rows per thread
  constexpr int NCH = COLS * 8;             // channels of the block
  static_assert(NL >= 1 && NL * S == G, "group must be a multiple of the slots per step");
  static_assert(NCH <= kThreadsQ, "one thread per channel in the parameter phase");
  constexpr int CB = kHeadDim * BITS / 8;
  __shared__ __align__(16) float part_hi[S][NCH];                        // per slot and channel: max (or abs-max)
  __shared__ __align__(16) float part_lo[ASYM ? S : 1][ASYM ? NCH : 4];  // and min
  __shared__ float4 prm_scale[2 * COLS], prm_inv[2 * COLS], prm_min[ASYM ? 2 * COLS : 1];

  const uint32_t col = threadIdx.x % COLS, slot = threadIdx.x / COLS;
  const uint32_t lane16 = col % kLanesPerRow;
  const uint32_t g = div_tiles.quot(blockIdx.x), tile = blockIdx.x - g * n_tiles;   // head tile fastest
  const uint32_t h0 = tile * HB, h = h0 + col / kLanesPerRow;
  const uint32_t l = blockIdx.y;
  const bool h_ok = h < a.H;
  const uint32_t i0 = g * G;
  const uint32_t Tp = a.rows_per_layer / a.H;

  // ---- all loads first ----
  uint4 raw[NL];
  const uint16_t* base_l = a.src + static_cast<int64_t>(l) * a.stride_l;
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    const uint32_t i = i0 + j * S + slot;
    raw[j] = make_uint4(0, 0, 0, 0);
    if (h_ok && i < a.n_slots) {
      uint32_t t = i;
      if (a.keep_idx) {
        // an out-of-contract index is clamped so that a bad keep list cannot fault the GPU
        t = static_cast<uint32_t>(a.keep_idx[(static_cast<int64_t>(l) * a.H + h) * a.k + i]);
        t = min(t, a.T - 1);
      }
      const uint16_t* row;
      if (mode == kPaged) {
        const uint32_t pg = a.div_bs.quot(t);
        const int64_t blk = min(static_cast<uint32_t>(a.block_table[pg]), a.num_blocks - 1);
        row = base_l + ((blk * a.bs + (t - pg * a.bs)) * a.H + h) * kHeadDim;
      } else {
        row = base_l + static_cast<int64_t>(t) * a.stride_t + static_cast<int64_t>(h) * a.stride_h;
      }
      raw[j] = load_stream16(row + lane16 * 8);
    }
  }

  // ---- extremes of this thread's rows, per channel ----
  {
    float hi[8], lo[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      hi[c] = ASYM ? -INFINITY : 0.0f;
      lo[c] = INFINITY;
    }
#pragma unroll
    for (int j = 0; j < NL; ++j) {
      float x[8];
      unpack_bf16x8(raw[j], x);
      if constexpr (ASYM) {
        if (i0 + j * S + slot < a.n_slots) {   // padding slots never enter a minimum or maximum
#pragma unroll
          for (int c = 0; c < 8; ++c) {
            hi[c] = fmaxf(hi[c], x[c]);
            lo[c] = fminf(lo[c], x[c]);
          }
        }
      } else {
#pragma unroll
        for (int c = 0; c < 8; ++c) hi[c] = fmaxf(hi[c], fabsf(x[c]));
      }
    }
    float4* ph = reinterpret_cast<float4*>(&part_hi[slot][col * 8]);
    ph[0] = make_float4(hi[0], hi[1], hi[2], hi[3]);
    ph[1] = make_float4(hi[4], hi[5], hi[6], hi[7]);
    if constexpr (ASYM) {
      float4* pl = reinterpret_cast<float4*>(&part_lo[slot][col * 8]);
      pl[0] = make_float4(lo[0], lo[1], lo[2], lo[3]);
      pl[1] = make_float4(lo[4], lo[5], lo[6], lo[7]);
    }
  }
  __syncthreads();

  // ---- one thread per channel: group extremes -> quantizer parameters, published to LDS and memory ----
  using CQ = ChannelQuantizer<BITS, ASYM>;
  if (threadIdx.x < NCH) {
    const uint32_t ch = threadIdx.x;
    float hi = part_hi[0][ch], lo = ASYM ? part_lo[0][ch] : 0.0f;
#pragma unroll
    for (int s = 1; s < S; ++s) {
      hi = fmaxf(hi, part_hi[s][ch]);
      if constexpr (ASYM) lo = fminf(lo, part_lo[s][ch]);
    }
    const uint32_t hc = h0 + ch / kHeadDim;   // head of this channel
    if (ASYM && (hc >= a.H || i0 >= a.n_slots)) hi = lo = 0.0f;   // idle column, or a group of padding slots only
    const CQ cq(lo, hi);
    const int ps = param_slot<COLS>(ch);
    reinterpret_cast<float*>(prm_scale)[ps] = cq.scale();
    reinterpret_cast<float*>(prm_inv)[ps] = cq.inv();
    if constexpr (ASYM) reinterpret_cast<float*>(prm_min)[ps] = cq.minimum();
    if (hc < a.H) {
      const int64_t so = ((static_cast<int64_t>(l) * n_groups + g) * a.H + hc) * kHeadDim + ch % kHeadDim;
      a.scales[so] = cq.scale();
      if constexpr (ASYM) a.mins[so] = cq.minimum();
    }
  }
  __syncthreads();

  // ---- encode ----
  float sc[8], iv[8], mn[8];
  {
    const float4 s0 = prm_scale[col], s1 = prm_scale[COLS + col], v0 = prm_inv[col], v1 = prm_inv[COLS + col];
    sc[0] = s0.x; sc[1] = s0.y; sc[2] = s0.z; sc[3] = s0.w; sc[4] = s1.x; sc[5] = s1.y; sc[6] = s1.z; sc[7] = s1.w;
    iv[0] = v0.x; iv[1] = v0.y; iv[2] = v0.z; iv[3] = v0.w; iv[4] = v1.x; iv[5] = v1.y; iv[6] = v1.z; iv[7] = v1.w;
    if constexpr (ASYM) {
      const float4 m0 = prm_min[col], m1 = prm_min[COLS + col];
      mn[0] = m0.x; mn[1] = m0.y; mn[2] = m0.z; mn[3] = m0.w; mn[4] = m1.x; mn[5] = m1.y; mn[6] = m1.z; mn[7] = m1.w;
    } else {
#pragma unroll
      for (int c = 0; c < 8; ++c) mn[c] = 0.0f;
    }
  }
  const CQ cq[8] = {CQ(sc[0], iv[0], mn[0]), CQ(sc[1], iv[1], mn[1]), CQ(sc[2], iv[2], mn[2]), CQ(sc[3], iv[3], mn[3]),
                    CQ(sc[4], iv[4], mn[4]), CQ(sc[5], iv[5], mn[5]), CQ(sc[6], iv[6], mn[6]), CQ(sc[7], iv[7], mn[7])};
  bool any_unsafe = false;
#pragma unroll
  for (int c = 0; c < 8; ++c) any_unsafe = any_unsafe || cq[c].unsafe();

  uint8_t* codes_l = a.codes + static_cast<int64_t>(l) * a.rows_per_layer * CB;
#pragma unroll
  for (int j = 0; j < NL; ++j) {
    const uint32_t i = i0 + j * S + slot;
    if (!h_ok || i >= Tp) continue;
    float x[8], q[8];
    unpack_bf16x8(raw[j], x);
#pragma unroll
    for (int c = 0; c < 8; ++c) q[c] = cq[c].fast(x[c]);
    if (__builtin_amdgcn_ballot_w64(any_unsafe)) {   // extreme magnitudes only
#pragma unroll
      for (int c = 0; c < 8; ++c)
        if (cq[c].unsafe()) q[c] = cq[c].slow(x[c]);
    }
    Packed<BITS> p = pack_codes<BITS, ASYM>(q);
    if (ASYM && i >= a.n_slots) p = zero_codes<BITS>();   // padding slots hold zero codes
    store_codes<BITS>(codes_l + (static_cast<int64_t>(i) * a.H + h) * CB, lane16, p);
  }
}

template <int BITS, int G, bool ASYM>
void launch_q_heads(const QuantArgs& a, int mode, int64_t L, hipStream_t st) {
  constexpr int HB = shape_for(G).heads, kThreadsQ = shape_for(G).threads;
  const uint32_t n_groups = static_cast<uint32_t>(ceil_div(a.rows_per_layer / a.H, G));
  const uint32_t n_tiles = (a.H + HB - 1) / HB;
  quantize_channel_kernel<BITS, G, HB, kThreadsQ, ASYM><<<dim3(n_groups * n_tiles, static_cast<unsigned>(L)), kThreadsQ, 0, st>>>(
      a, mode, n_groups, n_tiles, FastDiv(n_tiles));
}

template <int BITS, bool ASYM>
void launch_q_group(const QuantArgs& a, int group, int mode, int64_t L, hipStream_t st) {
  switch (group) {
    case 32: launch_q_heads<BITS, 32, ASYM>(a, mode, L, st); break;
    case 64: launch_q_heads<BITS, 64, ASYM>(a, mode, L, st); break;
    default: launch_q_heads<BITS, 128, ASYM>(a, mode, L, st); break;
  }
}

template <int BITS>
void launch_q_bits(const QuantArgs& a, int group, int mode, int64_t L, hipStream_t st) {
  if (a.mins)
    launch_q_group<BITS, true>(a, group, mode, L, st);
  else
    launch_q_group<BITS, false>(a, group, mode, L, st);
}

// ------------------------------------------------------------------------------------------------

constexpr int kThreadsD = 256;
constexpr int kRowsPerStepD = kThreadsD / kLanesPerRow;  // 16
constexpr int kUnrollD = 8;

template <int BITS, bool ASYM, bool SCATTER>
__global__ __launch_bounds__(kThreadsD) void dequantize_channel_kernel(const DequantArgs a, const uint32_t group,
                                                                       const uint32_t n_groups, const FastDiv div_h) {
  constexpr int CB = kHeadDim * BITS / 8;
  const int lane16 = threadIdx.x & (kLanesPerRow - 1);
  const uint32_t row_in_step = threadIdx.x / kLanesPerRow;
  const uint32_t page = blockIdx.x, l = blockIdx.y;
  const uint32_t t0 = page * a.bs;
  const uint32_t rows = min(a.bs, a.T - t0) * a.H;
  const int64_t blk = SCATTER ? 0 : min(static_cast<uint32_t>(a.block_table[page]), a.num_blocks - 1);
  const uint8_t* codes = a.codes + (static_cast<int64_t>(l) * a.Tp + t0) * a.H * CB;
  const int64_t group_row0 = (static_cast<int64_t>(l) * n_groups + t0 / group) * a.H;   // the page's group
  uint16_t* dst = a.pool + static_cast<int64_t>(l) * a.pool_stride_l + blk * a.bs * a.H * kHeadDim;
  // with H dividing the rows of a step, a thread meets one head only and loads its scales once
  const bool one_head = (kRowsPerStepD % a.H) == 0;

  float s[8], m[8];
  auto load_group = [&](uint32_t h) {
    const float4* sp = reinterpret_cast<const float4*>(a.scales + (group_row0 + h) * kHeadDim + lane16 * 8);
    const float4 s0 = sp[0], s1 = sp[1];
    s[0] = s0.x; s[1] = s0.y; s[2] = s0.z; s[3] = s0.w; s[4] = s1.x; s[5] = s1.y; s[6] = s1.z; s[7] = s1.w;
    if constexpr (ASYM) {
      const float4* mp = reinterpret_cast<const float4*>(a.mins + (group_row0 + h) * kHeadDim + lane16 * 8);
      const float4 m0 = mp[0], m1 = mp[1];
      m[0] = m0.x; m[1] = m0.y; m[2] = m0.z; m[3] = m0.w; m[4] = m1.x; m[5] = m1.y; m[6] = m1.z; m[7] = m1.w;
    }
  };
  if (one_head) load_group(row_in_step % a.H);

  for (uint32_t r0 = row_in_step; r0 < rows; r0 += kRowsPerStepD * kUnrollD) {
    uint2 c[kUnrollD];
#pragma unroll
    for (int u = 0; u < kUnrollD; ++u) {
      const uint32_t r = r0 + u * kRowsPerStepD;
      c[u] = make_uint2(0, 0);
      if (r < rows) c[u] = load_codes<BITS>(codes + static_cast<int64_t>(r) * CB, lane16);
    }
#pragma unroll
    for (int u = 0; u < kUnrollD; ++u) {
      const uint32_t r = r0 + u * kRowsPerStepD;
      if (r >= rows) continue;
      if (!one_head) load_group(r - div_h.quot(r) * a.H);
      uint32_t w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float y0 = static_cast<float>(field<BITS, ASYM>(c[u], 2 * i)) * s[2 * i];
        float y1 = static_cast<float>(field<BITS, ASYM>(c[u], 2 * i + 1)) * s[2 * i + 1];
        if constexpr (ASYM) {   // a separate binary32 add (contraction is off for this library)
          y0 = y0 + m[2 * i];
          y1 = y1 + m[2 * i + 1];
        }
        w[i] = pack_bf16x2(y0, y1);
      }
      uint16_t* out_row = SCATTER ? scatter_row(a, l, t0, r) : dst + static_cast<int64_t>(r) * kHeadDim;
      store_stream16(out_row + lane16 * 8, make_uint4(w[0], w[1], w[2], w[3]));
    }
  }
}

template <int BITS>
void launch_d_bits(const DequantArgs& a, int group, int64_t L, hipStream_t st) {
  const dim3 grid(static_cast<unsigned>(ceil_div(a.T, a.bs)), static_cast<unsigned>(L));
  const uint32_t n_groups = static_cast<uint32_t>(ceil_div(a.Tp, group));
  const FastDiv dh(a.H);
  if (a.mins) {
    if (a.keep_idx)
      dequantize_channel_kernel<BITS, true, true><<<grid, kThreadsD, 0, st>>>(a, group, n_groups, dh);
    else
      dequantize_channel_kernel<BITS, true, false><<<grid, kThreadsD, 0, st>>>(a, group, n_groups, dh);
  } else {
    if (a.keep_idx)
      dequantize_channel_kernel<BITS, false, true><<<grid, kThreadsD, 0, st>>>(a, group, n_groups, dh);
    else
      dequantize_channel_kernel<BITS, false, false><<<grid, kThreadsD, 0, st>>>(a, group, n_groups, dh);
  }
}

}  // namespace

void quantize_channel_launch(const QuantArgs& a, int bits, int group, int mode, int64_t L, hipStream_t st) {
  switch (bits) {
    case 8: launch_q_bits<8>(a, group, mode, L, st); break;
    case 4: launch_q_bits<4>(a, group, mode, L, st); break;
    default: launch_q_bits<2>(a, group, mode, L, st); break;
  }
}

void dequantize_channel_launch(const DequantArgs& a, int bits, int group, int64_t L, hipStream_t st) {
  switch (bits) {
    case 8: launch_d_bits<8>(a, group, L, st); break;
    case 4: launch_d_bits<4>(a, group, L, st); break;
    default: launch_d_bits<2>(a, group, L, st); break;
  }
}

}  // namespace kvp
