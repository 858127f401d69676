// Quantization groups that run along the TOKEN axis inside one channel ("per-channel" key
// quantization of the KIVI / KVQuant family that the paper's Related work and Limitations name as
// members of a richer compression pool).  The per-element arithmetic is that of the per-token codecs
// in quant_device.h; only the set of elements that share a scale differs: `group` consecutive slots
// of one channel of one head.
//
// Quantize.  A 1024-thread block owns one (token group, tile of HB heads, layer).  A thread owns one
// (head, 8-channel chunk) column and the token slots  slot, slot + S, ... of the group
// (S = 1024 / (16 HB) slots are loaded per step, so one step of the block reads S tokens x HB heads:
// one contiguous run of a flat plane).  All G / S rows of a thread are loaded up front and stay in
// registers; the per-channel extremes of the S slots meet in LDS (one barrier), every thread then
// builds the 8 quantizers of its channels and encodes its own rows.  The plane is read once.
//
// Dequantize.  One 256-thread block per (page, layer) as in the per-token kernel; a page lies inside
// one token group, so a lane keeps the 8 scales (and minima) of its channels in registers.

#include "kvp_common.h"
#include "kvp_internal.h"
#include "quant_device.h"

namespace kvp {
namespace {

constexpr int kThreadsQ = 1024;

template <int BITS, bool ASYM>
struct ChannelQuantizer;   // quantizer of one channel's group
template <int BITS>
struct ChannelQuantizer<BITS, true> {
  AsymQuantizer<(1 << BITS) - 1> q;
  __device__ __forceinline__ ChannelQuantizer(float lo, float hi) : q(lo, hi) {}
  __device__ __forceinline__ float scale() const { return q.scale; }
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
  __device__ __forceinline__ float scale() const { return q.scale; }
  __device__ __forceinline__ float minimum() const { return 0.0f; }
  __device__ __forceinline__ bool unsafe() const { return q.unsafe; }
  __device__ __forceinline__ float fast(float x) const { return q.code(x); }
  __device__ __forceinline__ float slow(float x) const { return rintf(x / q.scale); }
};
template <>
struct ChannelQuantizer<2, false> {
  TernaryQuantizer q;
  __device__ __forceinline__ ChannelQuantizer(float, float amax) : q(amax) {}
  __device__ __forceinline__ float scale() const { return q.amax; }
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

template <int BITS, int G, int HB, bool ASYM>
__global__ __launch_bounds__(kThreadsQ) void quantize_channel_kernel(const QuantArgs a, const int mode) {
  constexpr int COLS = kLanesPerRow * HB;   // (head, 8-channel chunk) columns of the block
  constexpr int S = kThreadsQ / COLS;       // token slots per load step
  constexpr int NL = G / S;                 // rows per thread
  static_assert(NL >= 1 && NL * S == G, "group must be a multiple of the slots per step");
  constexpr int CB = kHeadDim * BITS / 8;
  __shared__ float4 red_hi[S][2][COLS];
  __shared__ float4 red_lo[ASYM ? S : 1][2][ASYM ? COLS : 1];

  const uint32_t col = threadIdx.x % COLS, slot = threadIdx.x / COLS;
  const uint32_t lane16 = col % kLanesPerRow;
  const uint32_t h = blockIdx.y * HB + col / kLanesPerRow;
  const uint32_t g = blockIdx.x, l = blockIdx.z;
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
  red_hi[slot][0][col] = make_float4(hi[0], hi[1], hi[2], hi[3]);
  red_hi[slot][1][col] = make_float4(hi[4], hi[5], hi[6], hi[7]);
  if constexpr (ASYM) {
    red_lo[slot][0][col] = make_float4(lo[0], lo[1], lo[2], lo[3]);
    red_lo[slot][1][col] = make_float4(lo[4], lo[5], lo[6], lo[7]);
  }
  __syncthreads();
#pragma unroll 4
  for (int s = 0; s < S; ++s) {
    const float4 u0 = red_hi[s][0][col], u1 = red_hi[s][1][col];
    hi[0] = fmaxf(hi[0], u0.x); hi[1] = fmaxf(hi[1], u0.y); hi[2] = fmaxf(hi[2], u0.z); hi[3] = fmaxf(hi[3], u0.w);
    hi[4] = fmaxf(hi[4], u1.x); hi[5] = fmaxf(hi[5], u1.y); hi[6] = fmaxf(hi[6], u1.z); hi[7] = fmaxf(hi[7], u1.w);
    if constexpr (ASYM) {
      const float4 v0 = red_lo[s][0][col], v1 = red_lo[s][1][col];
      lo[0] = fminf(lo[0], v0.x); lo[1] = fminf(lo[1], v0.y); lo[2] = fminf(lo[2], v0.z); lo[3] = fminf(lo[3], v0.w);
      lo[4] = fminf(lo[4], v1.x); lo[5] = fminf(lo[5], v1.y); lo[6] = fminf(lo[6], v1.z); lo[7] = fminf(lo[7], v1.w);
    }
  }
  if (ASYM && (!h_ok || i0 >= a.n_slots)) {   // a group of padding slots only (or an idle column): scale 0, minimum 0
#pragma unroll
    for (int c = 0; c < 8; ++c) hi[c] = lo[c] = 0.0f;
  }

  // ---- the 8 quantizers of this thread's channels; slot 0 publishes scales and minima ----
  using CQ = ChannelQuantizer<BITS, ASYM>;
  const CQ cq[8] = {CQ(lo[0], hi[0]), CQ(lo[1], hi[1]), CQ(lo[2], hi[2]), CQ(lo[3], hi[3]),
                    CQ(lo[4], hi[4]), CQ(lo[5], hi[5]), CQ(lo[6], hi[6]), CQ(lo[7], hi[7])};
  bool any_unsafe = false;
#pragma unroll
  for (int c = 0; c < 8; ++c) any_unsafe = any_unsafe || cq[c].unsafe();
  if (slot == 0 && h_ok) {
    const int64_t so = ((static_cast<int64_t>(l) * gridDim.x + g) * a.H + h) * kHeadDim + lane16 * 8;
    float4* sp = reinterpret_cast<float4*>(a.scales + so);
    sp[0] = make_float4(cq[0].scale(), cq[1].scale(), cq[2].scale(), cq[3].scale());
    sp[1] = make_float4(cq[4].scale(), cq[5].scale(), cq[6].scale(), cq[7].scale());
    if constexpr (ASYM) {
      float4* mp = reinterpret_cast<float4*>(a.mins + so);
      mp[0] = make_float4(cq[0].minimum(), cq[1].minimum(), cq[2].minimum(), cq[3].minimum());
      mp[1] = make_float4(cq[4].minimum(), cq[5].minimum(), cq[6].minimum(), cq[7].minimum());
    }
  }

  // ---- encode ----
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
  const unsigned n_groups = static_cast<unsigned>(ceil_div(a.rows_per_layer / a.H, G));
  // heads per block: 8 when the plane has that many, so that a load step is one contiguous run;
  // 4 for groups of 128 slots, which keeps a thread at 8 rows (16 would spill registers)
  if (a.H >= 8 && G <= 64) {
    quantize_channel_kernel<BITS, G, 8, ASYM><<<dim3(n_groups, (a.H + 7) / 8, L), kThreadsQ, 0, st>>>(a, mode);
  } else if (a.H >= 4) {
    quantize_channel_kernel<BITS, G, 4, ASYM><<<dim3(n_groups, (a.H + 3) / 4, L), kThreadsQ, 0, st>>>(a, mode);
  } else {
    quantize_channel_kernel<BITS, G, 2, ASYM><<<dim3(n_groups, (a.H + 1) / 2, L), kThreadsQ, 0, st>>>(a, mode);
  }
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

template <int BITS, bool ASYM>
__global__ __launch_bounds__(kThreadsD) void dequantize_channel_kernel(const DequantArgs a, const uint32_t group,
                                                                       const uint32_t n_groups, const FastDiv div_h) {
  constexpr int CB = kHeadDim * BITS / 8;
  const int lane16 = threadIdx.x & (kLanesPerRow - 1);
  const uint32_t row_in_step = threadIdx.x / kLanesPerRow;
  const uint32_t page = blockIdx.x, l = blockIdx.y;
  const uint32_t t0 = page * a.bs;
  const uint32_t rows = min(a.bs, a.T - t0) * a.H;
  const int64_t blk = min(static_cast<uint32_t>(a.block_table[page]), a.num_blocks - 1);
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
      store_stream16(dst + static_cast<int64_t>(r) * kHeadDim + lane16 * 8, make_uint4(w[0], w[1], w[2], w[3]));
    }
  }
}

template <int BITS>
void launch_d_bits(const DequantArgs& a, int group, int64_t L, hipStream_t st) {
  const dim3 grid(static_cast<unsigned>(ceil_div(a.T, a.bs)), static_cast<unsigned>(L));
  const uint32_t n_groups = static_cast<uint32_t>(ceil_div(a.Tp, group));
  if (a.mins)
    dequantize_channel_kernel<BITS, true><<<grid, kThreadsD, 0, st>>>(a, group, n_groups, FastDiv(a.H));
  else
    dequantize_channel_kernel<BITS, false><<<grid, kThreadsD, 0, st>>>(a, group, n_groups, FastDiv(a.H));
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
