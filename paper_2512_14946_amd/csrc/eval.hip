// kvp_eval_configs: quality-loss proxy of every candidate (bits, group, keep_k) configuration of one
// context (the paper's profiler compresses a KV cache with every method and ratio of its pool and
// scores every version; this is the quality term of its utility function with the attention-output
// error standing in for the answer-similarity metric that needs model weights).
//
//   loss[c] = sqrt( sum (O_c - O_full)^2 / sum O_full^2 ),  O = softmax(Q K^T / sqrt(D)) V
//
// Pipeline (all on the caller's stream, scratch in the caller's workspace):
//   1. token scores of the unquantized K (kvp_score_tokens, causal, window forced);
//   2. one top-k keep list per distinct keep_k < T (kvp_select_topk's kernel); the keep-sets are
//      nested (the ranking is a total order), so the tokens split into shells: shell j holds the
//      tokens that enter the keep-set at the j-th smallest keep_k.  One kernel turns the lists into
//      a permutation of the tokens ordered by shell;
//   3. ONE stream per distinct (bits, group): attention of the window rows over the tokens in shell
//      order with K and V quantized and dequantized on the fly; at every shell boundary the running
//      output is the output of that keep level and is stored.  Every candidate keep level of a codec
//      therefore costs one pass over its largest keep-set instead of one pass each.  The 16-bit
//      stream also walks the tokens no level keeps: its last state is O_full (the reference);
//   4. sum (O_level - O_full)^2 per stored output and sum O_full^2 (compare kernel);
//   5. a reduction in a fixed order (deterministic) to loss[] and partial[].
//
// The attention kernel (step 3) walks the tokens in tiles of 32.  Per tile: 256 threads
// load 32 K rows and 32 V rows (16 lanes per row, 8 channels per lane), run the bit-exact group
// quantizer and dequantizer of quant_device.h on them, and stage K-hat and V-hat as bf16
// in LDS.  Each of the 4 waves owns 32 of the block's 128 query rows (stationary MFMA operand in
// registers) and computes S^T = K-hat Q^T with 8 v_mfma_f32_32x32x16_bf16, so a lane holds one
// query and 16 keys and the online-softmax statistics stay lane-private.  The P.V product has two
// implementations, chosen per call:
//   vector ALU, 16-bit operands (default): token pairs of the probabilities (rounded to fp16, nearest even) and
//     of V-hat (a bf16 value, exact in fp16 for 2^-14 <= |v| <= 65504; larger magnitudes become infinite and the
//     loss non-finite) go to LDS as packed halves, and each thread
//     accumulates an 8x8 tile of the 128x128 output in fp32 with v_dot2_f32_f16, two tokens per instruction (the
//     matrix cores are kept for the query x key contraction).  The row sums use the rounded probabilities, so every
//     output stays a convex combination of V-hat rows; rounding P moves the losses by less than 1e-4 relative;
//   vector ALU, fp32 (KVP_EVAL_PV_FP32): probabilities and V-hat in LDS as fp32, one fma per token and output;
//   matrix cores (KVP_EVAL_PV_MATRIX_CORES): O^T = V-hat^T P^T with V-hat exact in bf16 (it is a
//     dequantized value) and each probability split into two bf16 terms hi + lo (the loss is a
//     difference of two nearly equal outputs: rounding P to one bf16 moves the losses by 1e-3
//     relative; the two-term split leaves an error of 2^-18).  The probabilities never leave
//     registers: the tokens a lane holds after the logits tile are exactly the tokens its P^T
//     operand must hold, given a matching (permuted) token order in the V-hat^T operand, and the
//     per-query rescaling is lane-private.

#include "kvp_internal.h"
#include "quant_device.h"

namespace kvp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// implementations of the P.V product (template argument of attention_kernel)
constexpr int kPvDot2 = 0, kPvMatrix = 1, kPvFp32 = 2;

// resident waves per SIMD the attention kernel is compiled for (2 blocks per CU; 3 would spill)
#ifndef KVP_EVAL_WAVES_PER_SIMD
#define KVP_EVAL_WAVES_PER_SIMD 2
#endif
constexpr int kThreads = 256;
constexpr int kTile = 32;                  // tokens per tile
constexpr int kRowsPerBlock = 128;         // query rows per block
constexpr int kPitch = 136;                // bf16 elements per staged K row (272 B)
constexpr int kMaxCfgs = 64;
constexpr int kMaxLevels = 8;
constexpr float kLog2e = 1.4426950408889634f;

struct StreamDesc {
  int32_t bits, group;   // bits == 16: no quantization
};

struct EvalArgs {
  const uint16_t* q;
  int64_t q_sl, q_st, q_sh;
  const uint16_t* k;
  int64_t k_sl, k_st, k_sh;
  const uint16_t* v;
  int64_t v_sl, v_st, v_sh;
  int32_t T, W, G, Hkv, M, RB, L;
  float scale2;
  int32_t n_streams, n_cfgs, n_levels;
  int32_t level_k[kMaxLevels];           // ascending
  const int32_t* level_idx[kMaxLevels];  // [L*Hkv][k] ascending keep list, or null when k == T
  StreamDesc streams[kMaxCfgs + 1];      // + a hidden 16-bit stream when no configuration asks for one
  int32_t ref_stream;                    // the 16-bit stream: it walks all T tokens and doubles as the reference
  uint8_t cfg_stream[kMaxCfgs], cfg_level[kMaxCfgs];
  uint8_t* shell;   // [L*Hkv][T] scratch: index of the first keep level that holds the token
  int32_t* order;   // [L*Hkv][T] tokens ordered by shell, ascending inside a shell
  float* o_levels;  // [L*Hkv][RB][n_streams][n_levels + 1][128 x 128]: normalized output of a stream at each level
                    // (slot n_levels: the reference's state after all T tokens)
  float* den_part;  // [L*Hkv][RB]
  float* num_part;  // [L*Hkv][RB][n_streams][n_levels]
  double* layer_part;  // [L][n_cfgs][2] scratch of the final reduction
  float* loss;      // [n_cfgs]
  float* partial;   // [L][n_cfgs][2] or null
};

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

__device__ __forceinline__ uint32_t as_u32(half2_t h) {
  union { half2_t h; uint32_t u; } c;
  c.h = h;
  return c.u;
}
__device__ __forceinline__ half2_t as_half2(uint32_t u) {
  union { uint32_t u; half2_t h; } c;
  c.u = u;
  return c.h;
}
// two floats as packed halves, round to nearest even: exact for values fp16 holds, infinite beyond 65504 (so an
// out-of-range V-hat surfaces as a non-finite loss instead of a plausible wrong one)
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  typedef float float2_t __attribute__((ext_vector_type(2)));
  return as_u32(__builtin_convertvector(float2_t{lo, hi}, half2_t));
}

__device__ __forceinline__ int acc_row(int lane, int v) { return (lane >> 5) * 4 + (v >> 2) * 8 + (v & 3); }

// One lane's 8 channels of a row through quantize -> dequantize at (bits, group), returned as the
// 8 packed bf16 values decoding would read back (dequantized values are rounded to bf16, as
// kvp_dequantize_paged stores them).  bits and group are uniform across the block.
__device__ __forceinline__ uint4 fake_quant8(const uint4 raw, int bits, int group) {
  if (bits == 16) return raw;
  float x[8], q[8];
  unpack_bf16x8(raw, x);
  const float amax = group_max(abs_max8(x), group / 8);
  float scale;
  if (bits == 2) {
    const TernaryQuantizer tq(amax);
    tq.codes8(x, q);
    scale = amax;   // +-amax or 0
  } else if (bits == 4) {
    const GroupQuantizer<7> gq(amax);
    gq.codes8(x, q);
    scale = gq.scale;
  } else {
    const GroupQuantizer<127> gq(amax);
    gq.codes8(x, q);
    scale = gq.scale;
  }
  return make_uint4(pack_bf16x2(q[0] * scale, q[1] * scale), pack_bf16x2(q[2] * scale, q[3] * scale),
                    pack_bf16x2(q[4] * scale, q[5] * scale), pack_bf16x2(q[6] * scale, q[7] * scale));
}

__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// Tokens of one (layer, kv head) ordered by shell.  One 1024-thread block per row: the keep lists
// are scattered into a shell id per token (largest level first, so the smallest level wins), then a
// counting sort by (shell, token) writes the permutation.
constexpr int kOrderThreads = 1024;
__global__ __launch_bounds__(kOrderThreads) void build_order_kernel(const EvalArgs a) {
  __shared__ uint32_t count_s[kMaxLevels + 1][kOrderThreads];
  __shared__ uint32_t wave_s[kOrderThreads / 64];
  __shared__ uint32_t carry_s;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t lh = blockIdx.x;
  uint8_t* shell = a.shell + lh * a.T;
  int32_t* order = a.order + lh * a.T;
  const int n_shells = a.n_levels + 1;  // the last shell holds the tokens no keep level contains

  for (int t = tid; t < a.T; t += kOrderThreads) shell[t] = static_cast<uint8_t>(a.n_levels);
  __syncthreads();
  for (int j = a.n_levels - 1; j >= 0; --j) {
    const int32_t* list = a.level_idx[j];
    if (list) {
      list += lh * a.level_k[j];
      for (int i = tid; i < a.level_k[j]; i += kOrderThreads) shell[min(max(list[i], 0), a.T - 1)] = static_cast<uint8_t>(j);
    } else {
      for (int t = tid; t < a.T; t += kOrderThreads) shell[t] = static_cast<uint8_t>(j);
    }
    __syncthreads();
  }
  // thread tid owns the contiguous token range [t0, t1)
  const int per = (a.T + kOrderThreads - 1) / kOrderThreads;
  const int t0 = min(a.T, tid * per), t1 = min(a.T, t0 + per);
  for (int sidx = 0; sidx < n_shells; ++sidx) count_s[sidx][tid] = 0;
  for (int t = t0; t < t1; ++t) count_s[shell[t]][tid] += 1;
  if (tid == 0) carry_s = 0;
  __syncthreads();
  // exclusive scan over (shell major, thread minor); count_s becomes the first output slot
  for (int sidx = 0; sidx < n_shells; ++sidx) {
    const uint32_t mine = count_s[sidx][tid];
    uint32_t incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t n = __shfl_up(incl, off, 64);
      if (lane >= off) incl += n;
    }
    if (lane == 63) wave_s[wave] = incl;
    __syncthreads();
    uint32_t before = carry_s;
    for (int w = 0; w < wave; ++w) before += wave_s[w];
    count_s[sidx][tid] = before + incl - mine;
    __syncthreads();
    if (tid == kOrderThreads - 1) carry_s = before + incl;
    __syncthreads();
  }
  for (int t = t0; t < t1; ++t) {
    const uint32_t pos = count_s[shell[t]][tid]++;
    order[pos] = t;
  }
}

// V-hat^T in LDS.  The contraction index of the P.V product is the token, so the V-hat operand of a
// lane is 8 tokens of ONE channel: the tile is staged transposed, one row per channel, and a lane's
// 8 tokens of k-step ks are made the ones its accumulator of the logits tile already holds,
//   token(ks, half, e) = 16 ks + 8 (e >> 2) + 4 half + (e & 3),
// by storing token t = 16 ks + 8 b + 4 half + e' at column 16 ks + 8 half + 4 b + e'.  The
// probabilities then go from the softmax straight into the other operand without leaving registers.
// Channel ch lives in row (ch % 8) * 17 + ch / 8 with a row pitch of 80 bytes: the 16-byte operand
// reads of 8 adjacent lanes then cover all 32 banks, and so do the 8-byte transposing writes.
constexpr int kVtPitch = 40;                  // bf16 elements per row (32 used)
constexpr int kVtRows = 7 * 17 + 16;
__device__ __forceinline__ int vt_row(int ch) { return (ch & 7) * 17 + (ch >> 3); }

__device__ __forceinline__ bf16x8 v_operand(const uint16_t* vt_s, int ch, int ks, int half) {
  return as_bf16x8(*reinterpret_cast<const uint4*>(vt_s + vt_row(ch) * kVtPitch + 16 * ks + 8 * half));
}

// Staging of V-hat^T.  The four 16-lane rows of a wave hold four consecutive tokens (same 8
// channels in the same lane of each row); a 4x4 transpose of 32-bit words across the rows
// (v_permlane32_swap then v_permlane16_swap: each exchanges one lane-index bit with one register-index
// bit) leaves row j with channels 2j, 2j+1 of all four tokens, which are two 8-byte LDS writes.
__device__ __forceinline__ void stage_v_transposed(uint16_t* vt_s, uint4 vp, int q4, int part, int lane) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  u32x2 s02 = __builtin_amdgcn_permlane32_swap(vp.x, vp.z, false, false);
  u32x2 s13 = __builtin_amdgcn_permlane32_swap(vp.y, vp.w, false, false);
  u32x2 s01 = __builtin_amdgcn_permlane16_swap(s02[0], s13[0], false, false);
  u32x2 s23 = __builtin_amdgcn_permlane16_swap(s02[1], s13[1], false, false);
  const uint32_t t0 = s01[0], t1 = s01[1], t2 = s23[0], t3 = s23[1];   // channel pair j of tokens 0..3
  const int j = lane >> 4;
  // tokens 4 q4 .. 4 q4 + 3 land at columns 4 q' .. with q' = q4 with its two low bits exchanged
  const int col = 4 * ((q4 & 4) | ((q4 & 1) << 1) | ((q4 >> 1) & 1));
  const uint2 even = make_uint2((t0 & 0xffffu) | (t1 << 16), (t2 & 0xffffu) | (t3 << 16));
  const uint2 odd = make_uint2((t0 >> 16) | (t1 & 0xffff0000u), (t2 >> 16) | (t3 & 0xffff0000u));
  *reinterpret_cast<uint2*>(vt_s + vt_row(part * 8 + 2 * j) * kVtPitch + col) = even;
  *reinterpret_cast<uint2*>(vt_s + vt_row(part * 8 + 2 * j + 1) * kVtPitch + col) = odd;
}

// Work item of a block.  The streams of one (layer, kv head, row block) read the same K and V tiles, in the same
// order and at about the same pace.  Workgroups go to the 8 XCDs (each with its own L2) round-robin by linear
// id, so block b serves item (b mod 8) * ceil(items / 8) + b / 8: every XCD gets a contiguous run of items, with
// the stream index varying fastest, and the streams of a cell find each other's tiles in their XCD's L2.
struct WorkItem {
  int rb, lh, stream;
  bool valid;
};
constexpr int kXcds = 8;
__device__ __forceinline__ WorkItem work_item(const EvalArgs& a) {
  const int items = a.RB * a.L * a.Hkv * a.n_streams;
  const int per_xcd = (items + kXcds - 1) / kXcds;
  const int w = static_cast<int>(blockIdx.x % kXcds) * per_xcd + static_cast<int>(blockIdx.x / kXcds);
  WorkItem it;
  it.valid = static_cast<int>(blockIdx.x / kXcds) < per_xcd && w < items;
  it.stream = w % a.n_streams;
  const int cell = w / a.n_streams;
  it.rb = cell % a.RB;
  it.lh = cell / a.RB;
  return it;
}

// One launch covers every stream; the 16-bit stream also walks the tokens no keep level holds and so ends
// as the reference O_full.  Outputs are compared afterwards (compare_kernel).
// PV: how the P.V product is formed (kPvDot2: packed fp16 pairs on the vector ALU; kPvMatrix: two-term bf16 split
// of P on the matrix cores; kPvFp32: fp32 on the vector ALU).
template <int PV>
__global__ __launch_bounds__(kThreads, KVP_EVAL_WAVES_PER_SIMD) void attention_kernel(const EvalArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t k_s[kTile * kPitch];
  // V-hat: transposed bf16 for the matrix cores (see v_operand), or fp32 [token][channel] for the vector ALU
  constexpr bool PV_MFMA = PV == kPvMatrix;
  constexpr bool PV_FP32 = PV == kPvFp32;
  constexpr bool PV_DOT2 = PV == kPvDot2;
  __shared__ __attribute__((aligned(16))) uint16_t vt_s[PV_MFMA ? kVtRows * kVtPitch : 8];
  __shared__ __attribute__((aligned(16))) float v_s[PV_FP32 ? kTile * kHeadDim : 4];
  __shared__ __attribute__((aligned(16))) float p_s[PV_FP32 ? kTile * kRowsPerBlock : 4];
  // token pairs as packed halves: [pair][channel] and [pair][query row]; low half = the even token
  __shared__ __attribute__((aligned(16))) uint32_t v2_s[PV_DOT2 ? (kTile / 2) * kHeadDim : 4];
  __shared__ __attribute__((aligned(16))) uint32_t p2_s[PV_DOT2 ? (kTile / 2) * kRowsPerBlock : 4];
  __shared__ __attribute__((aligned(16))) float alpha_s[PV_MFMA ? 4 : kRowsPerBlock];
  __shared__ __attribute__((aligned(16))) float z_s[PV_MFMA ? 4 : kRowsPerBlock];
  __shared__ int tok_s[kTile];
  __shared__ int mask_s[2];   // per tile parity: some slot of the tile needs the causal / padding mask

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5;
  const WorkItem item = work_item(a);
  if (!item.valid) return;
  const int rb = item.rb, lh = item.lh, stream = item.stream;
  const int l = lh / a.Hkv, h = lh - l * a.Hkv;
  const int bits = a.streams[stream].bits, group = a.streams[stream].group;
  const bool is_ref = stream == a.ref_stream;
  const int32_t* order = a.order + static_cast<int64_t>(lh) * a.T;
  const uint16_t* kbase = a.k + static_cast<int64_t>(l) * a.k_sl + static_cast<int64_t>(h) * a.k_sh;
  const uint16_t* vbase = a.v + static_cast<int64_t>(l) * a.v_sl + static_cast<int64_t>(h) * a.v_sh;
  const int win0 = a.T - a.W;

  // stationary operand: this wave's 32 query rows
  bf16x8 q[8];
  const int qrow = rb * kRowsPerBlock + wave * 32 + (lane & 31);
  {
    if (qrow < a.M) {
      const int u = qrow / a.W, w = qrow - u * a.W;
      const uint16_t* row = a.q + static_cast<int64_t>(l) * a.q_sl + static_cast<int64_t>(w) * a.q_st +
                            static_cast<int64_t>(h * a.G + u) * a.q_sh;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) q[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(row + ks * 16 + half * 8));
    } else {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) q[ks] = as_bf16x8(make_uint4(0, 0, 0, 0));
    }
  }
  const int qpos = win0 + (qrow % a.W);
  float run_m = -INFINITY, run_z = 0.0f;  // per query (lane%32); run_z is this half-wave's share

  // Output accumulators, 64 per thread.
  //   matrix cores: O^T of this wave's 32 queries, o[16 ct + v] = channel 32 ct + acc_row(lane, v) of query lane%32
  //   vector ALU:   an 8x8 tile, o[8 i + j] = row {4ty.., 64+4ty..}[i], channel {4tx.., 64+4tx..}[j]
  float o[64];
#pragma unroll
  for (int i = 0; i < 64; ++i) o[i] = 0.0f;
  const int ty = tid >> 4, tx = tid & 15;
  // this block's output slots; each thread's 64 values of a level are contiguous
  float* levels_out = a.o_levels + (((static_cast<int64_t>(lh) * a.RB + rb) * a.n_streams + stream) * (a.n_levels + 1)) *
                                       (kRowsPerBlock * kHeadDim) + tid * 64;

  // segments end at the keep levels (tiles never straddle a level boundary, so the state at a
  // boundary is exactly that level's attention).  The 16-bit stream also walks the tokens no level
  // keeps (one more segment), which makes its final state the reference.
  const int n_seg = a.n_levels + ((is_ref && a.level_k[a.n_levels - 1] < a.T) ? 1 : 0);
  auto seg_end_of = [&](int sg) { return sg < a.n_levels ? a.level_k[sg] : a.T; };

  // Tile cursor: tile = positions [pos, min(pos + 32, end)) of segment seg.  Global loads run ahead of
  // the arithmetic: the permutation entries of a tile are fetched two tiles early and its K and V rows
  // one tile early, so neither of the two dependent latencies sits between two tiles.
  struct Cursor { int pos, seg, end; };
  auto advance = [&](Cursor c) {
    c.pos += kTile;
    if (c.pos >= c.end && c.seg < n_seg) {
      c.pos = c.end;
      c.seg += 1;
      if (c.seg < n_seg) c.end = seg_end_of(c.seg);
    }
    return c;
  };
  const int tk_a = tid >> 4, tk_b = (tid + kThreads) >> 4, part = tid & 15;   // this thread's two staging slots
  auto load_token = [&](const Cursor& c, int tk) {
    int t = 0x7fffffff;  // beyond every query position: masked
    if (c.seg < n_seg && c.pos + tk < c.end) t = min(max(order[c.pos + tk], 0), a.T - 1);
    return t;
  };
  auto load_row = [&](const uint16_t* base, int64_t stride, int t) {
    uint4 raw = make_uint4(0, 0, 0, 0);
    if (t != 0x7fffffff) raw = *reinterpret_cast<const uint4*>(base + static_cast<int64_t>(t) * stride + part * 8);
    return raw;
  };
  bool has_window = false;
  auto stage = [&](int tk, int t, const uint4 kraw, const uint4 vraw) {
    const uint4 kp = fake_quant8(kraw, bits, group), vp = fake_quant8(vraw, bits, group);
    *reinterpret_cast<uint4*>(k_s + tk * kPitch + part * 8) = kp;
    if constexpr (PV_MFMA) {
      stage_v_transposed(vt_s, vp, tk >> 2, part, lane);
    } else if constexpr (PV_DOT2) {
      // Tokens tk and tk ^ 1 sit 16 lanes apart (tk even: an even 16-lane row).  v_permlane16_swap exchanges the
      // first operand's odd rows with the second operand's even rows: afterwards the even token's lane holds
      // channels 0..3 of both tokens and the odd token's lane channels 4..7, even token first.
      typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
      const bool odd = (tk & 1) != 0;
      const u32x2 c01 = __builtin_amdgcn_permlane16_swap(vp.x, vp.z, false, false);
      const u32x2 c23 = __builtin_amdgcn_permlane16_swap(vp.y, vp.w, false, false);
      const uint32_t e0 = c01[0], o0 = c01[1], e1 = c23[0], o1 = c23[1];
      const uint4 packed = make_uint4(pack_f16x2(bf16lo(e0), bf16lo(o0)), pack_f16x2(bf16hi(e0), bf16hi(o0)),
                                      pack_f16x2(bf16lo(e1), bf16lo(o1)), pack_f16x2(bf16hi(e1), bf16hi(o1)));
      *reinterpret_cast<uint4*>(v2_s + (tk >> 1) * kHeadDim + part * 8 + (odd ? 4 : 0)) = packed;
    } else {
      float* vrow = v_s + tk * kHeadDim + part * 8;
      *reinterpret_cast<float4*>(vrow) = make_float4(bf16lo(vp.x), bf16hi(vp.x), bf16lo(vp.y), bf16hi(vp.y));
      *reinterpret_cast<float4*>(vrow + 4) = make_float4(bf16lo(vp.z), bf16hi(vp.z), bf16lo(vp.w), bf16hi(vp.w));
    }
    if (part == 0) tok_s[tk] = t;
    has_window |= (t >= win0);   // window tokens and padding slots of a ragged tile need the mask
  };

  Cursor cur{0, 0, seg_end_of(0)};
  Cursor nxt = advance(cur);
  int t_a = load_token(cur, tk_a), t_b = load_token(cur, tk_b);
  uint4 k_a = load_row(kbase, a.k_st, t_a), v_a = load_row(vbase, a.v_st, t_a);
  uint4 k_b = load_row(kbase, a.k_st, t_b), v_b = load_row(vbase, a.v_st, t_b);
  int tn_a = load_token(nxt, tk_a), tn_b = load_token(nxt, tk_b);

  if (tid == 0) mask_s[0] = mask_s[1] = 0;
  int parity = 0;
  while (cur.seg < n_seg) {
    const int seg = cur.seg;
    {
      __syncthreads();  // the previous tile's LDS is no longer read
      if (tid == 0) mask_s[parity ^ 1] = 0;   // the previous tile's flag has been read by everybody
      // ---- stage 32 tokens: K-hat and V-hat (the dequantized values are bf16 values) ----
      has_window = false;
      stage(tk_a, t_a, k_a, v_a);
      stage(tk_b, t_b, k_b, v_b);
      if (has_window) mask_s[parity] = 1;     // rare; every writer stores the same value
      // ---- run ahead: rows of the next tile, permutation entries of the one after ----
      const Cursor nn = advance(nxt);
      t_a = tn_a;
      t_b = tn_b;
      k_a = load_row(kbase, a.k_st, t_a);
      v_a = load_row(vbase, a.v_st, t_a);
      k_b = load_row(kbase, a.k_st, t_b);
      v_b = load_row(vbase, a.v_st, t_b);
      tn_a = load_token(nn, tk_a);
      tn_b = load_token(nn, tk_b);
      cur = nxt;
      nxt = nn;
      __syncthreads();                         // publishes the stage and the flag
      const bool need_mask = mask_s[parity] != 0;
      parity ^= 1;

      // ---- logits of 32 keys x this wave's 32 queries, online softmax ----
      floatx16 acc = {0};
      {
        const uint16_t* krow = k_s + (lane & 31) * kPitch + half * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(*reinterpret_cast<const uint4*>(krow + ks * 16)),
                                                        q[ks], acc, 0, 0, 0);
      }
      if (need_mask) {
        asm volatile("" ::: "memory");  // keep this a real (block-uniform, rarely taken) branch
#pragma unroll
        for (int vv = 0; vv < 16; ++vv)
          if (tok_s[acc_row(lane, vv)] > qpos) acc[vv] = -INFINITY;
      }
      float tmax = acc[0];
#pragma unroll
      for (int vv = 1; vv < 16; ++vv) tmax = fmaxf(tmax, acc[vv]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      const float m_new = fmaxf(run_m, tmax * a.scale2);  // scale2 > 0: max commutes with it
      const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(run_m - m_safe);
      run_m = m_new;

      if constexpr (PV_MFMA) {
        // probabilities, split into two bf16 terms p = hi + lo (|p - hi - lo| <= 2^-18 p): the product
        // with the bf16-exact V-hat then carries fp32-like accuracy through two matrix instructions
        uint32_t p_hi[8], p_lo[8];
        float zsum = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(acc[2 * e], a.scale2, -m_safe));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(acc[2 * e + 1], a.scale2, -m_safe));
          zsum += p0 + p1;
          p_hi[e] = pack_bf16x2(p0, p1);
          p_lo[e] = pack_bf16x2(p0 - bf16lo(p_hi[e]), p1 - bf16hi(p_hi[e]));
        }
        run_z = run_z * alpha + zsum;
        // ---- O^T = O^T * alpha + V-hat^T P^T on the matrix cores ----
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {   // the running maximum moved for some query of the wave
#pragma unroll
          for (int i = 0; i < 64; ++i) o[i] *= alpha;
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const bf16x8 bh = as_bf16x8(make_uint4(p_hi[4 * ks], p_hi[4 * ks + 1], p_hi[4 * ks + 2], p_hi[4 * ks + 3]));
          const bf16x8 bl = as_bf16x8(make_uint4(p_lo[4 * ks], p_lo[4 * ks + 1], p_lo[4 * ks + 2], p_lo[4 * ks + 3]));
          bf16x8 vt[4];
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) vt[ct] = v_operand(vt_s, 32 * ct + (lane & 31), ks, half);
          // the four channel tiles are independent accumulation chains: interleave them
#pragma unroll
          for (int pass = 0; pass < 2; ++pass)
#pragma unroll
            for (int ct = 0; ct < 4; ++ct) {
              floatx16 oc;
#pragma unroll
              for (int vv = 0; vv < 16; ++vv) oc[vv] = o[16 * ct + vv];
              oc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt[ct], pass == 0 ? bh : bl, oc, 0, 0, 0);
#pragma unroll
              for (int vv = 0; vv < 16; ++vv) o[16 * ct + vv] = oc[vv];
            }
        }
      } else {
        float zsum = 0.0f;
        const int rloc = wave * 32 + (lane & 31);
        if constexpr (PV_DOT2) {
          // probabilities to LDS as fp16 pairs of adjacent tokens, [pair][query row]; the row sum takes the rounded values
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float p0 = __builtin_amdgcn_exp2f(fmaf(acc[2 * e], a.scale2, -m_safe));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(acc[2 * e + 1], a.scale2, -m_safe));
            typedef float float2_t __attribute__((ext_vector_type(2)));
            const half2_t ph = __builtin_convertvector(float2_t{p0, p1}, half2_t);   // round to nearest even
            zsum = __builtin_amdgcn_fdot2(ph, half2_t{1, 1}, zsum, false);
            p2_s[(acc_row(lane, 2 * e) >> 1) * kRowsPerBlock + rloc] = as_u32(ph);
          }
        } else {
          // probabilities to LDS in fp32, [token][query row]
#pragma unroll
          for (int vv = 0; vv < 16; ++vv) {
            const float p = __builtin_amdgcn_exp2f(fmaf(acc[vv], a.scale2, -m_safe));
            zsum += p;
            p_s[acc_row(lane, vv) * kRowsPerBlock + rloc] = p;
          }
        }
        run_z = run_z * alpha + zsum;
        if (lane < 32) alpha_s[rloc] = alpha;
        __syncthreads();
        // ---- O = O * alpha + P V-hat on the vector ALU, fp32 accumulation ----
        const float4 a0 = *reinterpret_cast<const float4*>(alpha_s + 4 * ty);
        const float4 a1 = *reinterpret_cast<const float4*>(alpha_s + 64 + 4 * ty);
        const float al[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
        bool moved = false;
#pragma unroll
        for (int i = 0; i < 8; ++i) moved |= al[i] != 1.0f;
        if (__builtin_amdgcn_ballot_w64(moved)) {   // the running maximum of one of this wave's rows moved
#pragma unroll
          for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j) o[8 * i + j] *= al[i];
        }
        if constexpr (PV_DOT2) {
#pragma unroll 4
          for (int tp = 0; tp < kTile / 2; ++tp) {
            const uint4 p0 = *reinterpret_cast<const uint4*>(p2_s + tp * kRowsPerBlock + 4 * ty);
            const uint4 p1 = *reinterpret_cast<const uint4*>(p2_s + tp * kRowsPerBlock + 64 + 4 * ty);
            const uint4 v0 = *reinterpret_cast<const uint4*>(v2_s + tp * kHeadDim + 4 * tx);
            const uint4 v1 = *reinterpret_cast<const uint4*>(v2_s + tp * kHeadDim + 64 + 4 * tx);
            const uint32_t pr[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
            const uint32_t vc[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
              for (int j = 0; j < 8; ++j)
                o[8 * i + j] = __builtin_amdgcn_fdot2(as_half2(pr[i]), as_half2(vc[j]), o[8 * i + j], false);
          }
        } else {
#pragma unroll 4
          for (int tk = 0; tk < kTile; ++tk) {
            const float4 p0 = *reinterpret_cast<const float4*>(p_s + tk * kRowsPerBlock + 4 * ty);
            const float4 p1 = *reinterpret_cast<const float4*>(p_s + tk * kRowsPerBlock + 64 + 4 * ty);
            const float4 v0 = *reinterpret_cast<const float4*>(v_s + tk * kHeadDim + 4 * tx);
            const float4 v1 = *reinterpret_cast<const float4*>(v_s + tk * kHeadDim + 64 + 4 * tx);
            const float pr[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
            const float vc[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
              for (int j = 0; j < 8; ++j) o[8 * i + j] = fmaf(pr[i], vc[j], o[8 * i + j]);
          }
        }
      }
    }
    if (cur.seg == seg) continue;                      // more tiles in this segment

    // ---- end of a segment: store the normalized output of this level ----
    float inv[8];      // 1 / row sum of the rows this thread's accumulators belong to
    if constexpr (PV_MFMA) {
      const float one = 1.0f / (run_z + __shfl_xor(run_z, 32, 64));
#pragma unroll
      for (int i = 0; i < 8; ++i) inv[i] = one;
    } else {
      const float z = run_z + __shfl_xor(run_z, 32, 64);
      __syncthreads();
      if (lane < 32) z_s[wave * 32 + lane] = z;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 8; ++i) inv[i] = 1.0f / z_s[(i < 4) ? 4 * ty + i : 64 + 4 * ty + (i - 4)];
    }
    float4* cell = reinterpret_cast<float4*>(levels_out + static_cast<int64_t>(seg) * (kRowsPerBlock * kHeadDim));
#pragma unroll
    for (int i = 0; i < 8; ++i)       // accumulators 8 i .. 8 i + 7 share a row in the vector-ALU layout
#pragma unroll
      for (int jh = 0; jh < 2; ++jh) {
        const int e = 8 * i + 4 * jh;
        cell[e >> 2] = make_float4(o[e] * inv[i], o[e + 1] * inv[i], o[e + 2] * inv[i], o[e + 3] * inv[i]);
      }
    // the reference state is the last one the 16-bit stream reaches; keep it in the extra slot as well
    if (is_ref && seg == n_seg - 1 && seg != a.n_levels) {
      float4* last = reinterpret_cast<float4*>(levels_out + static_cast<int64_t>(a.n_levels) * (kRowsPerBlock * kHeadDim));
#pragma unroll
      for (int q4 = 0; q4 < 16; ++q4) last[q4] = cell[q4];
    }
  }
}

// Squared distances between every stored level of every stream and the reference, and the reference's own
// squared norm; one block per (row block, layer x head, stream).  A stored output is 256 runs of 64 floats (one
// run per thread of attention_kernel); here consecutive threads read consecutive 16-byte pieces, and the
// query row a piece belongs to follows from its position.
template <bool PV_MFMA>
__global__ __launch_bounds__(kThreads) void compare_kernel(const EvalArgs a) {
  __shared__ float red_s[4];
  const int tid = threadIdx.x;
  const WorkItem item = work_item(a);
  if (!item.valid) return;
  const int rb = item.rb, lh = item.lh, st = item.stream;
  const int64_t cellrow = static_cast<int64_t>(lh) * a.RB + rb;
  const int64_t per_level = kRowsPerBlock * kHeadDim;
  const float4* ref = reinterpret_cast<const float4*>(
      a.o_levels + ((cellrow * a.n_streams + a.ref_stream) * (a.n_levels + 1) + a.n_levels) * per_level);
  // piece f = 256 j + tid is piece (f mod 16) of the run of writer thread f / 16 = 16 j + tid / 16
  const int q4 = tid & 15, i = q4 >> 1;   // accumulators 8 i .. 8 i + 7 of the writer
  bool live[16];
  float4 r[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int writer = 16 * j + (tid >> 4);
    const int ty = writer >> 4;
    const int rloc = PV_MFMA ? (writer >> 6) * 32 + (writer & 31) : ((i < 4) ? 4 * ty + i : 64 + 4 * ty + (i - 4));
    live[j] = rb * kRowsPerBlock + rloc < a.M;
    r[j] = ref[256 * j + tid];
  }
  if (st == a.ref_stream) {
    float sq = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (live[j]) sq += r[j].x * r[j].x + r[j].y * r[j].y + r[j].z * r[j].z + r[j].w * r[j].w;
    const float total = block_sum(sq, red_s);
    if (tid == 0) a.den_part[cellrow] = total;
  }
  for (int lev = 0; lev < a.n_levels; ++lev) {
    const float4* val =
        reinterpret_cast<const float4*>(a.o_levels + ((cellrow * a.n_streams + st) * (a.n_levels + 1) + lev) * per_level);
    float sq = 0.0f;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const float4 v = val[256 * j + tid];
      const float dx = v.x - r[j].x, dy = v.y - r[j].y, dz = v.z - r[j].z, dw = v.w - r[j].w;
      if (live[j]) sq += dx * dx + dy * dy + dz * dz + dw * dw;
    }
    const float total = block_sum(sq, red_s);
    if (tid == 0) a.num_part[(cellrow * a.n_streams + st) * a.n_levels + lev] = total;
  }
}

// Fixed-order reduction.  Thread (c, l) sums one layer of one configuration over kv heads and row
// blocks; then thread c adds the layers in order.
constexpr int kFinishThreads = 1024;
__global__ __launch_bounds__(kFinishThreads) void finish_kernel(const EvalArgs a) {
  double* layer_s = a.layer_part;  // [L][n_cfgs][2]
  for (int item = threadIdx.x; item < a.n_cfgs * a.L; item += kFinishThreads) {
    const int c = item % a.n_cfgs, l = item / a.n_cfgs;
    const int s = a.cfg_stream[c], lev = a.cfg_level[c];
    double num_l = 0.0, den_l = 0.0;
    for (int h = 0; h < a.Hkv; ++h)
      for (int rb = 0; rb < a.RB; ++rb) {
        const int64_t cell = (static_cast<int64_t>(l) * a.Hkv + h) * a.RB + rb;
        num_l += static_cast<double>(a.num_part[(cell * a.n_streams + s) * a.n_levels + lev]);
        den_l += static_cast<double>(a.den_part[cell]);
      }
    layer_s[(l * a.n_cfgs + c) * 2 + 0] = num_l;
    layer_s[(l * a.n_cfgs + c) * 2 + 1] = den_l;
    if (a.partial) {
      a.partial[(static_cast<int64_t>(l) * a.n_cfgs + c) * 2 + 0] = static_cast<float>(num_l);
      a.partial[(static_cast<int64_t>(l) * a.n_cfgs + c) * 2 + 1] = static_cast<float>(den_l);
    }
  }
  __syncthreads();
  if (static_cast<int>(threadIdx.x) < a.n_cfgs) {
    const int c = threadIdx.x;
    double num = 0.0, den = 0.0;
    for (int l = 0; l < a.L; ++l) {
      num += layer_s[(l * a.n_cfgs + c) * 2 + 0];
      den += layer_s[(l * a.n_cfgs + c) * 2 + 1];
    }
    a.loss[c] = static_cast<float>(sqrt(num / den));
  }
}

size_t align256(size_t n) { return (n + 255) / 256 * 256; }

struct EvalPlan {
  int64_t LH, M, RB;
  size_t score_ws, select_ws, scores, idx, shell, order, o_levels, den, num, layer, total;
};

EvalPlan make_plan(int64_t L, int64_t Hkv, int64_t Hq, int64_t W, int64_t T, int32_t n_cfgs) {
  EvalPlan p{};
  p.LH = L * Hkv;
  p.M = (Hq / Hkv) * W;
  p.RB = ceil_div(p.M, kRowsPerBlock);
  const int64_t cfgs = n_cfgs > 0 ? n_cfgs : 1;
  const int64_t levels = cfgs < kMaxLevels ? cfgs : kMaxLevels;
  p.score_ws = align256(kvp_score_workspace_bytes(L, Hkv, Hq, W, T));
  p.select_ws = align256(select_workspace_bytes(p.LH, T));   // shared by the keep levels (same stream)
  p.scores = align256(static_cast<size_t>(p.LH) * T * sizeof(float));
  p.idx = align256(static_cast<size_t>(levels) * p.LH * T * sizeof(int32_t));
  p.shell = align256(static_cast<size_t>(p.LH) * T);
  p.order = align256(static_cast<size_t>(p.LH) * T * sizeof(int32_t));
  // distinct codecs: at most 3 bit widths x 3 group sizes, plus the 16-bit one (listed or hidden)
  const int64_t streams = cfgs + 1 < 10 ? cfgs + 1 : 10;
  p.o_levels = align256(static_cast<size_t>(p.LH) * p.RB * streams * (levels + 1) * kRowsPerBlock * kHeadDim * sizeof(float));
  p.den = align256(static_cast<size_t>(p.LH) * p.RB * sizeof(float));
  p.num = align256(static_cast<size_t>(p.LH) * p.RB * streams * levels * sizeof(float));
  p.layer = align256(static_cast<size_t>(L) * cfgs * 2 * sizeof(double));
  p.total = p.score_ws + p.select_ws + p.scores + p.idx + p.shell + p.order + p.o_levels + p.den + p.num + p.layer;
  return p;
}

}  // namespace
}  // namespace kvp

extern "C" size_t kvp_eval_workspace_bytes(int64_t L, int64_t Hkv, int64_t Hq, int64_t W, int64_t T, int32_t n_cfgs) {
  if (L <= 0 || Hkv <= 0 || Hq <= 0 || W <= 0 || T <= 0 || Hq % Hkv != 0 || n_cfgs < 0) return 0;
  return kvp::make_plan(L, Hkv, Hq, W, T, n_cfgs).total;
}

extern "C" int32_t kvp_eval_configs_ex(const kvp_view* q_win, const kvp_view* k, const kvp_view* v,
                                       const kvp_config* cfgs, int32_t n_cfgs, float* loss, float* partial, void* ws,
                                       size_t ws_bytes, uint32_t flags, void* stream) {
  using namespace kvp;
  if (flags & ~static_cast<uint32_t>(KVP_EVAL_PV_MATRIX_CORES | KVP_EVAL_PV_FP32)) return KVP_ERR_UNSUPPORTED;
  if ((flags & KVP_EVAL_PV_MATRIX_CORES) && (flags & KVP_EVAL_PV_FP32)) return KVP_ERR_UNSUPPORTED;
  int32_t rc = check_view(q_win);
  if (rc != KVP_OK) return rc;
  rc = check_view(k);
  if (rc != KVP_OK) return rc;
  rc = check_view(v);
  if (rc != KVP_OK) return rc;
  if (n_cfgs < 0) return KVP_ERR_SHAPE;
  if (n_cfgs == 0) return KVP_OK;
  if (!cfgs || !loss) return KVP_ERR_NULL;
  if (n_cfgs > kMaxCfgs) return KVP_ERR_UNSUPPORTED;
  const int64_t L = k->L, T = k->T, Hkv = k->H, Hq = q_win->H, W = q_win->T;
  if (v->L != L || v->T != T || v->H != Hkv || q_win->L != L || Hq % Hkv != 0 || W > T) return KVP_ERR_SHAPE;
  if (L * Hkv > 65535 || T >= (1ll << 30)) return KVP_ERR_SHAPE;

  EvalArgs a{};
  // distinct keep levels (ascending) and distinct (bits, group) streams
  for (int32_t c = 0; c < n_cfgs; ++c) {
    const kvp_config& cf = cfgs[c];
    if (cf.bits != 16 && cf.bits != 8 && cf.bits != 4 && cf.bits != 2) return KVP_ERR_UNSUPPORTED;
    if (cf.bits != 16 && cf.group != 32 && cf.group != 64 && cf.group != 128) return KVP_ERR_UNSUPPORTED;
    if (cf.keep_k < 1 || cf.keep_k > T) return KVP_ERR_SHAPE;
    bool known = false;
    for (int j = 0; j < a.n_levels; ++j) known |= a.level_k[j] == cf.keep_k;
    if (!known) {
      if (a.n_levels == kMaxLevels) return KVP_ERR_UNSUPPORTED;
      int j = a.n_levels++;
      for (; j > 0 && a.level_k[j - 1] > cf.keep_k; --j) a.level_k[j] = a.level_k[j - 1];  // insertion sort
      a.level_k[j] = static_cast<int32_t>(cf.keep_k);
    }
  }
  for (int32_t c = 0; c < n_cfgs; ++c) {
    const kvp_config& cf = cfgs[c];
    for (int j = 0; j < a.n_levels; ++j)
      if (a.level_k[j] == cf.keep_k) a.cfg_level[c] = static_cast<uint8_t>(j);
    const int32_t grp = cf.bits == 16 ? 128 : cf.group;
    int s = -1;
    for (int j = 0; j < a.n_streams; ++j)
      if (a.streams[j].bits == cf.bits && a.streams[j].group == grp) s = j;
    if (s < 0) {
      s = a.n_streams++;
      a.streams[s] = StreamDesc{cf.bits, grp};
    }
    a.cfg_stream[c] = static_cast<uint8_t>(s);
  }

  a.ref_stream = -1;
  for (int j = 0; j < a.n_streams; ++j)
    if (a.streams[j].bits == 16) a.ref_stream = j;
  if (a.ref_stream < 0) {
    a.ref_stream = a.n_streams++;
    a.streams[a.ref_stream] = StreamDesc{16, 128};
  }
  // the reference stream walks the most tokens: give it the lowest block indices so that its blocks start first
  if (a.ref_stream != 0) {
    const StreamDesc first = a.streams[0];
    a.streams[0] = a.streams[a.ref_stream];
    a.streams[a.ref_stream] = first;
    for (int32_t c = 0; c < n_cfgs; ++c) {
      if (a.cfg_stream[c] == 0)
        a.cfg_stream[c] = static_cast<uint8_t>(a.ref_stream);
      else if (a.cfg_stream[c] == a.ref_stream)
        a.cfg_stream[c] = 0;
    }
    a.ref_stream = 0;
  }

  const EvalPlan p = make_plan(L, Hkv, Hq, W, T, n_cfgs);
  if (!ws || ws_bytes < p.total || (reinterpret_cast<uintptr_t>(ws) & 15u)) return KVP_ERR_WORKSPACE;
  char* cursor = static_cast<char*>(ws);
  auto take = [&cursor](size_t bytes) { char* r = cursor; cursor += bytes; return r; };
  void* score_ws = take(p.score_ws);
  void* select_ws = take(p.select_ws);
  float* scores = reinterpret_cast<float*>(take(p.scores));
  int32_t* idx = reinterpret_cast<int32_t*>(take(p.idx));
  a.shell = reinterpret_cast<uint8_t*>(take(p.shell));
  a.order = reinterpret_cast<int32_t*>(take(p.order));
  a.o_levels = reinterpret_cast<float*>(take(p.o_levels));
  a.den_part = reinterpret_cast<float*>(take(p.den));
  a.num_part = reinterpret_cast<float*>(take(p.num));
  a.layer_part = reinterpret_cast<double*>(take(p.layer));

  a.q = static_cast<const uint16_t*>(q_win->ptr);
  a.q_sl = q_win->stride_l; a.q_st = q_win->stride_t; a.q_sh = q_win->stride_h;
  a.k = static_cast<const uint16_t*>(k->ptr);
  a.k_sl = k->stride_l; a.k_st = k->stride_t; a.k_sh = k->stride_h;
  a.v = static_cast<const uint16_t*>(v->ptr);
  a.v_sl = v->stride_l; a.v_st = v->stride_t; a.v_sh = v->stride_h;
  a.T = static_cast<int32_t>(T); a.W = static_cast<int32_t>(W); a.G = static_cast<int32_t>(Hq / Hkv);
  a.Hkv = static_cast<int32_t>(Hkv); a.M = static_cast<int32_t>(p.M); a.RB = static_cast<int32_t>(p.RB);
  a.L = static_cast<int32_t>(L);
  a.scale2 = kLog2e / sqrtf(static_cast<float>(kHeadDim));
  a.n_cfgs = n_cfgs;
  a.loss = loss;
  a.partial = partial;

  const int64_t items = static_cast<int64_t>(p.RB) * p.LH * a.n_streams;
  if (items >= (1ll << 30)) return KVP_ERR_SHAPE;   // before anything is enqueued
  const hipStream_t st = as_stream(stream);
  rc = score_tokens_impl(q_win, k, 1, 1, scores, score_ws, p.score_ws, st);
  if (rc != KVP_OK) return rc;
  for (int j = 0; j < a.n_levels; ++j) {
    if (a.level_k[j] == T) {
      a.level_idx[j] = nullptr;  // every token
    } else {
      int32_t* out = idx + static_cast<int64_t>(j) * p.LH * T;
      select_topk_launch(scores, p.LH, T, T, a.level_k[j], out, select_ws, st);
      a.level_idx[j] = out;
    }
  }
  build_order_kernel<<<dim3(static_cast<unsigned>(p.LH)), kOrderThreads, 0, st>>>(a);
  const dim3 grid(static_cast<unsigned>(kXcds * ceil_div(items, kXcds)));
  if (flags & KVP_EVAL_PV_MATRIX_CORES) {
    attention_kernel<kPvMatrix><<<grid, kThreads, 0, st>>>(a);
    compare_kernel<true><<<grid, kThreads, 0, st>>>(a);
  } else if (flags & KVP_EVAL_PV_FP32) {
    attention_kernel<kPvFp32><<<grid, kThreads, 0, st>>>(a);
    compare_kernel<false><<<grid, kThreads, 0, st>>>(a);
  } else {
    attention_kernel<kPvDot2><<<grid, kThreads, 0, st>>>(a);
    compare_kernel<false><<<grid, kThreads, 0, st>>>(a);
  }
  finish_kernel<<<1, kFinishThreads, 0, st>>>(a);
  return launch_status();
}

extern "C" int32_t kvp_eval_configs(const kvp_view* q_win, const kvp_view* k, const kvp_view* v, const kvp_config* cfgs,
                                    int32_t n_cfgs, float* loss, float* partial, void* ws, size_t ws_bytes,
                                    void* stream) {
  return kvp_eval_configs_ex(q_win, k, v, cfgs, n_cfgs, loss, partial, ws, ws_bytes, 0u, stream);
}
