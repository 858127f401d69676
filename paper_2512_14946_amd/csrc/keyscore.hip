// kvp_score_keys: key-only token importance of the paper's two other token-dropping methods
// (Evaluation, Baselines):
//   knorm   score[t] = ||k_t||_2                                  (tokens with a low norm are dropped)
//   keydiff score[t] = - mean over t' != t of cos(k_t, k_t')       (tokens similar to the rest are dropped)
// Both feed kvp_select_topk (keep the largest scores).
//
// keydiff is evaluated in closed form: with unit keys u_t = k_t / ||k_t|| and S = sum_t u_t,
//   mean_{t' != t} cos = (u_t . S - |u_t|^2) / (T - 1),
// so it costs two streaming passes over K instead of T^2 dot products: pass 1 reduces S per
// (layer, head) in a fixed order (per-chunk partials, then a small second kernel: deterministic),
// pass 2 scores every token.  HBM-bound: one (knorm) or two (keydiff) reads of K.
//
// Mapping: a row (one token of one head, 256 B) is read by 16 adjacent lanes with one 128-bit
// streaming load each; sums over a row are 4 DPP adds inside the 16-lane row.  A 256-thread block
// covers kTokensPerBlock tokens of one (layer, head).

#include "kvp_internal.h"

namespace kvp {
namespace {

constexpr int kThreads = 256;
constexpr int kRowsPerStep = kThreads / kLanesPerRow;   // 16 tokens per step
constexpr int kSteps = 4;
constexpr int kTokensPerBlock = kRowsPerStep * kSteps;  // 64: knorm / keydiff pass 2
constexpr int kSumTokens = 2048;                        // tokens per block in keydiff pass 1

struct KeyArgs {
  const uint16_t* k;
  int64_t k_sl, k_st, k_sh;
  int32_t T, H, n_chunks;
  float* partial;   // [L*H][n_chunks][128]
  float* sum;       // [L*H][128]
  float* scores;    // [L*H][T]
};

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
// sum over the 16 lanes of a DPP row; every lane gets the total
__device__ __forceinline__ float row_sum16(float v) {
  v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]
  v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]
  v = dpp_add<0x141>(v);   // row_half_mirror
  v = dpp_add<0x140>(v);   // row_mirror
  return v;
}

__device__ __forceinline__ void unpack8(const uint4 raw, float x[8]) {
  const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = bf16lo(w[i]);
    x[2 * i + 1] = bf16hi(w[i]);
  }
}

// KEYDIFF false: knorm.  KEYDIFF true: pass 2 of keydiff (a.sum holds S).
template <bool KEYDIFF>
__global__ __launch_bounds__(kThreads) void key_score_kernel(const KeyArgs a) {
  const int lane_in_row = threadIdx.x & (kLanesPerRow - 1);
  const int row_in_step = threadIdx.x / kLanesPerRow;
  const int lh = blockIdx.y;
  const int l = lh / a.H, h = lh - l * a.H;
  const uint16_t* kbase = a.k + static_cast<int64_t>(l) * a.k_sl + static_cast<int64_t>(h) * a.k_sh + lane_in_row * 8;
  const int t0 = blockIdx.x * kTokensPerBlock + row_in_step;
  float s[8];
  if constexpr (KEYDIFF) {
    const float4 s0 = *reinterpret_cast<const float4*>(a.sum + static_cast<int64_t>(lh) * kHeadDim + lane_in_row * 8);
    const float4 s1 = *reinterpret_cast<const float4*>(a.sum + static_cast<int64_t>(lh) * kHeadDim + lane_in_row * 8 + 4);
    s[0] = s0.x; s[1] = s0.y; s[2] = s0.z; s[3] = s0.w; s[4] = s1.x; s[5] = s1.y; s[6] = s1.z; s[7] = s1.w;
  }
  uint4 raw[kSteps];
#pragma unroll
  for (int i = 0; i < kSteps; ++i) {
    const int t = t0 + i * kRowsPerStep;
    raw[i] = make_uint4(0, 0, 0, 0);
    if (t < a.T) raw[i] = load_stream16(kbase + static_cast<int64_t>(t) * a.k_st);
  }
  const float inv_others = a.T > 1 ? 1.0f / static_cast<float>(a.T - 1) : 0.0f;
#pragma unroll
  for (int i = 0; i < kSteps; ++i) {
    const int t = t0 + i * kRowsPerStep;
    float x[8];
    unpack8(raw[i], x);
    float ss = 0.0f, dot = 0.0f;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      ss = fmaf(x[c], x[c], ss);
      if constexpr (KEYDIFF) dot = fmaf(x[c], s[c], dot);
    }
    ss = row_sum16(ss);
    float score;
    if constexpr (KEYDIFF) {
      dot = row_sum16(dot);
      // u . S - |u|^2 with u = k / sqrt(ss); a zero key has cosine 0 with everything
      score = ss > 0.0f ? -(dot / sqrtf(ss) - 1.0f) * inv_others : 0.0f;
    } else {
      score = sqrtf(ss);
    }
    if (lane_in_row == 0 && t < a.T) a.scores[static_cast<int64_t>(lh) * a.T + t] = score;
  }
}

// keydiff pass 1: partial[lh][chunk][:] = sum over the chunk's tokens of k_t / ||k_t||
__global__ __launch_bounds__(kThreads) void unit_key_sum_kernel(const KeyArgs a) {
  __shared__ float red[kRowsPerStep][kHeadDim];
  const int lane_in_row = threadIdx.x & (kLanesPerRow - 1);
  const int row_in_step = threadIdx.x / kLanesPerRow;
  const int lh = blockIdx.y;
  const int l = lh / a.H, h = lh - l * a.H;
  const uint16_t* kbase = a.k + static_cast<int64_t>(l) * a.k_sl + static_cast<int64_t>(h) * a.k_sh + lane_in_row * 8;
  const int c_begin = blockIdx.x * kSumTokens;
  const int c_end = min(a.T, c_begin + kSumTokens);
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int tb = c_begin + row_in_step; tb < c_end; tb += kRowsPerStep * kSteps) {
    uint4 raw[kSteps];
#pragma unroll
    for (int i = 0; i < kSteps; ++i) {
      const int t = tb + i * kRowsPerStep;
      raw[i] = make_uint4(0, 0, 0, 0);
      if (t < c_end) raw[i] = load_stream16(kbase + static_cast<int64_t>(t) * a.k_st);
    }
#pragma unroll
    for (int i = 0; i < kSteps; ++i) {
      float x[8];
      unpack8(raw[i], x);
      float ss = 0.0f;
#pragma unroll
      for (int c = 0; c < 8; ++c) ss = fmaf(x[c], x[c], ss);
      ss = row_sum16(ss);
      const float inv = ss > 0.0f ? 1.0f / sqrtf(ss) : 0.0f;   // zero rows (also the padding) add nothing
#pragma unroll
      for (int c = 0; c < 8; ++c) acc[c] = fmaf(x[c], inv, acc[c]);
    }
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) red[row_in_step][lane_in_row * 8 + c] = acc[c];
  __syncthreads();
  if (threadIdx.x < kHeadDim) {
    float sum = 0.0f;
#pragma unroll
    for (int r = 0; r < kRowsPerStep; ++r) sum += red[r][threadIdx.x];
    a.partial[(static_cast<int64_t>(lh) * a.n_chunks + blockIdx.x) * kHeadDim + threadIdx.x] = sum;
  }
}

__global__ void chunk_sum_kernel(const KeyArgs a) {
  const int lh = blockIdx.x;
  if (threadIdx.x < kHeadDim) {
    float sum = 0.0f;
    for (int c = 0; c < a.n_chunks; ++c) sum += a.partial[(static_cast<int64_t>(lh) * a.n_chunks + c) * kHeadDim + threadIdx.x];
    a.sum[static_cast<int64_t>(lh) * kHeadDim + threadIdx.x] = sum;
  }
}

size_t partial_bytes(int64_t L, int64_t H, int64_t T) {
  return (static_cast<size_t>(L * H) * ceil_div(T, kSumTokens) * kHeadDim * sizeof(float) + 255) / 256 * 256;
}

}  // namespace
}  // namespace kvp

extern "C" size_t kvp_score_keys_workspace_bytes(int64_t L, int64_t H, int64_t T, int32_t method) {
  if (L <= 0 || H <= 0 || T <= 0 || method != KVP_SCORE_KEYDIFF) return 0;
  return kvp::partial_bytes(L, H, T) + static_cast<size_t>(L * H) * kvp::kHeadDim * sizeof(float);
}

extern "C" int32_t kvp_score_keys(const kvp_view* k, int32_t method, float* scores, void* ws, size_t ws_bytes,
                                  void* stream) {
  using namespace kvp;
  int32_t rc = check_view(k);
  if (rc != KVP_OK) return rc;
  if (!scores) return KVP_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(scores) & 3u) return KVP_ERR_ALIGN;
  if (method != KVP_SCORE_KNORM && method != KVP_SCORE_KEYDIFF) return KVP_ERR_UNSUPPORTED;
  if (k->T >= (1ll << 30) || k->L * k->H > 65535) return KVP_ERR_SHAPE;
  KeyArgs a{};
  a.k = static_cast<const uint16_t*>(k->ptr);
  a.k_sl = k->stride_l; a.k_st = k->stride_t; a.k_sh = k->stride_h;
  a.T = static_cast<int32_t>(k->T); a.H = static_cast<int32_t>(k->H);
  a.scores = scores;
  const hipStream_t st = as_stream(stream);
  const unsigned lh = static_cast<unsigned>(k->L * k->H);
  const dim3 grid(static_cast<unsigned>(ceil_div(k->T, kTokensPerBlock)), lh);
  if (method == KVP_SCORE_KNORM) {
    key_score_kernel<false><<<grid, kThreads, 0, st>>>(a);
    return launch_status();
  }
  const size_t need = kvp_score_keys_workspace_bytes(k->L, k->H, k->T, method);
  if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15u)) return KVP_ERR_WORKSPACE;
  a.n_chunks = static_cast<int32_t>(ceil_div(k->T, kSumTokens));
  a.partial = static_cast<float*>(ws);
  a.sum = reinterpret_cast<float*>(static_cast<char*>(ws) + partial_bytes(k->L, k->H, k->T));
  unit_key_sum_kernel<<<dim3(static_cast<unsigned>(a.n_chunks), lh), kThreads, 0, st>>>(a);
  chunk_sum_kernel<<<dim3(lh), 128, 0, st>>>(a);
  key_score_kernel<true><<<grid, kThreads, 0, st>>>(a);
  return launch_status();
}
