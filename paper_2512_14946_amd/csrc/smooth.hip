// kvp_smooth_scores: 1-D average / maximum pooling of the prefix scores along the token axis, the
// smoothing step of the published snapkv method (the paper's Evaluation, Baselines) that runs
// between kvp_score_tokens and kvp_select_topk.
//
// One 256-thread block per (tile of 2048 tokens, row): the tile and its halo of kernel/2 taps on each
// side are staged in LDS once (out-of-prefix taps as the pooling's neutral element), then each thread
// produces 8 outputs, lanes on adjacent tokens so that LDS reads are conflict-free and stores coalesce.
// Traffic is one read and one write of the score rows (a few tens of MB): the kernel is short.

#include "kvp_common.h"

namespace kvp {
namespace {

constexpr int kThreads = 256;
constexpr int kTile = 2048;
constexpr int kMaxKernel = 63;

template <bool MAXPOOL>
__global__ __launch_bounds__(kThreads) void smooth_kernel(const float* __restrict__ scores, int64_t row_stride, uint32_t T,
                                                          uint32_t P, int r, float* __restrict__ out, int64_t out_stride) {
  __shared__ float tile[kTile + kMaxKernel - 1];
  const float* in = scores + static_cast<int64_t>(blockIdx.x) * row_stride;   // x: row (up to 2^31 - 1), y: tile
  float* o = out + static_cast<int64_t>(blockIdx.x) * out_stride;
  const uint32_t t0 = blockIdx.y * kTile;
  const float neutral = MAXPOOL ? -INFINITY : 0.0f;
  const int span = kTile + 2 * r;
  for (int i = threadIdx.x; i < span; i += kThreads) {
    const int64_t u = static_cast<int64_t>(t0) - r + i;
    tile[i] = (u >= 0 && u < static_cast<int64_t>(P)) ? in[u] : neutral;
  }
  __syncthreads();
  const int taps = 2 * r + 1;
  const float divisor = static_cast<float>(taps);
  for (int j = threadIdx.x; j < kTile; j += kThreads) {
    const uint32_t t = t0 + j;
    if (t >= T) break;
    float v;
    if (t < P) {
      v = tile[j];                      // tap t - r
      for (int d = 1; d < taps; ++d) v = MAXPOOL ? fmaxf(v, tile[j + d]) : v + tile[j + d];
      if (!MAXPOOL) v = v / divisor;
    } else {
      v = in[t];                        // observation window: copied through
    }
    o[t] = v;
  }
}

}  // namespace
}  // namespace kvp

extern "C" int32_t kvp_smooth_scores(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t window,
                                     int32_t kernel, int32_t mode, float* out, int64_t out_stride, void* stream) {
  using namespace kvp;
  if (!scores || !out) return KVP_ERR_NULL;
  if (n_rows < 0 || T <= 0 || T >= (1ll << 31) || row_stride < T || out_stride < T || window < 0 || window > T)
    return KVP_ERR_SHAPE;
  if (n_rows >= (1ll << 31) || ceil_div(T, kTile) > 65535) return KVP_ERR_SHAPE;
  if (kernel < 1 || kernel > kMaxKernel || kernel % 2 == 0) return KVP_ERR_UNSUPPORTED;
  if (mode != KVP_SMOOTH_AVG && mode != KVP_SMOOTH_MAX) return KVP_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(scores) & 3u) || (reinterpret_cast<uintptr_t>(out) & 3u)) return KVP_ERR_ALIGN;
  if (n_rows == 0) return KVP_OK;
  {  // the two row sets must not overlap (a block reads its halo after neighbours may have written)
    const char* a0 = reinterpret_cast<const char*>(scores);
    const char* a1 = a0 + ((n_rows - 1) * row_stride + T) * 4;
    const char* b0 = reinterpret_cast<const char*>(out);
    const char* b1 = b0 + ((n_rows - 1) * out_stride + T) * 4;
    if (a0 < b1 && b0 < a1) return KVP_ERR_SHAPE;
  }
  const dim3 grid(static_cast<unsigned>(n_rows), static_cast<unsigned>(ceil_div(T, kTile)));
  const hipStream_t st = as_stream(stream);
  const uint32_t P = static_cast<uint32_t>(T - window);
  if (mode == KVP_SMOOTH_MAX)
    smooth_kernel<true><<<grid, kThreads, 0, st>>>(scores, row_stride, static_cast<uint32_t>(T), P, kernel / 2, out, out_stride);
  else
    smooth_kernel<false><<<grid, kThreads, 0, st>>>(scores, row_stride, static_cast<uint32_t>(T), P, kernel / 2, out, out_stride);
  return launch_status();
}
