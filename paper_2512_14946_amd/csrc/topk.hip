// kvp_select_topk: per-row top-k keep-set by radix select (the paper's token dropping keeps the
// tokens with the highest attention scores: Evaluation, Baselines, snapkv / IMPRESS "top X%").
//
// One 1024-thread block owns one row.  Scores are mapped to order-preserving unsigned keys; four
// most-significant-digit-first passes over 8-bit digits find the key tau of the k-th largest score
// and how many elements equal to tau belong to the keep-set.  Histograms live in LDS, replicated
// 32 times and interleaved so that the 32 lanes of a half-wave always hit 32 different banks (token
// scores crowd into a few exponent bins, which would serialize a single histogram).  A final pass
// writes the kept indices in ascending order with a block-wide prefix sum: position = (number of
// earlier elements above tau) + min(number of earlier elements equal to tau, quota), so ties at
// the threshold go to the lowest indices.  Integer compares only: the result is exact.
//
// The row is re-read from global memory in every pass; after the first pass it is served by L2
// (a row is at most 512 KiB at T = 131072).

#include "kvp_internal.h"

namespace kvp {
namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / kWave;
constexpr int kCopies = 32;
constexpr int kBins = 256;
constexpr int kPerThread = 4;                       // consecutive elements per thread per chunk
constexpr int kChunk = kThreads * kPerThread;       // 4096 elements

// IEEE order -> unsigned order; -0.0 is folded onto +0.0 so that they tie, as with operator>.
__device__ __forceinline__ uint32_t to_key(float f) {
  uint32_t u = __float_as_uint(f);
  u = (u == 0x80000000u) ? 0u : u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ void load4(const float* row, int64_t i, int64_t T, bool vec, uint32_t key[kPerThread],
                                      bool valid[kPerThread]) {
  if (vec && i + kPerThread <= T) {
    const float4 v = *reinterpret_cast<const float4*>(row + i);
    key[0] = to_key(v.x); key[1] = to_key(v.y); key[2] = to_key(v.z); key[3] = to_key(v.w);
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) valid[e] = true;
  } else {
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      valid[e] = i + e < T;
      key[e] = valid[e] ? to_key(row[i + e]) : 0u;
    }
  }
}

// inclusive scan across the 64 lanes of a wave
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const uint32_t n = __shfl_up(v, off, kWave);
    if (lane >= off) v += n;
  }
  return v;
}

__global__ __launch_bounds__(kThreads) void select_topk_kernel(const float* __restrict__ scores, int64_t T,
                                                               int64_t row_stride, int64_t k,
                                                               int32_t* __restrict__ idx_out) {
  __shared__ uint32_t hist[kBins * kCopies];
  __shared__ uint32_t cnt[kBins];
  __shared__ uint32_t s_prefix, s_krem;
  __shared__ uint32_t wave_gt[kWaves], wave_eq[kWaves];

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  const float* row = scores + static_cast<int64_t>(blockIdx.x) * row_stride;
  int32_t* out = idx_out + static_cast<int64_t>(blockIdx.x) * k;
  const bool vec = ((reinterpret_cast<uintptr_t>(row) & 15u) == 0);

  uint32_t prefix = 0, mask = 0, krem = static_cast<uint32_t>(k);

  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int i = tid; i < kBins * kCopies; i += kThreads) hist[i] = 0;
    __syncthreads();
    for (int64_t base = 0; base < T; base += kChunk) {
      uint32_t key[kPerThread];
      bool valid[kPerThread];
      load4(row, base + static_cast<int64_t>(tid) * kPerThread, T, vec, key, valid);
#pragma unroll
      for (int e = 0; e < kPerThread; ++e)
        if (valid[e] && (key[e] & mask) == prefix)
          atomicAdd(&hist[((key[e] >> shift) & 0xffu) * kCopies + (lane & (kCopies - 1))], 1u);
    }
    __syncthreads();
    if (tid < kBins) {
      uint32_t sum = 0;
#pragma unroll
      for (int c = 0; c < kCopies; ++c) sum += hist[tid * kCopies + ((c + tid) & (kCopies - 1))];
      cnt[tid] = sum;
    }
    __syncthreads();
    if (wave == 0) {
      // lane j owns digits 255-4j .. 252-4j (descending); find the digit holding the krem-th largest
      uint32_t c4[4], local = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        c4[e] = cnt[255 - 4 * lane - e];
        local += c4[e];
      }
      const uint32_t incl = wave_inclusive_scan(local);
      uint32_t above = incl - local;  // elements in digits larger than this lane's
      if (above < krem && krem <= incl) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (above < krem && krem <= above + c4[e]) {
            s_prefix = prefix | (static_cast<uint32_t>(255 - 4 * lane - e) << shift);
            s_krem = krem - above;
          }
          above += c4[e];
        }
      }
    }
    __syncthreads();
    prefix = s_prefix;
    krem = s_krem;
    mask |= 0xffu << shift;
    __syncthreads();
  }

  // prefix is now the key of the k-th largest score, krem the quota of elements equal to it.
  const uint32_t tau = prefix;
  uint32_t gt_base = 0, eq_base = 0;
  for (int64_t base = 0; base < T; base += kChunk) {
    uint32_t key[kPerThread];
    bool valid[kPerThread];
    const int64_t i0 = base + static_cast<int64_t>(tid) * kPerThread;
    load4(row, i0, T, vec, key, valid);
    uint32_t gt = 0, eq = 0;
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      gt += (valid[e] && key[e] > tau) ? 1u : 0u;
      eq += (valid[e] && key[e] == tau) ? 1u : 0u;
    }
    const uint32_t gt_incl = wave_inclusive_scan(gt);
    const uint32_t eq_incl = wave_inclusive_scan(eq);
    if (lane == kWave - 1) {
      wave_gt[wave] = gt_incl;
      wave_eq[wave] = eq_incl;
    }
    __syncthreads();
    uint32_t gt_before = gt_base + gt_incl - gt, eq_before = eq_base + eq_incl - eq;
    uint32_t gt_total = 0, eq_total = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t g = wave_gt[w], q = wave_eq[w];
      if (w < wave) {
        gt_before += g;
        eq_before += q;
      }
      gt_total += g;
      eq_total += q;
    }
#pragma unroll
    for (int e = 0; e < kPerThread; ++e) {
      if (!valid[e]) continue;
      if (key[e] > tau) {
        out[gt_before + min(eq_before, krem)] = static_cast<int32_t>(i0 + e);
        ++gt_before;
      } else if (key[e] == tau) {
        if (eq_before < krem) out[gt_before + eq_before] = static_cast<int32_t>(i0 + e);
        ++eq_before;
      }
    }
    gt_base += gt_total;
    eq_base += eq_total;
    __syncthreads();
  }
}

}  // namespace

void select_topk_launch(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                        int32_t* idx_out, hipStream_t st) {
  select_topk_kernel<<<dim3(static_cast<unsigned>(n_rows)), kThreads, 0, st>>>(scores, T, row_stride, k, idx_out);
}

}  // namespace kvp

extern "C" size_t kvp_select_workspace_bytes(int64_t, int64_t, int64_t) { return 0; }

extern "C" int32_t kvp_select_topk(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                                   int32_t* idx_out, void* ws, size_t ws_bytes, void* stream) {
  using namespace kvp;
  (void)ws;
  (void)ws_bytes;
  if (!scores || (!idx_out && k > 0)) return KVP_ERR_NULL;
  if (n_rows < 0 || T <= 0 || T >= (1ll << 31) || k < 0 || k > T || row_stride < T || n_rows >= (1ll << 31))
    return KVP_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(scores) & 3u) || (reinterpret_cast<uintptr_t>(idx_out) & 3u)) return KVP_ERR_ALIGN;
  if (n_rows == 0 || k == 0) return KVP_OK;
  select_topk_launch(scores, n_rows, T, row_stride, k, idx_out, as_stream(stream));
  return launch_status();
}
