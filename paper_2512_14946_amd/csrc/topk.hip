// kvp_select_topk: per-row top-k keep-set by radix select (the paper's token dropping keeps the
// tokens with the highest attention scores: Evaluation, Baselines, snapkv / IMPRESS "top X%").
//
// One block owns one row.  Scores are mapped to order-preserving unsigned keys; four
// most-significant-digit-first passes over 8-bit digits find the key tau of the k-th largest score
// and how many elements equal to tau belong to the keep-set.  Histograms live in LDS, replicated
// 32 times and interleaved so that the 32 lanes of a half-wave always hit 32 different banks (token
// scores crowd into a few exponent bins, which would serialize a single histogram).  A final pass
// writes the kept indices in ascending order with a block-wide prefix sum: position = (number of
// earlier elements above tau) + min(number of earlier elements equal to tau, quota), so ties at
// the threshold go to the lowest indices.  Integer compares only: the result is exact.
//
// Rows of up to 16384 scores are read from HBM exactly once and stay in registers through all
// passes: 16 keys per thread in a 1024-thread block, or 32 keys per thread in a 512-thread block
// when there are more rows than the chip holds wide blocks (the work is bound by vector-ALU
// instruction issue, about 60 per key, so what counts then is rows in flight per CU).  Longer rows
// are processed in 16384-element spans that are re-read (from L2 after the first pass) with the
// loads of the next two spans in flight while the current span is consumed.  Every wave redoes the 256-bin
// digit search and the scan of the wave totals itself, so a pass costs two block barriers.

#include "kvp_internal.h"

namespace kvp {
namespace {

constexpr int kCopies = 32;
constexpr int kBins = 256;
constexpr int kSpan = 16384;                        // elements a block holds in registers at a time

// Block shapes: THREADS threads hold a span as ITEMS float4 items each.
template <int THREADS>
struct Shape {
  static constexpr int kWaves = THREADS / kWave;
  static constexpr int kChunk = THREADS * 4;        // elements covered by one item of all threads
  static constexpr int kItems = kSpan / kChunk;     // 4 (1024 threads) or 8 (512 threads)
};

// IEEE order -> unsigned order; -0.0 is folded onto +0.0 so that they tie, as with operator>.
// Key 0 would be a negative NaN (out of contract): it marks slots beyond the end of the row and
// sorts below every real score.
__device__ __forceinline__ uint32_t to_key(float f) {
  uint32_t u = __float_as_uint(f);
  u = (u == 0x80000000u) ? 0u : u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int ITEMS>
struct Span {
  uint32_t key[ITEMS][4];
};

// Element index of (item c, thread tid, lane element e) inside a span: c * kChunk + tid * 4 + e.
template <int THREADS>
__device__ __forceinline__ void load_span(const float* row, int64_t base, int64_t T, bool vec,
                                          Span<Shape<THREADS>::kItems>& s) {
#pragma unroll
  for (int c = 0; c < Shape<THREADS>::kItems; ++c) {
    const int64_t i = base + c * Shape<THREADS>::kChunk + static_cast<int64_t>(threadIdx.x) * 4;
    // raw bit patterns only: nothing here waits for the loads (slots beyond the row get a negative NaN, key 0)
    if (vec && i + 4 <= T) {
      const uint4 v = *reinterpret_cast<const uint4*>(row + i);
      s.key[c][0] = v.x; s.key[c][1] = v.y; s.key[c][2] = v.z; s.key[c][3] = v.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) s.key[c][e] = (i + e < T) ? __float_as_uint(row[i + e]) : 0xffffffffu;
    }
  }
}

// raw bit patterns -> keys, once the span is about to be consumed
template <int ITEMS>
__device__ __forceinline__ Span<ITEMS> to_keys(const Span<ITEMS>& raw) {
  Span<ITEMS> s;
#pragma unroll
  for (int c = 0; c < ITEMS; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) s.key[c][e] = to_key(__uint_as_float(raw.key[c][e]));
  return s;
}

template <int ITEMS>
__device__ __forceinline__ void histogram_span(const Span<ITEMS>& s, uint32_t mask, uint32_t prefix, int shift,
                                               uint32_t* hist) {
  const int copy = threadIdx.x & (kCopies - 1);
#pragma unroll
  for (int c = 0; c < ITEMS; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t key = s.key[c][e];
      // (end-of-row slots, key 0, fall into the lowest bin below every real score: harmless)
      if ((key & mask) == prefix) atomicAdd(&hist[((key >> shift) & 0xffu) * kCopies + copy], 1u);
    }
}

// inclusive scan across the 64 lanes of a wave with DPP row shifts and row broadcasts (no LDS traffic)
template <int CTRL, int ROW_MASK, int BANK_MASK>
__device__ __forceinline__ uint32_t dpp_or_zero(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), CTRL, ROW_MASK, BANK_MASK, false));
}
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
  uint32_t t = v;
  t += dpp_or_zero<0x111, 0xf, 0xf>(v);   // row_shr:1
  t += dpp_or_zero<0x112, 0xf, 0xf>(v);   // row_shr:2
  t += dpp_or_zero<0x113, 0xf, 0xf>(v);   // row_shr:3
  t += dpp_or_zero<0x114, 0xf, 0xe>(t);   // row_shr:4 into lanes 4..15 of each row
  t += dpp_or_zero<0x118, 0xf, 0xc>(t);   // row_shr:8 into lanes 8..15 of each row
  t += dpp_or_zero<0x142, 0xa, 0xf>(t);   // row_bcast:15 into rows 1 and 3
  t += dpp_or_zero<0x143, 0xc, 0xf>(t);   // row_bcast:31 into rows 2 and 3
  return t;
}

// RESIDENT: T <= kSpan, the whole row lives in registers (8 waves per SIMD: two 1024-thread or four
// 512-thread blocks per CU).
template <int THREADS, bool RESIDENT>
__global__ __launch_bounds__(THREADS, RESIDENT ? 8 : 4) void select_topk_kernel(const float* __restrict__ scores,
                                                                                int64_t T, int64_t row_stride,
                                                                                int64_t k,
                                                                                int32_t* __restrict__ idx_out) {
  constexpr int kThreads = THREADS;
  constexpr int kWaves = Shape<THREADS>::kWaves, kItems = Shape<THREADS>::kItems, kChunk = Shape<THREADS>::kChunk;
  static_assert(THREADS >= kBins, "one thread per digit in the histogram reduction");
  __shared__ uint32_t hist[kBins * kCopies];
  __shared__ uint32_t cnt[kBins];
  __shared__ uint32_t wave_tot[4][kWaves];

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // uniform: usable as a lane selector
  const float* row = scores + static_cast<int64_t>(blockIdx.x) * row_stride;
  int32_t* out = idx_out + static_cast<int64_t>(blockIdx.x) * k;
  const bool vec = ((reinterpret_cast<uintptr_t>(row) & 15u) == 0);
  constexpr bool resident = RESIDENT;

  // Streaming rows keep two spans in flight behind the one being consumed; the spans are visited cyclically
  // (0 .. n-1, then 0 again for the next pass), so the prefetch stream never stops between passes.
  const int64_t n_spans = (T + kSpan - 1) / kSpan;
  int64_t fetch = 0;   // index of the next span to request
  auto next_base = [&]() {
    const int64_t b = fetch * kSpan;
    fetch = fetch + 1 < n_spans ? fetch + 1 : 0;
    return b;
  };
  Span<kItems> cur, ahead;   // cur holds keys, ahead (and far below) raw bits still in flight
  load_span<THREADS>(row, next_base(), T, vec, cur);
  if (!resident) load_span<THREADS>(row, next_base(), T, vec, ahead);
  cur = to_keys(cur);
  for (int i = tid; i < kBins * kCopies; i += kThreads) hist[i] = 0;
  __syncthreads();

  uint32_t prefix = 0, mask = 0, krem = static_cast<uint32_t>(k);
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (resident) {
      histogram_span(cur, mask, prefix, shift, hist);
    } else {
      for (int64_t base = 0; base < T; base += kSpan) {
        Span<kItems> far;
        load_span<THREADS>(row, next_base(), T, vec, far);
        histogram_span(cur, mask, prefix, shift, hist);
        cur = to_keys(ahead);
        ahead = far;
      }
    }
    __syncthreads();
    if (tid < kBins) {
      uint32_t sum = 0;
#pragma unroll 8
      for (int c = 0; c < kCopies; ++c) {
        const int slot = (tid * kCopies + (tid & (kCopies - 1))) ^ c;   // copy (tid ^ c) mod 32: a different bank per lane
        sum += hist[slot];
        hist[slot] = 0;   // ready for the next pass
      }
      cnt[tid] = sum;
    }
    __syncthreads();
    {
      // every wave: lane j owns digits 255-4j .. 252-4j (descending); find the digit of the krem-th largest
      uint32_t c4[4], local = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        c4[e] = cnt[255 - 4 * lane - e];
        local += c4[e];
      }
      const uint32_t incl = wave_inclusive_scan(local);
      uint32_t above = incl - local;  // elements in digits larger than this lane's
      const bool mine = above < krem && krem <= incl;
      uint32_t new_prefix = 0, new_krem = 0;
      if (mine) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (above < krem && krem <= above + c4[e]) {
            new_prefix = prefix | (static_cast<uint32_t>(255 - 4 * lane - e) << shift);
            new_krem = krem - above;
          }
          above += c4[e];
        }
      }
      const int src = __ffsll(static_cast<long long>(__builtin_amdgcn_ballot_w64(mine))) - 1;  // exactly one lane
      prefix = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(new_prefix), src));
      krem = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(new_krem), src));
    }
    mask |= 0xffu << shift;
  }

  // prefix is now the key of the k-th largest score, krem the quota of elements equal to it.
  const uint32_t tau = prefix;
  uint32_t gt_base = 0, eq_base = 0;
  for (int64_t base = 0; base < T; base += kSpan) {
    Span<kItems> far;
    if (!resident) load_span<THREADS>(row, next_base(), T, vec, far);
    // per item: (#greater, #equal) of this thread's 4 elements, packed 16 + 16 bits (a span holds
    // at most 16384 elements), scanned across the block in element order, four items per round
#pragma unroll
    for (int c0 = 0; c0 < kItems; c0 += 4) {
      if (c0 > 0) __syncthreads();   // wave_tot is rewritten
      uint32_t excl[4];              // (greater, equal) of the earlier lanes of this wave, per item
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t g = 0, q = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          g += cur.key[c0 + j][e] > tau ? 1u : 0u;
          q += cur.key[c0 + j][e] == tau ? 1u : 0u;
        }
        const uint32_t mine = g | (q << 16);
        const uint32_t incl = wave_inclusive_scan(mine);
        if (lane == kWave - 1) wave_tot[j][wave] = incl;
        excl[j] = incl - mine;
      }
      __syncthreads();
      // the 4 x kWaves wave totals are in element order: every wave scans them, one per lane
      static_assert(4 * kWaves <= kWave, "one wave total per lane");
      const uint32_t tot_mine = lane < 4 * kWaves ? (&wave_tot[0][0])[lane] : 0u;
      const uint32_t tot_incl = wave_inclusive_scan(tot_mine);
      const uint32_t tot_excl = tot_incl - tot_mine;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // everything before this wave's part of the item, then this thread's place inside it
        const uint32_t before =
            static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(tot_excl), j * kWaves + wave)) + excl[j];
        uint32_t gt_before = gt_base + (before & 0xffffu), eq_before = eq_base + (before >> 16);
        const int32_t i0 = static_cast<int32_t>(base) + (c0 + j) * kChunk + tid * 4;   // T < 2^31
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t key = cur.key[c0 + j][e];
          if (key > tau) {
            out[gt_before + min(eq_before, krem)] = i0 + e;
            ++gt_before;
          } else if (key == tau) {
            if (eq_before < krem) out[gt_before + eq_before] = i0 + e;
            ++eq_before;
          }
        }
      }
      const uint32_t round_tot = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(tot_incl), kWave - 1));
      gt_base += round_tot & 0xffffu;
      eq_base += round_tot >> 16;
    }
    if (!resident) {
      cur = to_keys(ahead);
      ahead = far;
      __syncthreads();   // wave_tot is rewritten by the next span
    }
  }
}

}  // namespace

void select_topk_launch(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                        int32_t* idx_out, hipStream_t st) {
  const dim3 grid(static_cast<unsigned>(n_rows));
  if (T > kSpan) {
    select_topk_kernel<1024, false><<<grid, 1024, 0, st>>>(scores, T, row_stride, k, idx_out);
    return;
  }
  // A CU holds two 1024-thread blocks or four 512-thread ones.  Up to 512 rows every row gets a slot either way
  // and the wider block finishes a row sooner; beyond that the narrower shape keeps twice the rows in flight.
  if (n_rows <= 2 * 256)
    select_topk_kernel<1024, true><<<grid, 1024, 0, st>>>(scores, T, row_stride, k, idx_out);
  else
    select_topk_kernel<512, true><<<grid, 512, 0, st>>>(scores, T, row_stride, k, idx_out);
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
