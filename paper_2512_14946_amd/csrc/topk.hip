// kvp_select_topk: per-row top-k keep-set by radix select (the paper's token dropping keeps the
// tokens with the highest attention scores: Evaluation, Baselines, snapkv / IMPRESS top X %).
//
// Scores are mapped to order-preserving unsigned keys (-0 folded onto +0).  A block finds the key
// tau of the k-th largest score and the quota of elements equal to tau that belong to the keep-set
// by interval refinement, 2048 bins per pass: three most-significant-digit-first passes over 11 + 11 +
// 10 bits when it starts from the whole key range (LDS histograms, four interleaved copies), then writes the kept indices in ascending order: position = (number of
// earlier elements above tau) + min(number of earlier elements equal to tau, quota), so ties at the
// threshold go to the lowest indices.  Integer compares only: the result is exact.  Ranks inside a
// wave come from ballots (v_cmp into a scalar mask, v_mbcnt), ranks across waves from one scan of
// the packed (greater, equal) wave totals.  After the second digit the chosen bin almost always
// holds exactly the elements still wanted, and the third pass is skipped.
//
// Three launch shapes:
//   * rows of up to 16384 scores: one block per row, the row is read once and stays in registers
//     (16 keys per thread in a 1024-thread block, 32 in a 512-thread block when there are more rows
//     than the chip holds wide blocks);
//   * longer rows (up to 2^18 scores) are split into 16384-element spans, one block per span, in
//     three launches, so that the whole chip works on a few long rows:
//       pivots     one block per row histograms an evenly spread sample of the row in fine bins
//                  below the sample's maximum and derives two keys p_lo <= p_hi that bracket tau
//                  with overwhelming probability;
//       partition  every span counts its keys above p_hi and writes the few keys inside
//                  [p_lo, p_hi] (the candidates) to its slice of the row's list;
//       finish     every span block selects tau among the row's candidates (rank k minus the keys
//                  above p_hi), derives its own output offset from the counts of the earlier
//                  spans and writes its kept indices.
//     If the bracket misses (the k-th largest is not among the candidates) or a slice overflows
//     (heavy ties at the threshold), the first span's block redoes the row on its own:
//   * whole-row selection by one block (the same three passes, the spans re-read for every pass);
//     it also serves rows beyond 2^18 scores.
// The output never depends on the order in which blocks run or candidates are appended.

#include <algorithm>

#include "kvp_internal.h"

namespace kvp {
namespace {

constexpr int kSpan = 16384;          // elements a block holds in registers at a time
constexpr int kBins = 2048;           // bins of the widest digit
constexpr int kCopies = 4;            // interleaved histogram copies (lane & 3)
constexpr int kRowCap = 16384;        // candidates per row (what a 1024-thread block holds in registers)
constexpr int kLaneCap = 8;           // candidates one thread can stage per span
constexpr int kFineShift = 18;        // sample histogram: 32 bins per octave, 64 octaves below the maximum
constexpr int64_t kMaxSplitT = 1 << 18;

// Block shapes: THREADS threads hold a span as ITEMS float4 items each.
template <int THREADS>
struct Shape {
  static constexpr int kWaves = THREADS / kWave;
  static constexpr int kChunk = THREADS * 4;        // elements covered by one item of all threads
  static constexpr int kItems = kSpan / kChunk;     // 4 (1024 threads) or 8 (512 threads)
};

// IEEE order -> unsigned order.  x + 0 turns -0 into +0 under round-to-nearest and leaves every other
// value unchanged (denormals are not flushed in this library), so that the two zeros tie, as with
// operator>.  Key 0 would be a negative NaN (out of contract): it marks slots beyond the end of the
// row and sorts below every real score.
__device__ __forceinline__ uint32_t to_key(uint32_t raw) {
  const uint32_t u = __float_as_uint(__uint_as_float(raw) + 0.0f);
  return u ^ (static_cast<uint32_t>(static_cast<int32_t>(u) >> 31) | 0x80000000u);
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
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(wave_inclusive_scan(v)), kWave - 1));
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
  for (int d = 1; d < kWave; d *= 2) v = max(v, static_cast<uint32_t>(__shfl_xor(static_cast<int>(v), d, kWave)));
  return v;
}
// number of set bits of a wave mask below this lane, added to acc
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask, uint32_t acc) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), acc));
}
// out[p] = v with the byte offset formed in 32 bits (rows of this file's kernels hold fewer than 2^30
// indices), so that the store takes the scalar base + 32-bit vector offset form
__device__ __forceinline__ void store_index(int32_t* out, uint32_t p, int32_t v) {
  *reinterpret_cast<int32_t*>(reinterpret_cast<char*>(out) + static_cast<size_t>(p << 2)) = v;
}

struct alignas(16) SelectShared {
  uint32_t hist[kBins * kCopies];     // [bin][copy], 32 KiB
  uint32_t wave_tot[64];
  uint32_t result[4];                 // chosen digit, remaining rank, population of the chosen bin, second digit
  uint32_t reduce[8];
};

// Keys of one span in registers: element (item c, thread tid, e) is span element c * kChunk + tid * 4 + e.
template <int THREADS>
__device__ __forceinline__ void load_keys(const float* row, int64_t base, int64_t T, bool vec,
                                          uint32_t (&key)[Shape<THREADS>::kItems][4]) {
  constexpr int kItems = Shape<THREADS>::kItems, kChunk = Shape<THREADS>::kChunk;
  if (vec && base + kSpan <= T) {   // the common case: a whole span, 16-byte loads, no guards
    uint4 raw[kItems];
#pragma unroll
    for (int c = 0; c < kItems; ++c)
      raw[c] = *reinterpret_cast<const uint4*>(row + base + c * kChunk + static_cast<int64_t>(threadIdx.x) * 4);
#pragma unroll
    for (int c = 0; c < kItems; ++c) {
      key[c][0] = to_key(raw[c].x); key[c][1] = to_key(raw[c].y);
      key[c][2] = to_key(raw[c].z); key[c][3] = to_key(raw[c].w);
    }
  } else {
#pragma unroll
    for (int c = 0; c < kItems; ++c) {
      const int64_t i = base + c * kChunk + static_cast<int64_t>(threadIdx.x) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) key[c][e] = (i + e < T) ? to_key(__float_as_uint(row[i + e])) : 0u;
    }
  }
}

template <int THREADS>
__device__ __forceinline__ void clear_histogram(SelectShared& sh) {
  for (int i = threadIdx.x; i < kBins * kCopies / 4; i += THREADS)
    reinterpret_cast<uint4*>(sh.hist)[i] = make_uint4(0, 0, 0, 0);
}

// After a histogram pass (and a barrier): the bin that holds the krem-th largest key, counted from the
// top bin down; krem becomes the rank inside that bin, cnt its population.  With TWO, the same for a
// second rank krem2 >= krem (bin into digit2; krem2 and its population are not returned).  Every thread
// owns kBins / THREADS neighbouring bins (threads in descending bin order), clears them, and the wave
// totals meet in LDS.  Needs 1 <= krem (<= krem2) <= population of the histogram.  Ends with a barrier.
template <int THREADS, bool TWO>
__device__ __forceinline__ void find_digit(SelectShared& sh, uint32_t& krem, uint32_t& digit, uint32_t& cnt,
                                           uint32_t krem2, uint32_t& digit2) {
  constexpr int kWaves = Shape<THREADS>::kWaves;
  constexpr int BPT = kBins / THREADS;              // bins per thread: 2 or 4
  static_assert(kCopies == 4, "one uint4 per bin");
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const int lo_bin = kBins - (static_cast<int>(threadIdx.x) + 1) * BPT;
  uint4* mine = reinterpret_cast<uint4*>(&sh.hist[lo_bin * kCopies]);
  uint32_t c[BPT], local = 0;
#pragma unroll
  for (int j = 0; j < BPT; ++j) {
    const uint4 v = mine[j];
    mine[j] = make_uint4(0, 0, 0, 0);               // ready for the next pass
    c[j] = v.x + v.y + v.z + v.w;                   // bin lo_bin + j
    local += c[j];
  }
  const uint32_t incl = wave_inclusive_scan(local);
  if (lane == kWave - 1) sh.wave_tot[wave] = incl;
  __syncthreads();
  // totals of the earlier waves: one LDS read per lane, one scan, one lane read
  const uint32_t tot_mine = lane < kWaves ? sh.wave_tot[lane] : 0u;
  const uint32_t tot_incl = wave_inclusive_scan(tot_mine);
  uint32_t above = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(tot_incl - tot_mine), wave)) +
                   incl - local;                    // keys in bins above this thread's
  const bool first = above < krem && krem <= above + local;            // exactly one thread of the block
  const bool second = TWO && above < krem2 && krem2 <= above + local;   // likewise
  if (first || second) {
#pragma unroll
    for (int j = BPT - 1; j >= 0; --j) {
      if (first && above < krem && krem <= above + c[j]) {
        sh.result[0] = static_cast<uint32_t>(lo_bin + j);
        sh.result[1] = krem - above;
        sh.result[2] = c[j];
      }
      if (second && above < krem2 && krem2 <= above + c[j]) sh.result[3] = static_cast<uint32_t>(lo_bin + j);
      above += c[j];
    }
  }
  __syncthreads();
  digit = sh.result[0];
  krem = sh.result[1];
  cnt = sh.result[2];
  if (TWO) digit2 = sh.result[3];
}

// Block-wide selection by interval refinement.  visit(f) calls f(key) for every key this thread owns;
// first_visit does the same for the first pass (it may also produce the keys: convert them as their loads
// arrive).  Among the visited keys inside [lo, lo + width] (all others are ignored) it finds tau and quota
// such that the k largest of them are the keys above tau plus `quota` of the keys equal to tau.  Every
// pass counts the keys of the current interval in 2048 equal bins, picks the bin that holds the wanted
// rank and continues inside it: with lo = 0 and width = 2^32 - 1 these are three most-significant-
// digit-first passes over 11 + 11 + 10 bits.  1 <= k <= number of visited keys inside the interval.  The
// histogram must be clear on entry (and a barrier passed); it is clear again on return.
// FULL: the interval is all of [0, 2^32 - 1] (lo and width are ignored; the first pass needs no range test).
template <int THREADS, bool FULL, class FirstVisit, class Visit>
__device__ __forceinline__ void interval_select(FirstVisit&& first_visit, Visit&& visit, uint32_t k, uint32_t lo,
                                                uint32_t width, SelectShared& sh, uint32_t& tau, uint32_t& quota) {
  const uint32_t copy = threadIdx.x & (kCopies - 1);
  uint32_t krem = k, unused = 0;
  if (FULL) {
    lo = 0;
    width = 0xffffffffu;
  }
  // bins of 2^shift keys: the smallest shift for which the interval fits 2048 bins
  auto shift_for = [](uint32_t w) {
    const int bits = 32 - __builtin_clz(w | 1u);               // w < 2^bits
    return bits > 11 ? bits - 11 : 0;
  };
  int shift = shift_for(width);
  // after the counting of a pass: pick the bin, narrow the interval; true when tau is known
  auto settle = [&]() {
    __syncthreads();
    uint32_t bin, cnt;
    find_digit<THREADS, false>(sh, krem, bin, cnt, 0u, unused);
    lo += bin << shift;
    if (shift == 0) {               // bins are single keys
      tau = lo;
      quota = krem;
      return true;
    }
    width = min(width - (bin << shift), (1u << shift) - 1u);
    if (cnt == krem && lo != 0) {
      // every key of the chosen bin belongs to the k largest: keep exactly the keys >= lo
      tau = lo - 1;
      quota = 0;
      return true;
    }
    shift = shift_for(width);
    return false;
  };
  auto count = [&](uint32_t key) {
    const uint32_t d = key - lo;                                // wraps to a large value below lo
    if (d <= width) atomicAdd(&sh.hist[(d >> shift) * kCopies + copy], 1u);
  };
  if (FULL) first_visit([&](uint32_t key) { atomicAdd(&sh.hist[(key >> 21) * kCopies + copy], 1u); });
  else first_visit(count);
  while (!settle()) visit(count);
}

// Ordered compaction of one span held in registers: writes first_index + (span element index) of every
// kept element to out[] in ascending order.  gt_base / eq_base: kept-class counts of the row's elements
// before this span.  Returns the span's own class counts, greater | equal << 16.  Positions are checked
// against k before a store, so that inputs outside the contract (NaN scores) cannot make the kernel
// write outside its row of the output.
template <int THREADS>
__device__ __forceinline__ uint32_t compact_span(const uint32_t (&key)[Shape<THREADS>::kItems][4], uint32_t tau,
                                                 uint32_t quota, uint32_t gt_base, uint32_t eq_base,
                                                 int32_t first_index, uint32_t k, int32_t* __restrict__ out,
                                                 SelectShared& sh, int n_used = Shape<THREADS>::kItems) {
  // items n_used and beyond lie wholly past the end of the row (their keys are 0): nothing to count or emit
  constexpr int kWaves = Shape<THREADS>::kWaves, kItems = Shape<THREADS>::kItems, kChunk = Shape<THREADS>::kChunk;
  static_assert(kItems * kWaves == kWave, "one (item, wave) total per lane of the scanning wave");
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  // phase 1: class totals of this wave's part of every item (scalar popcounts of the compare masks)
  uint32_t eq_items = 0;      // wave-uniform: bit c set if this wave's part of item c holds an element equal to tau
#pragma unroll
  for (int c = 0; c < kItems; ++c) {
    uint32_t tg = 0, te = 0;
    if (c < n_used) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        tg += static_cast<uint32_t>(__builtin_popcountll(__builtin_amdgcn_ballot_w64(key[c][e] > tau)));
        te += static_cast<uint32_t>(__builtin_popcountll(__builtin_amdgcn_ballot_w64(key[c][e] == tau)));
      }
    }
    if (te != 0) eq_items |= 1u << c;
    // a span holds 16384 elements: both totals fit 16 bits, also when summed over the block
    if (lane == 0) sh.wave_tot[c * kWaves + wave] = tg | (te << 16);
  }
  __syncthreads();
  // the (item, wave) totals are in element order: every wave scans them, one per lane
  const uint32_t tot_mine = sh.wave_tot[lane];
  const uint32_t tot_incl = wave_inclusive_scan(tot_mine);
  const uint32_t tot_excl = tot_incl - tot_mine;
  // the compares are redone below rather than kept: sixteen wave masks per class do not fit the scalar registers
  uint32_t tau2 = tau;
  asm volatile("" : "+v"(tau2));
  // phase 2: ranks inside the wave, then the stores
#pragma unroll
  for (int c = 0; c < kItems; ++c) {
    if (c >= n_used) break;
    const uint32_t before = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(tot_excl), c * kWaves + wave));
    const int32_t i0 = first_index + c * kChunk + static_cast<int32_t>(threadIdx.x) * 4;   // T < 2^31
    uint32_t g = 0;             // kept-above elements of the earlier lanes of this wave, this item
#pragma unroll
    for (int e = 0; e < 4; ++e) g = lanes_below(__builtin_amdgcn_ballot_w64(key[c][e] > tau2), g);
    uint32_t gt_before = gt_base + (before & 0xffffu) + g;
    uint32_t eq_before = eq_base + (before >> 16);
    if ((eq_items & (1u << c)) == 0) {
      // no element of this wave's part equals tau: the kept ones are simply those above it
      uint32_t p = gt_before + min(eq_before, quota);
      if (__builtin_amdgcn_ballot_w64(p + 4 > k) == 0) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (key[c][e] > tau2) {
            store_index(out, p, i0 + e);
            ++p;
          }
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (key[c][e] > tau2) {
            if (p < k) store_index(out, p, i0 + e);
            ++p;
          }
        }
      }
    } else {
      uint32_t q = 0;
#pragma unroll
      for (int e = 0; e < 4; ++e) q = lanes_below(__builtin_amdgcn_ballot_w64(key[c][e] == tau2), q);
      eq_before += q;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t kk = key[c][e];
        if (kk > tau2) {
          const uint32_t p = gt_before + min(eq_before, quota);
          if (p < k) store_index(out, p, i0 + e);
          ++gt_before;
        } else if (kk == tau2) {
          if (eq_before < quota && gt_before + eq_before < k) store_index(out, gt_before + eq_before, i0 + e);
          ++eq_before;
        }
      }
    }
  }
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(tot_incl), kWave - 1));
}

// ---------------------------------------------------------------- rows that fit one span

template <int THREADS>
__global__ __launch_bounds__(THREADS, THREADS == 1024 ? 8 : 6) void select_resident_kernel(
    const float* __restrict__ scores, int64_t T, int64_t row_stride, int64_t k, int32_t* __restrict__ idx_out) {
  constexpr int kItems = Shape<THREADS>::kItems, kChunk = Shape<THREADS>::kChunk;
  __shared__ SelectShared sh;
  const float* row = scores + static_cast<int64_t>(blockIdx.x) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  const int n_full = vec ? static_cast<int>(T / kChunk) : 0;               // items read with unguarded 16-byte loads
  const int n_used = static_cast<int>((T + kChunk - 1) / kChunk);           // items that hold any score
  uint32_t key[kItems][4];
  uint4 raw[kItems];
  // the 16-byte loads stay in flight while the histogram is cleared; each item is turned into keys when the
  // first pass reaches it
#pragma unroll
  for (int c = 0; c < kItems; ++c) {
    if (c < n_full) {
      raw[c] = *reinterpret_cast<const uint4*>(row + c * kChunk + static_cast<int64_t>(threadIdx.x) * 4);
    } else {
      const int64_t i = static_cast<int64_t>(c) * kChunk + static_cast<int64_t>(threadIdx.x) * 4;
#pragma unroll
      for (int e = 0; e < 4; ++e) key[c][e] = (i + e < T) ? to_key(__float_as_uint(row[i + e])) : 0u;
    }
  }
  clear_histogram<THREADS>(sh);
  __syncthreads();
  auto visit = [&](auto&& f) {
#pragma unroll
    for (int c = 0; c < kItems; ++c) {
      if (c >= n_used) break;
#pragma unroll
      for (int e = 0; e < 4; ++e) f(key[c][e]);
    }
  };
  auto first_visit = [&](auto&& f) {
#pragma unroll
    for (int c = 0; c < kItems; ++c) {
      if (c >= n_used) break;
      if (c < n_full) {
        key[c][0] = to_key(raw[c].x); key[c][1] = to_key(raw[c].y);
        key[c][2] = to_key(raw[c].z); key[c][3] = to_key(raw[c].w);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) f(key[c][e]);
    }
  };
  uint32_t tau, quota;
  interval_select<THREADS, true>(first_visit, visit, static_cast<uint32_t>(k), 0u, 0xffffffffu, sh, tau, quota);
  compact_span<THREADS>(key, tau, quota, 0, 0, 0, static_cast<uint32_t>(k),
                        idx_out + static_cast<int64_t>(blockIdx.x) * k, sh, n_used);
}

// ---------------------------------------------------------------- one block, whole row of any length

// Three passes over all spans of the row (re-read for every pass), then the spans once more for the
// ordered output.  Block-wide; 1024 threads.  PREFETCH keeps the next span's loads in flight (16 more registers).
template <bool PREFETCH>
__device__ __forceinline__ void select_whole_row(const float* row, int64_t T, bool vec, uint32_t k, int32_t* out,
                                                 SelectShared& sh) {
  constexpr int THREADS = 1024, kItems = Shape<THREADS>::kItems;
  const int64_t n_spans = (T + kSpan - 1) / kSpan;
  clear_histogram<THREADS>(sh);
  __syncthreads();
  const int64_t n_fast = (PREFETCH && vec) ? T / kSpan : 0;   // whole spans, read with 16-byte loads, the next one in flight
  auto load_raw = [&](int64_t s, uint4 (&raw)[kItems]) {
#pragma unroll
    for (int c = 0; c < kItems; ++c)
      raw[c] = *reinterpret_cast<const uint4*>(row + s * kSpan + c * Shape<THREADS>::kChunk +
                                               static_cast<int64_t>(threadIdx.x) * 4);
  };
  auto visit = [&](auto&& f) {
    uint4 cur[kItems], nxt[kItems];
    if (n_fast > 0) load_raw(0, cur);
    for (int64_t s = 0; s < n_fast; ++s) {
      if (s + 1 < n_fast) load_raw(s + 1, nxt);
#pragma unroll
      for (int c = 0; c < kItems; ++c) {
        f(to_key(cur[c].x)); f(to_key(cur[c].y)); f(to_key(cur[c].z)); f(to_key(cur[c].w));
      }
#pragma unroll
      for (int c = 0; c < kItems; ++c) cur[c] = nxt[c];
    }
    for (int64_t s = n_fast; s < n_spans; ++s) {
      uint32_t key[kItems][4];
      load_keys<THREADS>(row, s * kSpan, T, vec, key);
#pragma unroll
      for (int c = 0; c < kItems; ++c)
#pragma unroll
        for (int e = 0; e < 4; ++e) f(key[c][e]);
    }
  };
  uint32_t tau, quota;
  interval_select<THREADS, true>(visit, visit, k, 0u, 0xffffffffu, sh, tau, quota);
  uint32_t gt_base = 0, eq_base = 0;
  for (int64_t s = 0; s < n_spans; ++s) {
    uint32_t key[kItems][4];
    load_keys<THREADS>(row, s * kSpan, T, vec, key);
    const uint32_t tot = compact_span<THREADS>(key, tau, quota, gt_base, eq_base, static_cast<int32_t>(s * kSpan), k,
                                               out, sh);
    gt_base += tot & 0xffffu;
    eq_base += tot >> 16;
    __syncthreads();   // the wave totals are rewritten by the next span
  }
}

__global__ __launch_bounds__(1024, 4) void select_whole_row_kernel(const float* __restrict__ scores, int64_t T,
                                                                   int64_t row_stride, int64_t k,
                                                                   int32_t* __restrict__ idx_out) {
  __shared__ SelectShared sh;
  const float* row = scores + static_cast<int64_t>(blockIdx.x) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  select_whole_row<true>(row, T, vec, static_cast<uint32_t>(k), idx_out + static_cast<int64_t>(blockIdx.x) * k, sh);
}

// ---------------------------------------------------------------- long rows: pivots, partition, finish

// Workspace of the three-launch path (device pointers into the caller's workspace).  A thread of the finish
// step holds 16 candidate slots; slot j belongs to span j / slots_per_span, so a span's slice holds
// slots_per_span * 1024 candidates.
struct SelectWs {
  uint32_t* pivot;    // [n_rows][2]  p_lo, p_hi
  uint32_t* flag;     // [n_rows]     set by partition: a thread ran out of staging slots
  uint32_t* above;    // [n_rows][n_spans]  keys above p_hi in the span
  uint32_t* n_cand;   // [n_rows][n_spans]  keys inside [p_lo, p_hi] in the span (may exceed the slice: overflow)
  uint32_t* cand;     // [n_rows][kRowCap]  the spans' slices, each dense from its start
  int32_t n_spans;    // at most 16
  int32_t slots_per_span;   // 16 / n_spans
  int32_t spans_per_block;  // finish step: neighbouring spans one block writes
};

struct SamplePlan {
  int32_t n_items;    // float4 items in the sample (4 per 64-byte chunk), at most 4096
  int32_t spacing;    // elements between chunk slots
  uint32_t rank_hi;   // sample rank (1-based, from the top) that p_hi must stay above; 0: no upper pivot
  uint32_t rank_lo;   // sample rank that p_lo must stay below; 0: no lower pivot
};

// One block per row: p_hi and p_lo from a sample of the row.  The sample is n_items / 4 chunks of 16
// consecutive scores, one chunk per `spacing` elements at a position that a hash of the chunk number
// jitters (so that a periodic pattern in the scores cannot line up with the sample).  The sample keys
// are counted in bins of 2^kFineShift keys (1/32 of an octave) below the sample's maximum, keys more than
// 64 octaves below it share bin 0; p_hi is the upper edge of the bin that holds sample rank rank_hi,
// p_lo the lower edge of the bin that holds rank_lo.
__global__ __launch_bounds__(1024, 8) void select_pivots_kernel(const float* __restrict__ scores, int64_t T,
                                                                int64_t row_stride, SamplePlan plan, SelectWs ws) {
  constexpr int THREADS = 1024, kItems = Shape<THREADS>::kItems, kWaves = Shape<THREADS>::kWaves;
  __shared__ SelectShared sh;
  const float* row = scores + static_cast<int64_t>(blockIdx.x) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  uint32_t key[kItems][4];
  uint32_t top = 0;
#pragma unroll
  for (int c = 0; c < kItems; ++c) {
    const int q = c * THREADS + static_cast<int>(threadIdx.x);   // sample item
#pragma unroll
    for (int e = 0; e < 4; ++e) key[c][e] = 0u;
    if (q < plan.n_items) {
      const uint32_t chunk = static_cast<uint32_t>(q) >> 2;
      const uint32_t slots = static_cast<uint32_t>(plan.spacing - 16) / 4 + 1;      // 4-aligned start positions
      const uint32_t jitter = ((chunk * 2654435761u) >> 8) % slots * 4;
      const int64_t i = static_cast<int64_t>(chunk) * plan.spacing + jitter + (q & 3) * 4;   // i + 4 <= T
      if (vec) {
        const uint4 raw = *reinterpret_cast<const uint4*>(row + i);
        key[c][0] = to_key(raw.x); key[c][1] = to_key(raw.y); key[c][2] = to_key(raw.z); key[c][3] = to_key(raw.w);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) key[c][e] = to_key(__float_as_uint(row[i + e]));
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) top = max(top, key[c][e]);
  }
  clear_histogram<THREADS>(sh);
  top = wave_max(top);
  if ((threadIdx.x & (kWave - 1)) == 0) sh.wave_tot[threadIdx.x / kWave] = top;
  __syncthreads();
  top = sh.wave_tot[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) top = max(top, sh.wave_tot[w]);
  constexpr uint32_t kReach = (static_cast<uint32_t>(kBins) << kFineShift) - 1;   // top - base
  const uint32_t base = top > kReach ? top - kReach : 0u;
  const uint32_t copy = threadIdx.x & (kCopies - 1);
#pragma unroll
  for (int c = 0; c < kItems; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // bin = (key - base) >> kFineShift, 0 for keys below base; at most kBins - 1 since key <= top
      const uint32_t bin = min((max(key[c][e], base) - base) >> kFineShift, static_cast<uint32_t>(kBins - 1));
      if (key[c][e] != 0) atomicAdd(&sh.hist[bin * kCopies + copy], 1u);   // slots that hold no score are skipped
    }
  __syncthreads();
  uint32_t r_hi = plan.rank_hi != 0 ? plan.rank_hi : 1u;
  const uint32_t r_lo = plan.rank_lo != 0 ? plan.rank_lo : r_hi;
  uint32_t bin_hi, bin_lo, cnt;
  find_digit<THREADS, true>(sh, r_hi, bin_hi, cnt, r_lo, bin_lo);
  if (threadIdx.x == 0) {
    // 64-bit: (bin + 1) << kFineShift may pass 2^32 when base is 0
    const uint64_t hi_edge = static_cast<uint64_t>(base) + ((static_cast<uint64_t>(bin_hi) + 1) << kFineShift) - 1;
    const uint32_t p_hi =
        plan.rank_hi != 0 ? static_cast<uint32_t>(min(hi_edge, static_cast<uint64_t>(0xffffffffu))) : 0xffffffffu;
    uint32_t p_lo = (plan.rank_lo != 0 && bin_lo != 0) ? base + (bin_lo << kFineShift) : 1u;
    if (p_lo == 0) p_lo = 1;   // key 0 marks slots beyond the row: never a candidate
    ws.pivot[2 * blockIdx.x + 0] = p_lo;
    ws.pivot[2 * blockIdx.x + 1] = p_hi;
    ws.flag[blockIdx.x] = 0;
  }
}

// One block per (row, span): keys above p_hi are counted, keys inside [p_lo, p_hi] are staged per thread in
// LDS and then written densely to the span's slice of the row's candidate list.
__global__ __launch_bounds__(1024, 8) void select_partition_kernel(const float* __restrict__ scores, int64_t T,
                                                                   int64_t row_stride, SelectWs ws) {
  constexpr int THREADS = 1024, kItems = Shape<THREADS>::kItems, kWaves = Shape<THREADS>::kWaves;
  __shared__ uint32_t stage[kLaneCap * THREADS];   // [slot][thread], 32 KiB
  __shared__ uint32_t wave_above[kWaves], wave_cand[kWaves];
  const int span = blockIdx.y, r = blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  const float* row = scores + static_cast<int64_t>(r) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  uint32_t key[kItems][4];
  load_keys<THREADS>(row, static_cast<int64_t>(span) * kSpan, T, vec, key);
  const uint32_t p_lo = ws.pivot[2 * r], p_hi = ws.pivot[2 * r + 1];
  const uint32_t width = p_hi - p_lo;
  uint32_t above = 0;      // wave-uniform
  uint32_t mine = 0;       // candidates this thread has staged
  bool lost = false;
#pragma unroll
  for (int c = 0; c < kItems; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t kk = key[c][e];
      above += static_cast<uint32_t>(__builtin_popcountll(__builtin_amdgcn_ballot_w64(kk > p_hi)));
      if (kk - p_lo <= width) {          // p_lo <= kk <= p_hi (unsigned wrap below p_lo)
        if (mine < kLaneCap) stage[mine * THREADS + threadIdx.x] = kk;
        else lost = true;
        ++mine;
      }
    }
  if (lost) {
    ws.flag[r] = 1;   // every writer stores the same value
    mine = kLaneCap;
  }
  const uint32_t incl = wave_inclusive_scan(mine);
  if (lane == kWave - 1) wave_cand[wave] = incl;
  if (lane == 0) wave_above[wave] = above;
  __syncthreads();
  uint32_t before = incl - mine, block_cand = 0, block_above = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t n = wave_cand[w];
    before += w < wave ? n : 0u;
    block_cand += n;
    block_above += wave_above[w];
  }
  if (threadIdx.x == 0) {
    ws.above[static_cast<int64_t>(r) * ws.n_spans + span] = block_above;
    ws.n_cand[static_cast<int64_t>(r) * ws.n_spans + span] = block_cand;
  }
  const uint32_t cap = static_cast<uint32_t>(ws.slots_per_span) * THREADS;
  uint32_t* slice = ws.cand + static_cast<int64_t>(r) * kRowCap + static_cast<int64_t>(span) * cap;
  for (uint32_t j = 0; j < mine; ++j)
    if (before + j < cap) slice[before + j] = stage[j * THREADS + threadIdx.x];
}

// Sum of `v` over the block (every thread gets it).  Uses sh.reduce[slot]; two barriers.
__device__ __forceinline__ uint32_t block_sum(uint32_t v, SelectShared& sh, int slot) {
  if (threadIdx.x == 0) sh.reduce[slot] = 0;
  __syncthreads();
  v = wave_sum(v);
  if ((threadIdx.x & (kWave - 1)) == 0) atomicAdd(&sh.reduce[slot], v);   // integer: order does not matter
  __syncthreads();
  return sh.reduce[slot];
}

// One block per (row, group of spans_per_block neighbouring spans): tau among the row's candidates (the same
// work for every block of a row, so blocks take several spans when there are more blocks than the chip holds
// at once), then the kept indices of its spans.
__global__ __launch_bounds__(1024, 8) void select_finish_kernel(const float* __restrict__ scores, int64_t T,
                                                                int64_t row_stride, int64_t k,
                                                                int32_t* __restrict__ idx_out, SelectWs ws) {
  constexpr int THREADS = 1024, kItems = Shape<THREADS>::kItems;
  constexpr int kSlots = kRowCap / THREADS;   // 16 candidate slots per thread
  __shared__ SelectShared sh;
  const int first_span = blockIdx.y * ws.spans_per_block, r = blockIdx.x;
  const int end_span = min(first_span + ws.spans_per_block, ws.n_spans);
  const float* row = scores + static_cast<int64_t>(r) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  int32_t* out = idx_out + static_cast<int64_t>(r) * k;
  const uint32_t kk = static_cast<uint32_t>(k);
  const uint32_t cap = static_cast<uint32_t>(ws.slots_per_span) * THREADS;

  // per-span counts first (lane s of every wave fetches span s; at most 16 spans), then the first span's own
  // scores, which stay in flight through the selection
  const int lane = threadIdx.x & (kWave - 1);
  uint32_t n_mine = 0, a_mine = 0;
  if (lane < ws.n_spans) {
    n_mine = ws.n_cand[static_cast<int64_t>(r) * ws.n_spans + lane];
    a_mine = ws.above[static_cast<int64_t>(r) * ws.n_spans + lane];
  }
  const uint32_t flagged = ws.flag[r];
  const bool whole = vec && static_cast<int64_t>(first_span + 1) * kSpan <= T;
  uint4 raw[kItems];
  if (whole) {
#pragma unroll
    for (int c = 0; c < kItems; ++c)
      raw[c] = *reinterpret_cast<const uint4*>(row + static_cast<int64_t>(first_span) * kSpan +
                                               c * Shape<THREADS>::kChunk + static_cast<int64_t>(threadIdx.x) * 4);
  }
  // the row's candidates: slot j of this thread is entry (j % slots_per_span) * 1024 + thread of span j / slots_per_span
  const uint32_t* list = ws.cand + static_cast<int64_t>(r) * kRowCap;
  uint32_t ck[kSlots];
  {
    int s = 0, sub = 0;   // uniform
#pragma unroll
    for (int j = 0; j < kSlots; ++j) {
      ck[j] = 0u;                                  // an empty slot
      if (s < ws.n_spans) {
        const uint32_t n = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(n_mine), s));
        const uint32_t i = static_cast<uint32_t>(sub) * THREADS + threadIdx.x;
        if (i < min(n, cap)) ck[j] = list[static_cast<int64_t>(s) * cap + i];
      }
      if (++sub == ws.slots_per_span) {
        sub = 0;
        ++s;
      }
    }
  }
  const uint32_t a_all = wave_sum(a_mine), c_all = wave_sum(n_mine);
  const uint32_t overflow = flagged | (__builtin_amdgcn_ballot_w64(n_mine > cap) != 0 ? 1u : 0u);
  if (overflow != 0 || !(a_all < kk && kk <= a_all + c_all)) {
    // a slice or a thread's staging slots overflowed, or the bracket missed: one block redoes the row
    if (first_span == 0) select_whole_row<false>(row, T, vec, kk, out, sh);
    return;
  }
  clear_histogram<THREADS>(sh);
  __syncthreads();
  auto visit = [&](auto&& f) {
#pragma unroll
    for (int j = 0; j < kSlots; ++j) f(ck[j]);   // empty slots hold key 0, outside [p_lo, p_hi]
  };
  const uint32_t p_lo = ws.pivot[2 * r], p_hi = ws.pivot[2 * r + 1];
  uint32_t tau, quota;
  interval_select<THREADS, false>(visit, visit, kk - a_all, p_lo, p_hi - p_lo, sh, tau, quota);
  for (int span = first_span; span < end_span; ++span) {
    uint32_t key[kItems][4];
    if (whole && span == first_span) {
#pragma unroll
      for (int c = 0; c < kItems; ++c) {
        key[c][0] = to_key(raw[c].x); key[c][1] = to_key(raw[c].y);
        key[c][2] = to_key(raw[c].z); key[c][3] = to_key(raw[c].w);
      }
    } else {
      load_keys<THREADS>(row, static_cast<int64_t>(span) * kSpan, T, vec, key);
    }
    // kept-class counts of the earlier spans: their keys above p_hi, plus their candidates above / equal to tau
    const uint32_t a_before = wave_sum(lane < span ? a_mine : 0u);
    uint32_t gq = 0;   // greater | equal << 16, each at most kRowCap
    {
      int s = 0, sub = 0;
#pragma unroll
      for (int j = 0; j < kSlots; ++j) {
        if (s < span && ck[j] != 0) gq += (ck[j] > tau ? 1u : 0u) + (ck[j] == tau ? 0x10000u : 0u);
        if (++sub == ws.slots_per_span) {
          sub = 0;
          ++s;
        }
      }
    }
    gq = block_sum(gq, sh, span & 7);
    compact_span<THREADS>(key, tau, quota, a_before + (gq & 0xffffu), gq >> 16, span * kSpan, kk, out, sh);
    __syncthreads();   // the wave totals are rewritten for the next span
  }
}

// ---------------------------------------------------------------- host side

size_t align256(size_t n) { return (n + 255) / 256 * 256; }

bool split_path(int64_t T) { return T > kSpan && T <= kMaxSplitT; }

struct SelectLayout {
  size_t pivot, flag, above, n_cand, cand, total;
  int64_t n_spans;
};

SelectLayout select_layout(int64_t n_rows, int64_t T) {
  SelectLayout w{};
  if (!split_path(T) || n_rows <= 0) return w;
  w.n_spans = ceil_div(T, kSpan);
  w.pivot = align256(static_cast<size_t>(n_rows) * 2 * sizeof(uint32_t));
  w.flag = align256(static_cast<size_t>(n_rows) * sizeof(uint32_t));
  w.above = align256(static_cast<size_t>(n_rows) * w.n_spans * sizeof(uint32_t));
  w.n_cand = w.above;
  w.cand = align256(static_cast<size_t>(n_rows) * kRowCap * sizeof(uint32_t));
  w.total = w.pivot + w.flag + w.above + w.n_cand + w.cand;
  return w;
}

// Sample size and the two sample ranks that bracket the k-th largest of the row.  With n sample elements
// the rank of tau inside the sample is close to k * n / T; its spread for an independent sample is
// sigma = sqrt(n f (1 - f)), f = k / T.  Scores of neighbouring tokens are correlated and the sample takes
// them 16 at a time, so the margin is generous: 6 sigma + 16 ranks on either side.
SamplePlan make_sample_plan(int64_t T, int64_t k) {
  SamplePlan p{};
  int64_t n = 4096;                       // sample elements: T / 8 rounded down to a power of two, in [4096, 16384]
  while (n < 16384 && n * 2 <= T / 8) n *= 2;
  p.n_items = static_cast<int32_t>(n / 4);
  p.spacing = static_cast<int32_t>(T / (n / 16)) & ~3;   // >= 64 elements per 16-element chunk, 16-byte steps
  const double f = static_cast<double>(k) / static_cast<double>(T);
  const double expect = f * static_cast<double>(n);
  const double sigma = sqrt(static_cast<double>(n) * f * (1.0 - f));
  const int64_t margin = static_cast<int64_t>(6.0 * sigma) + 16;
  const int64_t hi = static_cast<int64_t>(expect) - margin;       // floor(expect) - margin
  const int64_t lo = static_cast<int64_t>(expect) + 1 + margin;   // >= ceil(expect) + margin
  p.rank_hi = hi >= 1 ? static_cast<uint32_t>(hi) : 0u;
  p.rank_lo = lo <= n ? static_cast<uint32_t>(lo) : 0u;
  return p;
}

}  // namespace

size_t select_workspace_bytes(int64_t n_rows, int64_t T) { return select_layout(n_rows, T).total; }

void select_topk_launch(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                        int32_t* idx_out, void* ws, hipStream_t st) {
  const dim3 rows(static_cast<unsigned>(n_rows));
  if (T <= kSpan) {
    // A CU holds two 1024-thread blocks or three 512-thread ones.  The wider block finishes a row sooner, which wins
    // up to one and a half rounds of wide blocks (measured: 640 rows take 26.6 us wide, 28.3 us narrow); beyond
    // that the narrower shape, with more rows in flight, is ahead.
    if (n_rows <= 3 * 256)
      select_resident_kernel<1024><<<rows, 1024, 0, st>>>(scores, T, row_stride, k, idx_out);
    else
      select_resident_kernel<512><<<rows, 512, 0, st>>>(scores, T, row_stride, k, idx_out);
    return;
  }
  if (!split_path(T)) {
    select_whole_row_kernel<<<rows, 1024, 0, st>>>(scores, T, row_stride, k, idx_out);
    return;
  }
  const SelectLayout lay = select_layout(n_rows, T);
  char* base = static_cast<char*>(ws);
  SelectWs w{};
  w.pivot = reinterpret_cast<uint32_t*>(base);
  w.flag = reinterpret_cast<uint32_t*>(base + lay.pivot);
  w.above = reinterpret_cast<uint32_t*>(base + lay.pivot + lay.flag);
  w.n_cand = reinterpret_cast<uint32_t*>(base + lay.pivot + lay.flag + lay.above);
  w.cand = reinterpret_cast<uint32_t*>(base + lay.pivot + lay.flag + lay.above + lay.n_cand);
  w.n_spans = static_cast<int32_t>(lay.n_spans);
  w.slots_per_span = static_cast<int32_t>(16 / lay.n_spans);
  const SamplePlan plan = make_sample_plan(T, k);
  const dim3 spans(static_cast<unsigned>(n_rows), static_cast<unsigned>(lay.n_spans));   // at most 16 spans
  select_pivots_kernel<<<rows, 1024, 0, st>>>(scores, T, row_stride, plan, w);
  select_partition_kernel<<<spans, 1024, 0, st>>>(scores, T, row_stride, w);
  // the finish step repeats the selection among the candidates in every block of a row: with more blocks than the
  // chip holds at once (two per CU) a block takes several spans instead
  w.spans_per_block = static_cast<int32_t>(std::min<int64_t>(lay.n_spans, std::max<int64_t>(1, ceil_div(n_rows * lay.n_spans, 512))));
  const dim3 groups(static_cast<unsigned>(n_rows), static_cast<unsigned>(ceil_div(lay.n_spans, w.spans_per_block)));
  select_finish_kernel<<<groups, 1024, 0, st>>>(scores, T, row_stride, k, idx_out, w);
}

}  // namespace kvp

extern "C" size_t kvp_select_workspace_bytes(int64_t n_rows, int64_t T, int64_t k) {
  (void)k;
  if (n_rows <= 0 || T <= 0) return 0;
  return kvp::select_workspace_bytes(n_rows, T);
}

extern "C" int32_t kvp_select_topk(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                                   int32_t* idx_out, void* ws, size_t ws_bytes, void* stream) {
  using namespace kvp;
  if (!scores || (!idx_out && k > 0)) return KVP_ERR_NULL;
  if (n_rows < 0 || T <= 0 || T >= (1ll << 30) || k < 0 || k > T || row_stride < T || n_rows >= (1ll << 31))
    return KVP_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(scores) & 3u) || (reinterpret_cast<uintptr_t>(idx_out) & 3u)) return KVP_ERR_ALIGN;
  if (n_rows == 0 || k == 0) return KVP_OK;
  const size_t need = select_workspace_bytes(n_rows, T);
  if (need != 0 && (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15u))) return KVP_ERR_WORKSPACE;
  select_topk_launch(scores, n_rows, T, row_stride, k, idx_out, ws, as_stream(stream));
  return launch_status();
}
