// kvp_select_topk: per-row top-k keep-set by radix select (the paper's token dropping keeps the
// tokens with the highest attention scores: Evaluation, Baselines, snapkv / IMPRESS top X %).
//
// Scores are mapped to order-preserving unsigned keys (-0 folded onto +0).  A block finds the key
// tau of the k-th largest score and the quota of elements equal to tau that belong to the keep-set
// with three most-significant-digit-first passes over 11 + 11 + 10 bit digits (LDS histograms, four
// interleaved copies), then writes the kept indices in ascending order: position = (number of
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
//   * longer rows (up to 2^20 scores) are split into 16384-element spans, one block per span, in
//     three launches, so that the whole chip works on a few long rows:
//       pivots     one block per row selects, from an evenly spread sample of the row, two keys
//                  p_lo <= p_hi that bracket tau with overwhelming probability;
//       partition  every span counts its keys above p_hi and stores the few keys inside
//                  [p_lo, p_hi] (its candidates) in the workspace;
//       finish     every span block adds up the counts of its row, selects tau among the row's
//                  candidates (rank k minus the keys above p_hi), derives its own output offset
//                  from the counts of the earlier spans and writes its kept indices.
//     If the bracket misses (the k-th largest is not among the candidates) or a span has more
//     candidates than its workspace slice holds (heavy ties at the threshold), the finish step
//     flags the row and
//   * the streaming kernel (one block per row, spans re-read for every one of four 8-bit passes)
//     redoes flagged rows; it also serves rows beyond 2^20 scores.
// Every step is deterministic: the output never depends on the order in which blocks or candidates
// are processed.

#include "kvp_internal.h"

namespace kvp {
namespace {

constexpr int kSpan = 16384;          // elements a block holds in registers at a time
constexpr int kBins = 2048;           // bins of the widest digit
constexpr int kCopies = 4;            // interleaved histogram copies (lane & 3)
constexpr int kSpanCap = 4096;        // candidate slots per span in the workspace
constexpr int64_t kMaxSampledT = 1 << 20;

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
// number of set bits of a wave mask below this lane, added to acc
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask, uint32_t acc) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), acc));
}

struct alignas(16) SelectShared {
  uint32_t hist[kBins * kCopies];     // [bin][copy], 32 KiB
  uint32_t wave_tot[64];
  uint32_t result[4];                 // chosen digit, remaining rank, population of the chosen bin
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

// After a histogram pass (and a barrier): the digit whose bin holds the krem-th largest key, counted from
// the top bin down; krem becomes the rank inside that bin, cnt its population.  Clears the histogram.
// Needs 1 <= krem <= population of the histogram.  Ends with a barrier.
template <int THREADS>
__device__ __forceinline__ void find_digit(SelectShared& sh, uint32_t& krem, uint32_t& digit, uint32_t& cnt) {
  constexpr int kWaves = Shape<THREADS>::kWaves;
  constexpr int BPT = kBins / THREADS;              // bins per thread: 2 or 4
  static_assert(kCopies == 4, "one uint4 per bin");
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  // thread t owns the BPT bins below kBins - t * BPT (threads in descending bin order)
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
  const uint32_t tot_mine = lane < kWaves ? sh.wave_tot[lane] : 0u;
  const uint32_t tot_incl = wave_inclusive_scan(tot_mine);
  uint32_t above = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(tot_incl - tot_mine), wave)) +
                   incl - local;                    // keys in bins above this thread's
  if (above < krem && krem <= above + local) {      // exactly one thread of the block
#pragma unroll
    for (int j = BPT - 1; j >= 0; --j) {
      if (above < krem && krem <= above + c[j]) {
        sh.result[0] = static_cast<uint32_t>(lo_bin + j);
        sh.result[1] = krem - above;
        sh.result[2] = c[j];
      }
      above += c[j];
    }
  }
  __syncthreads();
  digit = sh.result[0];
  krem = sh.result[1];
  cnt = sh.result[2];
}

// Block-wide radix select over the keys `visit` enumerates: visit(f) calls f(key) for every key this
// thread owns (the same keys on every call).  Finds tau and quota such that the k largest keys are the
// keys above tau plus `quota` of the keys equal to tau.  1 <= k <= number of keys.  The histogram must be
// clear on entry (and a barrier passed); it is clear again on return.
template <int THREADS, class Visit>
__device__ __forceinline__ void radix_select(Visit&& visit, uint32_t k, SelectShared& sh, uint32_t& tau,
                                             uint32_t& quota) {
  const uint32_t copy = threadIdx.x & (kCopies - 1);
  uint32_t prefix = 0, mask = 0, krem = k;
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int shift = pass == 0 ? 21 : pass == 1 ? 10 : 0;
    const uint32_t dmask = pass == 2 ? 0x3ffu : 0x7ffu;
    visit([&](uint32_t key) {
      if (pass == 0 || (key & mask) == prefix) atomicAdd(&sh.hist[((key >> shift) & dmask) * kCopies + copy], 1u);
    });
    __syncthreads();
    uint32_t digit, cnt;
    find_digit<THREADS>(sh, krem, digit, cnt);
    prefix |= digit << shift;
    mask |= dmask << shift;
    if (pass < 2 && cnt == krem && prefix != 0) {
      // every key of the chosen bin belongs to the k largest: keep exactly the keys >= prefix
      tau = prefix - 1;
      quota = 0;
      return;
    }
  }
  tau = prefix;
  quota = krem;
}

// Ordered compaction of one span held in registers: writes first_index + (span element index) of every
// kept element to out[] in ascending order.  gt_base / eq_base: kept-class counts of the row's elements
// before this span.  Positions are checked against k before every store, so that inputs outside the
// contract (NaN scores) cannot make the kernel write outside its row of the output.
template <int THREADS>
__device__ __forceinline__ void compact_span(const uint32_t (&key)[Shape<THREADS>::kItems][4], uint32_t tau,
                                             uint32_t quota, uint32_t gt_base, uint32_t eq_base, int32_t first_index,
                                             uint32_t k, int32_t* __restrict__ out, SelectShared& sh) {
  constexpr int kWaves = Shape<THREADS>::kWaves, kItems = Shape<THREADS>::kItems, kChunk = Shape<THREADS>::kChunk;
  static_assert(kItems * kWaves == kWave, "one (item, wave) total per lane of the scanning wave");
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
  // phase 1: rank of this lane inside its wave, per item, for both classes; wave totals to LDS
  uint32_t rank[kItems];      // (greater | equal << 16) elements of the earlier lanes of this wave, per item
  uint32_t eq_items = 0;      // wave-uniform: bit c set if this wave's part of item c holds an element equal to tau
#pragma unroll
  for (int c = 0; c < kItems; ++c) {
    uint32_t g = 0, q = 0, tg = 0, te = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint64_t bg = __builtin_amdgcn_ballot_w64(key[c][e] > tau);
      g = lanes_below(bg, g);
      tg += static_cast<uint32_t>(__builtin_popcountll(bg));
      const uint64_t be = __builtin_amdgcn_ballot_w64(key[c][e] == tau);
      if (be != 0) {   // wave-uniform, rare
        q = lanes_below(be, q);
        te += static_cast<uint32_t>(__builtin_popcountll(be));
      }
    }
    rank[c] = g | (q << 16);
    if (te != 0) eq_items |= 1u << c;
    // a span holds 16384 elements: both totals fit 16 bits, also when summed over the block
    if (lane == 0) sh.wave_tot[c * kWaves + wave] = tg | (te << 16);
  }
  __syncthreads();
  // the (item, wave) totals are in element order: every wave scans them, one per lane
  const uint32_t tot_mine = sh.wave_tot[lane];
  const uint32_t tot_excl = wave_inclusive_scan(tot_mine) - tot_mine;
  // phase 2: emit
#pragma unroll
  for (int c = 0; c < kItems; ++c) {
    const uint32_t before = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(tot_excl), c * kWaves + wave));
    uint32_t gt_before = gt_base + (before & 0xffffu) + (rank[c] & 0xffffu);
    uint32_t eq_before = eq_base + (before >> 16) + (rank[c] >> 16);
    const int32_t i0 = first_index + c * kChunk + static_cast<int32_t>(threadIdx.x) * 4;   // T < 2^31
    if ((eq_items & (1u << c)) == 0) {
      // no element of this wave's part equals tau: the kept ones are simply those above it
      uint32_t p = gt_before + min(eq_before, quota);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (key[c][e] > tau) {
          if (p < k) out[p] = i0 + e;
          ++p;
        }
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t kk = key[c][e];
        if (kk > tau) {
          const uint32_t p = gt_before + min(eq_before, quota);
          if (p < k) out[p] = i0 + e;
          ++gt_before;
        } else if (kk == tau) {
          if (eq_before < quota && gt_before + eq_before < k) out[gt_before + eq_before] = i0 + e;
          ++eq_before;
        }
      }
    }
  }
}

// ---------------------------------------------------------------- rows that fit one span

template <int THREADS>
__global__ __launch_bounds__(THREADS, THREADS == 1024 ? 8 : 6) void select_resident_kernel(const float* __restrict__ scores, int64_t T,
                                                                     int64_t row_stride, int64_t k,
                                                                     int32_t* __restrict__ idx_out) {
  constexpr int kItems = Shape<THREADS>::kItems;
  __shared__ SelectShared sh;
  const float* row = scores + static_cast<int64_t>(blockIdx.x) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  uint32_t key[kItems][4];
  load_keys<THREADS>(row, 0, T, vec, key);
  clear_histogram<THREADS>(sh);
  __syncthreads();
  uint32_t tau, quota;
  radix_select<THREADS>(
      [&](auto&& f) {
#pragma unroll
        for (int c = 0; c < kItems; ++c)
#pragma unroll
          for (int e = 0; e < 4; ++e) f(key[c][e]);
      },
      static_cast<uint32_t>(k), sh, tau, quota);
  compact_span<THREADS>(key, tau, quota, 0, 0, 0, static_cast<uint32_t>(k), idx_out + static_cast<int64_t>(blockIdx.x) * k, sh);
}

// ---------------------------------------------------------------- long rows: pivots, partition, finish

// Workspace of the three-launch path (device pointers into the caller's workspace).
struct SelectWs {
  uint32_t* pivot;    // [n_rows][2]  p_lo, p_hi
  uint32_t* flag;     // [n_rows]     1: the streaming kernel has to redo the row
  uint32_t* above;    // [n_rows][n_spans]  keys above p_hi in the span
  uint32_t* n_cand;   // [n_rows][n_spans]  keys inside [p_lo, p_hi] in the span (may exceed kSpanCap: overflow)
  uint32_t* cand;     // [n_rows][n_spans][kSpanCap]
  int32_t n_spans;
};

struct SamplePlan {
  int32_t n_items;    // float4 items in the sample (4 per 64-byte chunk), at most 4096
  int32_t spacing;    // elements between chunk slots
  uint32_t rank_hi;   // sample rank (1-based, from the top) of p_hi; 0: no upper pivot
  uint32_t rank_lo;   // sample rank of p_lo; 0: no lower pivot
};

// One block per row: p_hi and p_lo from a sample of the row.  The sample is n_items / 4 chunks of 16
// consecutive scores, one chunk per `spacing` elements at a position that a hash of the chunk number
// jitters (so that a periodic pattern in the scores cannot line up with the sample).
__global__ __launch_bounds__(1024, 8) void select_pivots_kernel(const float* __restrict__ scores, int64_t T,
                                                                int64_t row_stride, SamplePlan plan, SelectWs ws) {
  constexpr int THREADS = 1024, kItems = Shape<THREADS>::kItems;
  __shared__ SelectShared sh;
  const float* row = scores + static_cast<int64_t>(blockIdx.x) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  uint32_t key[kItems][4];
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
  }
  clear_histogram<THREADS>(sh);
  __syncthreads();
  auto visit = [&](auto&& f) {
#pragma unroll
    for (int c = 0; c < kItems; ++c)
#pragma unroll
      for (int e = 0; e < 4; ++e) f(key[c][e]);
  };
  uint32_t p_hi = 0xffffffffu, p_lo = 1u, quota;
  if (plan.rank_hi != 0) radix_select<THREADS>(visit, plan.rank_hi, sh, p_hi, quota);
  if (plan.rank_lo != 0) radix_select<THREADS>(visit, plan.rank_lo, sh, p_lo, quota);
  if (p_lo == 0) p_lo = 1;   // key 0 marks slots beyond the row: never a candidate
  if (threadIdx.x == 0) {
    ws.pivot[2 * blockIdx.x + 0] = p_lo;
    ws.pivot[2 * blockIdx.x + 1] = p_hi;
    ws.flag[blockIdx.x] = 0;
  }
}

// One block per (row, span): keys above p_hi are counted, keys inside [p_lo, p_hi] go to the span's
// candidate slice (in arrival order: only their multiset is used later).
__global__ __launch_bounds__(1024, 8) void select_partition_kernel(const float* __restrict__ scores, int64_t T,
                                                                   int64_t row_stride, SelectWs ws) {
  constexpr int THREADS = 1024, kItems = Shape<THREADS>::kItems;
  __shared__ uint32_t n_above_s, n_cand_s;
  const int span = blockIdx.y, r = blockIdx.x;
  const float* row = scores + static_cast<int64_t>(r) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  uint32_t key[kItems][4];
  load_keys<THREADS>(row, static_cast<int64_t>(span) * kSpan, T, vec, key);
  if (threadIdx.x == 0) {
    n_above_s = 0;
    n_cand_s = 0;
  }
  __syncthreads();
  const uint32_t p_lo = ws.pivot[2 * r], p_hi = ws.pivot[2 * r + 1];
  uint32_t* slice = ws.cand + (static_cast<int64_t>(r) * ws.n_spans + span) * kSpanCap;
  uint32_t above = 0;
#pragma unroll
  for (int c = 0; c < kItems; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t kk = key[c][e];
      above += kk > p_hi ? 1u : 0u;
      if (kk >= p_lo && kk <= p_hi) {
        const uint32_t slot = atomicAdd(&n_cand_s, 1u);
        if (slot < kSpanCap) slice[slot] = kk;
      }
    }
  above = wave_sum(above);
  if ((threadIdx.x & (kWave - 1)) == 0) atomicAdd(&n_above_s, above);
  __syncthreads();
  if (threadIdx.x == 0) {
    ws.above[static_cast<int64_t>(r) * ws.n_spans + span] = n_above_s;
    ws.n_cand[static_cast<int64_t>(r) * ws.n_spans + span] = n_cand_s;
  }
}

// Sum of `v` over the block (every thread gets it).  Uses sh.reduce; two barriers.
template <int THREADS>
__device__ __forceinline__ uint32_t block_sum(uint32_t v, SelectShared& sh, int slot) {
  if (threadIdx.x == 0) sh.reduce[slot] = 0;
  __syncthreads();
  v = wave_sum(v);
  if ((threadIdx.x & (kWave - 1)) == 0) atomicAdd(&sh.reduce[slot], v);   // integer: order does not matter
  __syncthreads();
  return sh.reduce[slot];
}

// One block per (row, span): tau among the row's candidates, then the span's kept indices.
__global__ __launch_bounds__(1024, 8) void select_finish_kernel(const float* __restrict__ scores, int64_t T,
                                                                int64_t row_stride, int64_t k,
                                                                int32_t* __restrict__ idx_out, SelectWs ws) {
  constexpr int THREADS = 1024, kItems = Shape<THREADS>::kItems;
  __shared__ SelectShared sh;
  const int span = blockIdx.y, r = blockIdx.x;
  const float* row = scores + static_cast<int64_t>(r) * row_stride;
  const bool vec = (reinterpret_cast<uintptr_t>(row) & 15u) == 0;
  uint32_t key[kItems][4];
  load_keys<THREADS>(row, static_cast<int64_t>(span) * kSpan, T, vec, key);   // in flight during the selection

  const uint32_t* above = ws.above + static_cast<int64_t>(r) * ws.n_spans;
  const uint32_t* n_cand = ws.n_cand + static_cast<int64_t>(r) * ws.n_spans;
  const uint32_t* cand = ws.cand + static_cast<int64_t>(r) * ws.n_spans * kSpanCap;
  uint32_t a_all = 0, a_before = 0, c_all = 0, overflow = 0;
  for (int s = threadIdx.x; s < ws.n_spans; s += THREADS) {
    const uint32_t a = above[s], n = n_cand[s];
    a_all += a;
    a_before += s < span ? a : 0u;
    c_all += min(n, static_cast<uint32_t>(kSpanCap));
    overflow += n > kSpanCap ? 1u : 0u;
  }
  a_all = block_sum<THREADS>(a_all, sh, 0);
  a_before = block_sum<THREADS>(a_before, sh, 1);
  c_all = block_sum<THREADS>(c_all, sh, 2);
  overflow = block_sum<THREADS>(overflow, sh, 3);
  const uint32_t kk = static_cast<uint32_t>(k);
  if (overflow != 0 || !(a_all < kk && kk <= a_all + c_all)) {
    // the bracket missed, or a slice overflowed: the streaming kernel redoes this row
    if (span == 0 && threadIdx.x == 0) ws.flag[r] = 1;
    return;
  }
  clear_histogram<THREADS>(sh);
  __syncthreads();
  uint32_t tau, quota;
  radix_select<THREADS>(
      [&](auto&& f) {
        for (int s = 0; s < ws.n_spans; ++s) {
          const uint32_t n = n_cand[s];
          for (uint32_t i = threadIdx.x; i < n; i += THREADS) f(cand[static_cast<int64_t>(s) * kSpanCap + i]);
        }
      },
      kk - a_all, sh, tau, quota);
  const uint32_t p_lo = ws.pivot[2 * r];
  // an early exit of the selection returns "keep every candidate >= prefix" as tau = prefix - 1, which may lie
  // below p_lo, where the row has keys that are no candidates: they stay excluded
  if (tau < p_lo - 1) tau = p_lo - 1;
  // kept-class counts of the earlier spans: their keys above p_hi, plus their candidates above / equal to tau
  uint32_t g = 0, q = 0;
  for (int s = 0; s < span; ++s) {
    const uint32_t n = n_cand[s];
    for (uint32_t i = threadIdx.x; i < n; i += THREADS) {
      const uint32_t ck = cand[static_cast<int64_t>(s) * kSpanCap + i];
      g += ck > tau ? 1u : 0u;
      q += ck == tau ? 1u : 0u;
    }
  }
  g = block_sum<THREADS>(g, sh, 4);
  q = block_sum<THREADS>(q, sh, 5);
  compact_span<THREADS>(key, tau, quota, a_before + g, q, span * kSpan, kk, idx_out + static_cast<int64_t>(r) * k, sh);
}

// ---------------------------------------------------------------- streaming kernel (any row length)
//
// One block per row, four passes over 8-bit digits with a 32-way replicated histogram; the row is
// re-read span by span for every pass with the next two spans in flight.  Serves rows beyond the
// sampled path's limit and redoes the rows that path flags.

constexpr int kCopies8 = 32;
constexpr int kBins8 = 256;

__device__ __forceinline__ uint32_t to_key_f(float f) {
  uint32_t u = __float_as_uint(f);
  u = (u == 0x80000000u) ? 0u : u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <int ITEMS>
struct Span {
  uint32_t key[ITEMS][4];
};

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

template <int ITEMS>
__device__ __forceinline__ Span<ITEMS> to_keys(const Span<ITEMS>& raw) {
  Span<ITEMS> s;
#pragma unroll
  for (int c = 0; c < ITEMS; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) s.key[c][e] = to_key_f(__uint_as_float(raw.key[c][e]));
  return s;
}

template <int ITEMS>
__device__ __forceinline__ void histogram_span(const Span<ITEMS>& s, uint32_t mask, uint32_t prefix, int shift,
                                               uint32_t* hist) {
  const int copy = threadIdx.x & (kCopies8 - 1);
#pragma unroll
  for (int c = 0; c < ITEMS; ++c)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t key = s.key[c][e];
      // (end-of-row slots, key 0, fall into the lowest bin below every real score: harmless)
      if ((key & mask) == prefix) atomicAdd(&hist[((key >> shift) & 0xffu) * kCopies8 + copy], 1u);
    }
}

// flag: null, or one word per row; rows whose word is 0 are left alone.
__global__ __launch_bounds__(1024, 4) void select_streaming_kernel(const float* __restrict__ scores, int64_t T,
                                                                   int64_t row_stride, int64_t k,
                                                                   int32_t* __restrict__ idx_out,
                                                                   const uint32_t* __restrict__ flag) {
  constexpr int THREADS = 1024;
  constexpr int kThreads = THREADS;
  constexpr int kWaves = Shape<THREADS>::kWaves, kItems = Shape<THREADS>::kItems, kChunk = Shape<THREADS>::kChunk;
  if (flag != nullptr && flag[blockIdx.x] == 0) return;
  __shared__ uint32_t hist[kBins8 * kCopies8];
  __shared__ uint32_t cnt[kBins8];
  __shared__ uint32_t wave_tot[4][kWaves];

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);   // uniform: usable as a lane selector
  const float* row = scores + static_cast<int64_t>(blockIdx.x) * row_stride;
  int32_t* out = idx_out + static_cast<int64_t>(blockIdx.x) * k;
  const bool vec = ((reinterpret_cast<uintptr_t>(row) & 15u) == 0);

  // Two spans are kept in flight behind the one being consumed; the spans are visited cyclically
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
  load_span<THREADS>(row, next_base(), T, vec, ahead);
  cur = to_keys(cur);
  for (int i = tid; i < kBins8 * kCopies8; i += kThreads) hist[i] = 0;
  __syncthreads();

  uint32_t prefix = 0, mask = 0, krem = static_cast<uint32_t>(k);
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int64_t base = 0; base < T; base += kSpan) {
      Span<kItems> far;
      load_span<THREADS>(row, next_base(), T, vec, far);
      histogram_span(cur, mask, prefix, shift, hist);
      cur = to_keys(ahead);
      ahead = far;
    }
    __syncthreads();
    if (tid < kBins8) {
      uint32_t sum = 0;
#pragma unroll 8
      for (int c = 0; c < kCopies8; ++c) {
        const int slot = (tid * kCopies8 + (tid & (kCopies8 - 1))) ^ c;   // copy (tid ^ c) mod 32: a different bank per lane
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
    load_span<THREADS>(row, next_base(), T, vec, far);
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
    cur = to_keys(ahead);
    ahead = far;
    __syncthreads();   // wave_tot is rewritten by the next span
  }
}

// ---------------------------------------------------------------- host side

size_t align256(size_t n) { return (n + 255) / 256 * 256; }

bool sampled_path(int64_t T) { return T > kSpan && T <= kMaxSampledT; }

struct SelectLayout {
  size_t pivot, flag, above, n_cand, cand, total;
  int64_t n_spans;
};

SelectLayout select_layout(int64_t n_rows, int64_t T) {
  SelectLayout w{};
  if (!sampled_path(T) || n_rows <= 0) return w;
  w.n_spans = ceil_div(T, kSpan);
  w.pivot = align256(static_cast<size_t>(n_rows) * 2 * sizeof(uint32_t));
  w.flag = align256(static_cast<size_t>(n_rows) * sizeof(uint32_t));
  w.above = align256(static_cast<size_t>(n_rows) * w.n_spans * sizeof(uint32_t));
  w.n_cand = w.above;
  w.cand = align256(static_cast<size_t>(n_rows) * w.n_spans * kSpanCap * sizeof(uint32_t));
  w.total = w.pivot + w.flag + w.above + w.n_cand + w.cand;
  return w;
}

// Sample size and the two sample ranks that bracket the k-th largest of the row.  With n sample elements
// the rank of tau inside the sample is close to k * n / T; its spread for an independent sample is
// sigma = sqrt(n f (1 - f)), f = k / T.  Scores of neighbouring tokens are correlated and the sample takes
// them 16 at a time, so the margin is generous: 8 sigma + 16 ranks on either side.
SamplePlan make_sample_plan(int64_t T, int64_t k) {
  SamplePlan p{};
  int64_t n = 4096;                       // sample elements: T / 8 rounded down to a power of two, in [4096, 16384]
  while (n < 16384 && n * 2 <= T / 8) n *= 2;
  p.n_items = static_cast<int32_t>(n / 4);
  p.spacing = static_cast<int32_t>(T / (n / 16)) & ~3;   // >= 64 elements per 16-element chunk, 16-byte steps
  const double f = static_cast<double>(k) / static_cast<double>(T);
  const double expect = f * static_cast<double>(n);
  const double sigma = sqrt(static_cast<double>(n) * f * (1.0 - f));
  const int64_t margin = static_cast<int64_t>(8.0 * sigma) + 16;
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
  if (T <= kSpan) {
    const dim3 grid(static_cast<unsigned>(n_rows));
    // A CU holds two 1024-thread blocks or four 512-thread ones.  Up to 512 rows every row gets a slot either way
    // and the wider block finishes a row sooner; beyond that the narrower shape keeps twice the rows in flight.
    if (n_rows <= 2 * 256)
      select_resident_kernel<1024><<<grid, 1024, 0, st>>>(scores, T, row_stride, k, idx_out);
    else
      select_resident_kernel<512><<<grid, 512, 0, st>>>(scores, T, row_stride, k, idx_out);
    return;
  }
  if (!sampled_path(T)) {
    select_streaming_kernel<<<dim3(static_cast<unsigned>(n_rows)), 1024, 0, st>>>(scores, T, row_stride, k, idx_out,
                                                                                   nullptr);
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
  const SamplePlan plan = make_sample_plan(T, k);
  const dim3 rows(static_cast<unsigned>(n_rows));
  const dim3 spans(static_cast<unsigned>(n_rows), static_cast<unsigned>(lay.n_spans));   // at most 64 spans
  select_pivots_kernel<<<rows, 1024, 0, st>>>(scores, T, row_stride, plan, w);
  select_partition_kernel<<<spans, 1024, 0, st>>>(scores, T, row_stride, w);
  select_finish_kernel<<<spans, 1024, 0, st>>>(scores, T, row_stride, k, idx_out, w);
  select_streaming_kernel<<<rows, 1024, 0, st>>>(scores, T, row_stride, k, idx_out, w.flag);
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
  if (n_rows < 0 || T <= 0 || T >= (1ll << 31) || k < 0 || k > T || row_stride < T || n_rows >= (1ll << 31))
    return KVP_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(scores) & 3u) || (reinterpret_cast<uintptr_t>(idx_out) & 3u)) return KVP_ERR_ALIGN;
  if (n_rows == 0 || k == 0) return KVP_OK;
  const size_t need = select_workspace_bytes(n_rows, T);
  if (need != 0) {
    if (!ws || ws_bytes < need || (reinterpret_cast<uintptr_t>(ws) & 15u)) return KVP_ERR_WORKSPACE;
  }
  select_topk_launch(scores, n_rows, T, row_stride, k, idx_out, ws, as_stream(stream));
  return launch_status();
}
