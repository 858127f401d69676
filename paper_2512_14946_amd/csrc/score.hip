// kvp_score_tokens: attention-score token importance (the paper's snapkv baseline: cross attention
// between the tokens near the query and the earlier context; Evaluation, Baselines).
//
//   scores[l][h][t] = sum over the G*W window rows r of softmax_t(q_r . k_t / sqrt(D))
//
// Two passes over K, both with the query-window x key contraction on the bf16 MFMA
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate), because a softmax row must be normalized before it
// can be summed into a column:
//   pass A  row statistics: running max and sum of exponentials per window row, per key chunk;
//   combine per-row bias b_r = max_r + log2(sum_r) over all chunks (a tiny kernel, or the prologue of pass B
//           when there are few chunks);
//   pass B  column sums: scores[t] = sum_r 2^(s_rt - b_r).
// Logits are kept in the base-2 domain (s = q.k * log2(e)/sqrt(D)) so the exponential is one
// v_exp_f32.
//
// Tiling.  A block is 8 waves and owns one key chunk of one (layer, kv head).  The window queries
// (at most 512 rows) are staged once per block in LDS (row pitch 272 B so that the 16-byte operand
// reads of 8 lanes cover all 32 banks).  Every wave then works alone, without block barriers: it
// owns every 8th 32-key tile of the chunk, loads a tile straight from global memory into MFMA operand registers
// (the next tile is fetched while the current one is consumed), and walks all query tiles against
// it in a software pipeline (the MFMAs of query tile n+1 are issued before the vector-ALU work of
// tile n).  The MFMA operand layout is the same for A and B (lane = row or column index mod 32,
// 8 consecutive channels per lane, lanes 32..63 take the upper 8 of each 16-channel step), so the
// same registers serve both orientations:
//   pass A computes S^T = K Q^T: a lane holds one query column and 16 keys, so the running max/sum
//          of a row is lane-private; the waves of a block merge their statistics through LDS at the end;
//   pass B computes S = Q K^T: a lane holds one key column and 16 rows, so the column sum of a key
//          is lane-private adds plus one exchange between half-waves, and is complete inside the wave.
// Tiles that touch the causal window or the ragged end of the row run a separate instantiation, so
// the common tile carries no mask arithmetic.  Every key is owned by exactly one wave: no atomics,
// deterministic output.

#include <mutex>
#include <type_traits>

#include "kvp_internal.h"

namespace kvp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kWavesA = 8;                         // waves per block, pass A (256 VGPRs per wave)
constexpr int kWavesB = 8;                         // waves per block, pass B
constexpr int kPitch = 136;                        // bf16 elements per LDS row (272 B)
constexpr int kMaxRows = 512;                      // G*W limit (16 query tiles)
constexpr int kFoldChunks = 16;                    // up to this many key chunks pass B combines the chunk statistics itself
constexpr float kLog2e = 1.4426950408889634f;

struct ScoreArgs {
  const uint16_t* q;
  int64_t q_sl, q_st, q_sh;
  const uint16_t* k;
  int64_t k_sl, k_st, k_sh;
  int32_t T, W, G, Hkv, M, Mrows, nqt;      // nqt = query tiles in use (1 .. 16); Mrows = 32 * nqt
  int32_t chunk_keys, n_chunks;
  int32_t causal, force_window;
  int32_t fold_combine;                     // pass B combines the chunk statistics itself (few chunks: saves a launch)
  float scale2;                             // log2(e) / sqrt(D)
  float2* partial;                          // [L*Hkv][n_chunks][Mrows] (max, sum) in the base-2 domain
  float* bias;                              // [L*Hkv][Mrows]
  float* scores;                            // [L*Hkv][T]
};

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// row index inside a 32x32 accumulator tile held by vgpr v of this lane
__device__ __forceinline__ int acc_row(int lane, int v) { return (lane >> 5) * 4 + (v >> 2) * 8 + (v & 3); }

// 32 keys starting at tk0 as an MFMA operand, straight from global memory: lane holds key
// tk0 + lane%32, channels 16*ks + 8*(lane/32) .. +7.  Keys at or beyond T are zero.
__device__ __forceinline__ void load_key_tile(const ScoreArgs& a, const uint16_t* kbase, int tk0, int lane, uint4 out[8]) {
  const int t = tk0 + (lane & 31);
  if (t < a.T) {
    const uint16_t* row = kbase + static_cast<int64_t>(t) * a.k_st + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) out[ks] = *reinterpret_cast<const uint4*>(row + ks * 16);
  } else {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) out[ks] = make_uint4(0, 0, 0, 0);
  }
}

// bias_r = max_r + log2(sum_r) over all key chunks of (layer, head) lh; +inf for padding rows (they then contribute 0).
__device__ __forceinline__ float combined_bias(const ScoreArgs& a, int lh, int r) {
  if (r >= a.M) return INFINITY;
  const float2* part = a.partial + static_cast<int64_t>(lh) * a.n_chunks * a.Mrows + r;
  if (a.n_chunks <= kFoldChunks) {
    // all chunk statistics of the row requested at once (one memory latency instead of one per chunk)
    float2 p[kFoldChunks];
#pragma unroll
    for (int c = 0; c < kFoldChunks; ++c)
      p[c] = c < a.n_chunks ? part[static_cast<int64_t>(c) * a.Mrows] : make_float2(-INFINITY, 0.0f);
    float m = -INFINITY;
#pragma unroll
    for (int c = 0; c < kFoldChunks; ++c) m = fmaxf(m, p[c].x);
    float z = 0.0f;
#pragma unroll
    for (int c = 0; c < kFoldChunks; ++c)
      if (p[c].x != -INFINITY) z += p[c].y * __builtin_amdgcn_exp2f(p[c].x - m);
    return m + __builtin_amdgcn_logf(z);  // v_log_f32 is log2
  }
  float m = -INFINITY;
  for (int c = 0; c < a.n_chunks; ++c) m = fmaxf(m, part[static_cast<int64_t>(c) * a.Mrows].x);
  float z = 0.0f;
  for (int c = 0; c < a.n_chunks; ++c) {
    const float2 p = part[static_cast<int64_t>(c) * a.Mrows];
    if (p.x != -INFINITY) z += p.y * __builtin_amdgcn_exp2f(p.x - m);
  }
  return m + __builtin_amdgcn_logf(z);  // v_log_f32 is log2
}

template <int NQT, bool PASS_B>
__global__ __launch_bounds__((PASS_B ? kWavesB : kWavesA) * kWave, 2) void score_kernel(const ScoreArgs a) {
  constexpr int kWavesPerBlock = PASS_B ? kWavesB : kWavesA;
  constexpr int kThreads = kWavesPerBlock * kWave;
  __shared__ __attribute__((aligned(16))) uint16_t q_s[NQT * 32 * kPitch];
  __shared__ __attribute__((aligned(16))) float bias_s[PASS_B ? NQT * 32 : 4];
  __shared__ __attribute__((aligned(16))) int32_t wpos_s[NQT * 32];   // window offset r mod W of query row r (masked tiles)

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int lh = blockIdx.y;
  const int l = lh / a.Hkv, h = lh - l * a.Hkv;
  const int chunk = blockIdx.x;
  const uint16_t* kbase = a.k + static_cast<int64_t>(l) * a.k_sl + static_cast<int64_t>(h) * a.k_sh;
  const int win0 = a.T - a.W;  // first window position

  // this wave's first key tile is requested before anything else, so that its latency overlaps the prologue
  constexpr int kTileStride = 32 * kWavesPerBlock;
  const int t_begin = chunk * a.chunk_keys + wave * 32;
  const int t_end = min(a.T, (chunk + 1) * a.chunk_keys);   // chunk_keys is a multiple of kTileStride
  uint4 kop[8];
  if (t_begin < t_end) load_key_tile(a, kbase, t_begin, lane, kop);

  // ---- stage the window queries of this (layer, kv head): row r = u * W + w, zeros beyond M.  A thread's
  //      (at most NQT) pieces are all requested before the first one is stored ----
  {
    uint4 piece[NQT];
#pragma unroll
    for (int i = 0; i < NQT; ++i) {
      const int idx = static_cast<int>(threadIdx.x) + i * kThreads;
      const int r = idx >> 4, part = idx & 15;
      piece[i] = make_uint4(0, 0, 0, 0);
      if (r < a.M) {
        const int u = r / a.W, w = r - u * a.W;
        piece[i] = *reinterpret_cast<const uint4*>(a.q + static_cast<int64_t>(l) * a.q_sl + static_cast<int64_t>(w) * a.q_st +
                                                   static_cast<int64_t>(h * a.G + u) * a.q_sh + part * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < NQT; ++i) {
      const int idx = static_cast<int>(threadIdx.x) + i * kThreads;
      if (idx < a.Mrows * 16) *reinterpret_cast<uint4*>(q_s + (idx >> 4) * kPitch + (idx & 15) * 8) = piece[i];
    }
  }
  for (int r = threadIdx.x; r < a.Mrows; r += kThreads) {
    wpos_s[r] = r % a.W;
    // rows beyond M carry +inf: they contribute 2^-inf = 0
    if constexpr (PASS_B) bias_s[r] = a.fold_combine ? combined_bias(a, lh, r) : a.bias[static_cast<int64_t>(lh) * a.Mrows + r];
  }
  __syncthreads();

  // pass A state: running max / sum of this lane's query column (per query tile) over this lane's keys
  float run_m[PASS_B ? 1 : NQT], run_z[PASS_B ? 1 : NQT];
  if constexpr (!PASS_B) {
#pragma unroll
    for (int i = 0; i < NQT; ++i) {
      run_m[i] = -INFINITY;
      run_z[i] = 0.0f;
    }
  }

  auto q_operand = [&](int qt, bf16x8 out[8]) {
    const uint16_t* row = q_s + (qt * 32 + (lane & 31)) * kPitch + (lane >> 5) * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) out[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(row + ks * 16));
  };
  auto mfma_tile = [&](const uint4 kop[8], const bf16x8 qop[8]) {
    floatx16 acc = {0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if constexpr (PASS_B)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qop[ks], as_bf16x8(kop[ks]), acc, 0, 0, 0);  // rows = queries
      else
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kop[ks]), qop[ks], acc, 0, 0, 0);  // rows = keys
    }
    return acc;
  };

  // Vector-ALU work of one finished 32x32 tile `c` (query tile qt, keys tk0 .. tk0+31).
  auto consume = [&](auto masked_tag, floatx16& c, int qt, int tk0, float& col, float& m_run, float& z_run) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    if constexpr (!PASS_B) {
      // c[v] = raw dot product of key tk0 + acc_row(v) with query row qt*32 + lane%32
      if constexpr (MASKED) {
        const int qpos = win0 + wpos_s[qt * 32 + (lane & 31)];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int t = tk0 + acc_row(lane, v);
          if (t >= a.T || (a.causal && t > qpos)) c[v] = -INFINITY;
        }
      }
      float tmax = c[0];
#pragma unroll
      for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, c[v]);
      const float m_new = fmaxf(m_run, tmax * a.scale2);   // scale2 > 0: max commutes with it
      const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
      float z = z_run * __builtin_amdgcn_exp2f(m_run - m_safe);
#pragma unroll
      for (int v = 0; v < 16; ++v) z += __builtin_amdgcn_exp2f(fmaf(c[v], a.scale2, -m_safe));
      m_run = m_new;
      z_run = z;
    } else {
      // c[v] = raw dot product of query row qt*32 + acc_row(v) with key tk0 + lane%32
      float bias[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 b4 = *reinterpret_cast<const float4*>(bias_s + qt * 32 + g * 8 + (lane >> 5) * 4);
        bias[4 * g + 0] = b4.x; bias[4 * g + 1] = b4.y; bias[4 * g + 2] = b4.z; bias[4 * g + 3] = b4.w;
      }
      if constexpr (MASKED) {
        const int t = tk0 + (lane & 31);
        if (a.causal) {
#pragma unroll
          for (int g = 0; g < 4; ++g) {   // rows acc_row(lane, 4 g .. 4 g + 3), as for the bias
            const int4 w4 = *reinterpret_cast<const int4*>(wpos_s + qt * 32 + g * 8 + (lane >> 5) * 4);
            if (t > win0 + w4.x) c[4 * g + 0] = -INFINITY;
            if (t > win0 + w4.y) c[4 * g + 1] = -INFINITY;
            if (t > win0 + w4.z) c[4 * g + 2] = -INFINITY;
            if (t > win0 + w4.w) c[4 * g + 3] = -INFINITY;
          }
        }
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) col += __builtin_amdgcn_exp2f(fmaf(c[v], a.scale2, -bias[v]));
    }
  };

  // The LDS reads of a query tile's operands are issued one whole pipeline step before the MFMAs that
  // use them; a scheduling barrier keeps the compiler from sinking them back next to their use (where
  // every MFMA would wait out the LDS latency on its own).
  auto pin = [&]() { __builtin_amdgcn_sched_barrier(0); };

  // One 32-key tile against all query tiles as a software pipeline over the query tiles:
  //   step n:  LDS operand reads of tile n+2, then  MFMAs of tile n+1  |  vector-ALU work of tile n.
  // Query tiles in use.  Pass A is instantiated for the exact count (its per-tile statistics live in registers with
  // static indices), pass B for 1, 2, 4, 8 or 16 tiles of LDS with the count in use as a run-time value.
  const int nqt = PASS_B ? a.nqt : NQT;
  auto key_tile = [&](auto masked_tag, const uint4 kop[8], int tk0) {
    bf16x8 qop_a[8], qop_b[8];
    floatx16 acc_a, acc_b;
    float col = 0.0f, dummy_m = 0.0f, dummy_z = 0.0f;  // pass B: this lane's key column
    q_operand(0, qop_a);
    acc_a = mfma_tile(kop, qop_a);
    if (nqt > 1) q_operand(1, qop_b);
    // two pipeline steps: tile qt is finished in acc_a, the operands of tile qt+1 are in qop_b, tile qt+2 exists
    auto two_steps = [&](int qt, float& m0, float& z0, float& m1, float& z1) {
      q_operand(qt + 2, qop_a);
      pin();
      acc_b = mfma_tile(kop, qop_b);
      consume(masked_tag, acc_a, qt, tk0, col, m0, z0);
      pin();
      if (qt + 3 < nqt) q_operand(qt + 3, qop_b);
      pin();
      acc_a = mfma_tile(kop, qop_a);
      consume(masked_tag, acc_b, qt + 1, tk0, col, m1, z1);
      pin();
    };
    if constexpr (!PASS_B) {
      // fully unrolled: static register indices for the running statistics
#pragma unroll
      for (int qt = 0; qt + 2 < NQT; qt += 2) two_steps(qt, run_m[qt], run_z[qt], run_m[qt + 1], run_z[qt + 1]);
      if constexpr (NQT % 2 == 0) {
        acc_b = mfma_tile(kop, qop_b);
        consume(masked_tag, acc_a, NQT - 2, tk0, col, run_m[NQT - 2], run_z[NQT - 2]);
        pin();
        consume(masked_tag, acc_b, NQT - 1, tk0, col, run_m[NQT - 1], run_z[NQT - 1]);
      } else {
        consume(masked_tag, acc_a, NQT - 1, tk0, col, run_m[NQT - 1], run_z[NQT - 1]);
      }
    } else {
      // no per-tile state: a rolled loop keeps the register footprint independent of the tile count
      int qt = 0;
#pragma unroll 1
      for (; qt + 2 < nqt; qt += 2) two_steps(qt, dummy_m, dummy_z, dummy_m, dummy_z);
      if (qt + 1 < nqt) {
        acc_b = mfma_tile(kop, qop_b);
        consume(masked_tag, acc_a, qt, tk0, col, dummy_m, dummy_z);
        pin();
        consume(masked_tag, acc_b, qt + 1, tk0, col, dummy_m, dummy_z);
      } else {
        consume(masked_tag, acc_a, qt, tk0, col, dummy_m, dummy_z);
      }
      col += __shfl_xor(col, 32, 64);
      const int t = tk0 + lane;
      if (lane < 32 && t < a.T)
        a.scores[static_cast<int64_t>(lh) * a.T + t] = (a.force_window && t >= win0) ? INFINITY : col;
    }
  };

  // ---- this wave's key tiles: every kWavesPerBlock-th tile of the chunk, so that the few masked tiles at the
  //      end of a row (each costs more) are spread over the waves instead of all landing on the last one ----
  if (t_begin < t_end) {
    uint4 knext[8];
    for (int tk0 = t_begin; tk0 < t_end; tk0 += kTileStride) {
      const bool more = tk0 + kTileStride < t_end;
      if (more) load_key_tile(a, kbase, tk0 + kTileStride, lane, knext);
      const bool need_mask = (a.causal && tk0 + 32 > win0 + 1) || (tk0 + 32 > a.T);
      if (need_mask)
        key_tile(std::true_type{}, kop, tk0);
      else
        key_tile(std::false_type{}, kop, tk0);
      if (more) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) kop[ks] = knext[ks];
      }
    }
  }

  if constexpr (!PASS_B) {
    // merge the two half-waves (same query column, disjoint keys), then the 8 waves through LDS
    __syncthreads();                       // every wave is done reading q_s: reuse it as scratch
    float2* merge_s = reinterpret_cast<float2*>(q_s);   // [kWavesPerBlock][NQT*32]
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      const float m_o = __shfl_xor(run_m[qt], 32, 64);
      const float z_o = __shfl_xor(run_z[qt], 32, 64);
      const float m_new = fmaxf(run_m[qt], m_o);
      const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
      const float z = run_z[qt] * __builtin_amdgcn_exp2f(run_m[qt] - m_safe) + z_o * __builtin_amdgcn_exp2f(m_o - m_safe);
      if (lane < 32) merge_s[wave * (NQT * 32) + qt * 32 + lane] = make_float2(m_new, z);
    }
    __syncthreads();
    for (int r = threadIdx.x; r < a.Mrows; r += kThreads) {
      float m = -INFINITY;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) m = fmaxf(m, merge_s[w * (NQT * 32) + r].x);
      const float m_safe = (m == -INFINITY) ? 0.0f : m;
      float z = 0.0f;
#pragma unroll
      for (int w = 0; w < kWavesPerBlock; ++w) {
        const float2 p = merge_s[w * (NQT * 32) + r];
        z += p.y * __builtin_amdgcn_exp2f(p.x - m_safe);
      }
      a.partial[(static_cast<int64_t>(lh) * a.n_chunks + chunk) * a.Mrows + r] = make_float2(m, z);
    }
  }
}

// The same combination as its own launch, once per (layer, head), when there are many chunks.
__global__ void combine_kernel(const ScoreArgs a) {
  const int lh = blockIdx.x;
  for (int r = threadIdx.x; r < a.Mrows; r += blockDim.x) a.bias[static_cast<int64_t>(lh) * a.Mrows + r] = combined_bias(a, lh, r);
}

// Keys per block: large chunks amortize the query staging, small ones fill the chip.
int32_t choose_chunk_keys(int64_t n_lh, int64_t T) {
  int32_t kc = 4096;
  while (kc > 256 && n_lh * ceil_div(T, kc) < 512) kc /= 2;
  return kc;
}

struct ScorePlan {
  int32_t M, nqt, Mrows, chunk_keys, n_chunks;
  size_t partial_bytes, bias_bytes;
};

ScorePlan make_plan(int64_t L, int64_t Hkv, int64_t Hq, int64_t W, int64_t T) {
  ScorePlan p{};
  p.M = static_cast<int32_t>((Hq / Hkv) * W);
  p.nqt = (p.M + 31) / 32;              // query tiles in use (1 .. 16)
  p.Mrows = p.nqt * 32;
  p.chunk_keys = choose_chunk_keys(L * Hkv, T);
  p.n_chunks = static_cast<int32_t>(ceil_div(T, p.chunk_keys));
  p.partial_bytes = static_cast<size_t>(L * Hkv) * p.n_chunks * p.Mrows * sizeof(float2);
  p.partial_bytes = (p.partial_bytes + 255) / 256 * 256;
  p.bias_bytes = static_cast<size_t>(L * Hkv) * p.Mrows * sizeof(float);
  return p;
}

// Pass A is instantiated for every tile count 1 .. 16, pass B for 1, 2, 4, 8 and 16 tiles of LDS (M = 224 runs
// 7 tiles in the 8-tile instantiation).
template <int N>
void launch_pass_a(int nqt, dim3 grid, hipStream_t st, const ScoreArgs& a) {
  if constexpr (N <= 16) {
    if (nqt == N) score_kernel<N, false><<<grid, kWavesA * kWave, 0, st>>>(a);
    else launch_pass_a<N + 1>(nqt, grid, st, a);
  }
}

void launch_pass_b(int nqt, dim3 grid, hipStream_t st, const ScoreArgs& a) {
  constexpr int threads = kWavesB * kWave;
  if (nqt <= 1) score_kernel<1, true><<<grid, threads, 0, st>>>(a);
  else if (nqt <= 2) score_kernel<2, true><<<grid, threads, 0, st>>>(a);
  else if (nqt <= 4) score_kernel<4, true><<<grid, threads, 0, st>>>(a);
  else if (nqt <= 8) score_kernel<8, true><<<grid, threads, 0, st>>>(a);
  else score_kernel<16, true><<<grid, threads, 0, st>>>(a);
}

}  // namespace

// Shared with the configuration-evaluation path, which ranks tokens with the same scores.
int32_t score_tokens_impl(const kvp_view* q_win, const kvp_view* k, int32_t causal, int32_t force_window,
                          float* scores, void* ws, size_t ws_bytes, hipStream_t st) {
  int32_t rc = check_view(q_win);
  if (rc != KVP_OK) return rc;
  rc = check_view(k);
  if (rc != KVP_OK) return rc;
  if (!scores) return KVP_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(scores) & 3u) return KVP_ERR_ALIGN;
  const int64_t L = k->L, T = k->T, Hkv = k->H, Hq = q_win->H, W = q_win->T;
  if (q_win->L != L || Hq % Hkv != 0 || W > T || T >= (1ll << 30) || L * Hkv > 65535) return KVP_ERR_SHAPE;
  if ((Hq / Hkv) * W > kMaxRows) return KVP_ERR_UNSUPPORTED;
  const ScorePlan p = make_plan(L, Hkv, Hq, W, T);
  if (!ws || ws_bytes < p.partial_bytes + p.bias_bytes || (reinterpret_cast<uintptr_t>(ws) & 15u))
    return KVP_ERR_WORKSPACE;

  ScoreArgs a{};
  a.q = static_cast<const uint16_t*>(q_win->ptr);
  a.q_sl = q_win->stride_l; a.q_st = q_win->stride_t; a.q_sh = q_win->stride_h;
  a.k = static_cast<const uint16_t*>(k->ptr);
  a.k_sl = k->stride_l; a.k_st = k->stride_t; a.k_sh = k->stride_h;
  a.T = static_cast<int32_t>(T); a.W = static_cast<int32_t>(W); a.G = static_cast<int32_t>(Hq / Hkv);
  a.Hkv = static_cast<int32_t>(Hkv); a.M = p.M; a.Mrows = p.Mrows; a.nqt = p.nqt;
  a.chunk_keys = p.chunk_keys; a.n_chunks = p.n_chunks;
  a.causal = causal ? 1 : 0; a.force_window = force_window ? 1 : 0;
  a.scale2 = kLog2e / sqrtf(static_cast<float>(kHeadDim));
  a.partial = static_cast<float2*>(ws);
  a.bias = reinterpret_cast<float*>(static_cast<char*>(ws) + p.partial_bytes);
  a.scores = scores;

  const dim3 grid(static_cast<unsigned>(p.n_chunks), static_cast<unsigned>(L * Hkv));
  // With few chunks every pass-B block combines the chunk statistics of its (layer, head) itself (a few KiB of
  // reads from the cache): a call is two launches, which is what counts for small, launch-bound shapes.
  a.fold_combine = p.n_chunks <= kFoldChunks ? 1 : 0;
  launch_pass_a<1>(p.nqt, grid, st, a);
  if (!a.fold_combine) combine_kernel<<<dim3(static_cast<unsigned>(L * Hkv)), 256, 0, st>>>(a);
  launch_pass_b(p.nqt, grid, st, a);
  return launch_status();
}

}  // namespace kvp

extern "C" size_t kvp_score_workspace_bytes(int64_t L, int64_t Hkv, int64_t Hq, int64_t W, int64_t T) {
  if (L <= 0 || Hkv <= 0 || Hq <= 0 || W <= 0 || T <= 0 || Hq % Hkv != 0) return 0;
  const kvp::ScorePlan p = kvp::make_plan(L, Hkv, Hq, W, T);
  return p.partial_bytes + p.bias_bytes;
}

extern "C" int32_t kvp_score_tokens(const kvp_view* q_win, const kvp_view* k, int32_t causal, int32_t force_window,
                                    float* scores, void* ws, size_t ws_bytes, void* stream) {
  return kvp::score_tokens_impl(q_win, k, causal, force_window, scores, ws, ws_bytes, kvp::as_stream(stream));
}

// ---- kvp_score_tokens_static: the same kernels with their scratch in a device array of the library ----
//
// `scratch` is the host-side stand-in of the device array: host code never passes it to a kernel.  Its
// device address is looked up once per device (every GPU holds its own copy at its own address) and
// only that address is used from then on.
namespace kvp {
namespace {

static __device__ __align__(256) unsigned char scratch[KVP_SCORE_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on device i, once looked up

// Device address of the current device's copy of `scratch` (nullptr + rc on failure).  Allocates nothing.
int32_t static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVP_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return KVP_ERR_LAUNCH;
    }
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return KVP_OK;
}

}  // namespace
}  // namespace kvp

extern "C" int32_t kvp_score_tokens_static(const kvp_view* q_win, const kvp_view* k, int32_t causal,
                                           int32_t force_window, float* scores, void* stream) {
  using namespace kvp;
  // size check first (host arithmetic only), so that an oversized request fails before any lookup
  int32_t rc = check_view(q_win);
  if (rc != KVP_OK) return rc;
  rc = check_view(k);
  if (rc != KVP_OK) return rc;
  if (q_win->H % k->H != 0) return KVP_ERR_SHAPE;
  if (kvp_score_workspace_bytes(k->L, k->H, q_win->H, q_win->T, k->T) > KVP_SCORE_STATIC_SCRATCH_BYTES)
    return KVP_ERR_WORKSPACE;
  void* ptr = nullptr;
  rc = static_scratch(&ptr);
  if (rc != KVP_OK) return rc;
  // every word of the scratch that pass B and the combine step read is written earlier in the same call
  // (pass A stores the statistics of all chunks and all padded rows), so nothing has to be cleared
  return score_tokens_impl(q_win, k, causal, force_window, scores, ptr, KVP_SCORE_STATIC_SCRATCH_BYTES,
                           as_stream(stream));
}
