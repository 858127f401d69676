// kvp_score_tokens: attention-score token importance (the paper's snapkv baseline: cross attention
// between the tokens near the query and the earlier context; Evaluation, Baselines).
//
//   scores[l][h][t] = sum over the G*W window rows r of softmax_t(q_r . k_t / sqrt(D))
//
// Two passes over K, both with the query-window x key contraction on the bf16 MFMA
// (v_mfma_f32_32x32x16_bf16, fp32 accumulate), because a softmax row must be normalized before it
// can be summed into a column:
//   pass A  row statistics: running max and sum of exponentials per window row, per key chunk;
//   combine per-row bias b_r = max_r + log2(sum_r) over all chunks (tiny kernel);
//   pass B  column sums: scores[t] = sum_r 2^(s_rt - b_r).
// Logits are kept in the base-2 domain (s = q.k * log2(e)/sqrt(D)) so the exponential is one
// v_exp_f32.
//
// Tiling.  A block is 4 waves and owns one key chunk of one (layer, kv head).  The window rows are
// the stationary operand: each wave keeps its 32-row query tiles in registers for the whole chunk
// (up to 4 tiles = 128 VGPRs at G*W = 512).  K streams through LDS in 64-key stages shared by the
// four waves (row pitch 272 B so that the 16-byte operand reads of 8 lanes cover all 32 banks).
// The MFMA operand layout is the same for A and B (lane = row or column index mod 32, 8 consecutive
// channels per lane, lanes 32..63 take the upper 8 of each 16-channel step), so the same registers
// serve both orientations:
//   pass A computes S^T = K Q^T: a lane holds one query column and 16 keys, so the running max/sum
//          of a row is lane-private until one final exchange between the two half-waves;
//   pass B computes S = Q K^T: a lane holds one key column and 16 rows, so the column sum is
//          lane-private adds plus one exchange between half-waves and a 4-way sum across waves in LDS.
// Every key chunk is owned by exactly one block: no atomics, deterministic output.

#include <type_traits>

#include "kvp_internal.h"

namespace kvp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = 4;
constexpr int kStageKeys = 64;              // keys per LDS stage
constexpr int kPitch = 136;                 // bf16 elements per LDS row (272 B)
constexpr int kMaxRows = 512;               // G*W limit (16 query tiles)
constexpr float kLog2e = 1.4426950408889634f;

struct ScoreArgs {
  const uint16_t* q;
  int64_t q_sl, q_st, q_sh;
  const uint16_t* k;
  int64_t k_sl, k_st, k_sh;
  int32_t T, W, G, Hkv, M, Mpad;
  int32_t chunk_keys, n_chunks;
  int32_t causal, force_window;
  float scale2;                             // log2(e) / sqrt(D)
  float2* partial;                          // [L*Hkv][n_chunks][Mpad] (max, sum) in the base-2 domain
  float* bias;                              // [L*Hkv][Mpad]
  float* scores;                            // [L*Hkv][T]
};

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) {
  union { uint4 u; bf16x8 b; } c;
  c.u = v;
  return c.b;
}

// Query tile `qt` of (l, h) as an MFMA operand: lane holds row qt*32 + lane%32, channels
// 16*ks + 8*(lane/32) .. +7.  Rows at or beyond M are zero.
__device__ __forceinline__ void load_q_tile(const ScoreArgs& a, int l, int h, int qt, int lane, bf16x8 out[8]) {
  const int r = qt * 32 + (lane & 31);
  const int half = lane >> 5;
  if (r < a.M) {
    const int u = r / a.W, w = r - u * a.W;
    const uint16_t* row = a.q + static_cast<int64_t>(l) * a.q_sl + static_cast<int64_t>(w) * a.q_st +
                          static_cast<int64_t>(h * a.G + u) * a.q_sh;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) out[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(row + ks * 16 + half * 8));
  } else {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) out[ks] = as_bf16x8(make_uint4(0, 0, 0, 0));
  }
}

// A stage of 64 keys (zeros beyond T): global -> registers, then registers -> LDS, so that the next
// stage's loads are in flight while the current one is consumed.
constexpr int kStageVecs = (kStageKeys * 16) / kThreads;  // 16-byte pieces per thread and stage
__device__ __forceinline__ void fetch_stage(const ScoreArgs& a, const uint16_t* kbase, int t0, uint4 v[kStageVecs]) {
#pragma unroll
  for (int i = 0; i < kStageVecs; ++i) {
    const int idx = threadIdx.x + i * kThreads;
    const int key = idx >> 4, part = idx & 15;
    v[i] = make_uint4(0, 0, 0, 0);
    if (t0 + key < a.T) v[i] = load_stream16(kbase + static_cast<int64_t>(t0 + key) * a.k_st + part * 8);
  }
}
__device__ __forceinline__ void commit_stage(const uint4 v[kStageVecs], uint16_t* lds) {
#pragma unroll
  for (int i = 0; i < kStageVecs; ++i) {
    const int idx = threadIdx.x + i * kThreads;
    const int key = idx >> 4, part = idx & 15;
    *reinterpret_cast<uint4*>(lds + key * kPitch + part * 8) = v[i];
  }
}

__device__ __forceinline__ void load_k_operand(const uint16_t* lds, int sub, int lane, bf16x8 out[8]) {
  const uint16_t* row = lds + (sub * 32 + (lane & 31)) * kPitch + (lane >> 5) * 8;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) out[ks] = as_bf16x8(*reinterpret_cast<const uint4*>(row + ks * 16));
}

// row / column index inside a 32x32 accumulator tile held by vgpr v of this lane
__device__ __forceinline__ int acc_row(int lane, int v) { return (lane >> 5) * 4 + (v >> 2) * 8 + (v & 3); }

template <int QT, bool PASS_B>
__global__ __launch_bounds__(kThreads, QT >= 3 ? 1 : 2) void score_kernel(const ScoreArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t kstage[kStageKeys * kPitch];
  __shared__ __attribute__((aligned(16))) float bias_s[PASS_B ? kMaxRows : 4];
  __shared__ float colsum_s[PASS_B ? kWavesPerBlock * kStageKeys : 1];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int lh = blockIdx.y;
  const int l = lh / a.Hkv, h = lh - l * a.Hkv;
  const int chunk = blockIdx.x;
  const int t_begin = chunk * a.chunk_keys;
  const int t_end = min(a.T, t_begin + a.chunk_keys);
  const uint16_t* kbase = a.k + static_cast<int64_t>(l) * a.k_sl + static_cast<int64_t>(h) * a.k_sh;
  const int n_qt = a.Mpad / 32;
  const int win0 = a.T - a.W;  // first window position

  // this wave's query tiles: wave, wave + 4, ...
  bf16x8 q[QT][8];
#pragma unroll
  for (int i = 0; i < QT; ++i) {
    const int qt = wave + i * kWavesPerBlock;
    if (qt < n_qt) {
      load_q_tile(a, l, h, qt, lane, q[i]);
    } else {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) q[i][ks] = as_bf16x8(make_uint4(0, 0, 0, 0));
    }
  }

  if constexpr (PASS_B) {
    // rows beyond M (padding of the last tile, tiles a wave does not own) get +inf: they contribute 0
    for (int r = threadIdx.x; r < kMaxRows; r += kThreads)
      bias_s[r] = r < a.Mpad ? a.bias[static_cast<int64_t>(lh) * a.Mpad + r] : INFINITY;
  }

  // pass A state: running max / sum of this lane's query column over this lane's keys
  float run_m[QT], run_z[QT];
#pragma unroll
  for (int i = 0; i < QT; ++i) {
    run_m[i] = -INFINITY;
    run_z[i] = 0.0f;
  }
  // position of this lane's query row (pass A: column lane%32 of tile i)
  int qpos[QT];
#pragma unroll
  for (int i = 0; i < QT; ++i) {
    const int r = (wave + i * kWavesPerBlock) * 32 + (lane & 31);
    qpos[i] = win0 + (r % a.W);
  }

  // One 64-key stage.  The tiles (key sub-tile x query tile) are walked in a software pipeline: the
  // eight MFMAs of tile n+1 are issued before the vector-ALU work of tile n, so a wave never waits
  // for a matrix result.  MASKED stages (the causal window, the ragged end of the row) are a
  // separate instantiation so that the common stage carries no mask arithmetic.
  auto mfma_tile = [&](const bf16x8 kop[8], const bf16x8 qop[8]) {
    floatx16 acc = {0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if constexpr (PASS_B)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qop[ks], kop[ks], acc, 0, 0, 0);  // rows = queries, lane = key
      else
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[ks], qop[ks], acc, 0, 0, 0);  // rows = keys, lane = query
    }
    return acc;
  };

  auto stage = [&](auto masked_tag, int t0) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    constexpr int NT = (kStageKeys / 32) * QT;
    bf16x8 kop[8];
    floatx16 acc[2];
    load_k_operand(kstage, 0, lane, kop);
    acc[0] = mfma_tile(kop, q[0]);
    float col = 0.0f;  // pass B: this lane's key column
#pragma unroll
    for (int tt = 0; tt < NT; ++tt) {
      const int sub = tt / QT, i = tt % QT;
      if (tt + 1 < NT) {
        if ((tt + 1) % QT == 0) load_k_operand(kstage, (tt + 1) / QT, lane, kop);
        acc[(tt + 1) & 1] = mfma_tile(kop, q[(tt + 1) % QT]);
      }
      floatx16& c = acc[tt & 1];
      const int tk0 = t0 + sub * 32;
      const int qt = wave + i * kWavesPerBlock;
      if constexpr (!PASS_B) {
        // c[v] = raw dot product of key tk0 + acc_row(v) with query column lane%32
        if constexpr (MASKED) {
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int t = tk0 + acc_row(lane, v);
            if (t >= a.T || (a.causal && t > qpos[i])) c[v] = -INFINITY;
          }
        }
        float tmax = c[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, c[v]);
        const float m_new = fmaxf(run_m[i], tmax * a.scale2);   // scale2 > 0: max commutes with it
        const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
        float z = run_z[i] * __builtin_amdgcn_exp2f(run_m[i] - m_safe);
#pragma unroll
        for (int v = 0; v < 16; ++v) z += __builtin_amdgcn_exp2f(fmaf(c[v], a.scale2, -m_safe));
        run_m[i] = m_new;
        run_z[i] = z;
      } else {
        // c[v] = raw dot product of query row qt*32 + acc_row(v) with key column tk0 + lane%32
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
            for (int v = 0; v < 16; ++v) {
              const int r = qt * 32 + acc_row(lane, v);
              if (t > win0 + (r % a.W)) c[v] = -INFINITY;
            }
          }
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) col += __builtin_amdgcn_exp2f(fmaf(c[v], a.scale2, -bias[v]));
        if (i == QT - 1) {
          col += __shfl_xor(col, 32, 64);
          if (lane < 32) colsum_s[wave * kStageKeys + sub * 32 + lane] = col;
          col = 0.0f;
        }
      }
    }
  };

  uint4 pre[kStageVecs];
  fetch_stage(a, kbase, t_begin, pre);
  for (int t0 = t_begin; t0 < t_end; t0 += kStageKeys) {
    __syncthreads();  // previous stage fully consumed
    commit_stage(pre, kstage);
    __syncthreads();
    if (t0 + kStageKeys < t_end) fetch_stage(a, kbase, t0 + kStageKeys, pre);
    const bool need_mask = (a.causal && t0 + kStageKeys > win0 + 1) || (t0 + kStageKeys > a.T);
    if (need_mask)
      stage(std::true_type{}, t0);
    else
      stage(std::false_type{}, t0);

    if constexpr (PASS_B) {
      __syncthreads();
      if (threadIdx.x < kStageKeys) {
        const int t = t0 + threadIdx.x;
        if (t < t_end) {
          float sum = 0.0f;
#pragma unroll
          for (int w = 0; w < kWavesPerBlock; ++w) sum += colsum_s[w * kStageKeys + threadIdx.x];
          if (a.force_window && t >= win0) sum = INFINITY;
          a.scores[static_cast<int64_t>(lh) * a.T + t] = sum;
        }
      }
    }
  }

  if constexpr (!PASS_B) {
#pragma unroll
    for (int i = 0; i < QT; ++i) {
      const int qt = wave + i * kWavesPerBlock;
      if (qt >= n_qt) continue;
      // merge the two half-waves (same query column, disjoint keys)
      const float m_o = __shfl_xor(run_m[i], 32, 64);
      const float z_o = __shfl_xor(run_z[i], 32, 64);
      const float m_new = fmaxf(run_m[i], m_o);
      const float m_safe = (m_new == -INFINITY) ? 0.0f : m_new;
      const float z = run_z[i] * __builtin_amdgcn_exp2f(run_m[i] - m_safe) + z_o * __builtin_amdgcn_exp2f(m_o - m_safe);
      if (lane < 32) {
        const int r = qt * 32 + lane;
        a.partial[(static_cast<int64_t>(lh) * a.n_chunks + chunk) * a.Mpad + r] = make_float2(m_new, z);
      }
    }
  }
}

// bias_r = max_r + log2(sum_r) over all key chunks; +inf for padding rows (they then contribute 0).
__global__ void combine_kernel(const ScoreArgs a) {
  const int lh = blockIdx.x;
  for (int r = threadIdx.x; r < a.Mpad; r += blockDim.x) {
    float b = INFINITY;
    if (r < a.M) {
      float m = -INFINITY;
      for (int c = 0; c < a.n_chunks; ++c)
        m = fmaxf(m, a.partial[(static_cast<int64_t>(lh) * a.n_chunks + c) * a.Mpad + r].x);
      float z = 0.0f;
      for (int c = 0; c < a.n_chunks; ++c) {
        const float2 p = a.partial[(static_cast<int64_t>(lh) * a.n_chunks + c) * a.Mpad + r];
        if (p.x != -INFINITY) z += p.y * __builtin_amdgcn_exp2f(p.x - m);
      }
      b = m + __builtin_amdgcn_logf(z);  // v_log_f32 is log2
    }
    a.bias[static_cast<int64_t>(lh) * a.Mpad + r] = b;
  }
}

// Keys per block: large chunks amortize the stationary query tiles, small ones fill the chip.
int32_t choose_chunk_keys(int64_t n_lh, int64_t T) {
  int32_t kc = 2048;
  while (kc > 256 && n_lh * ceil_div(T, kc) < 1024) kc /= 2;
  return kc;
}

struct ScorePlan {
  int32_t M, Mpad, chunk_keys, n_chunks;
  size_t partial_bytes, bias_bytes;
};

ScorePlan make_plan(int64_t L, int64_t Hkv, int64_t Hq, int64_t W, int64_t T) {
  ScorePlan p{};
  p.M = static_cast<int32_t>((Hq / Hkv) * W);
  p.Mpad = (p.M + 31) / 32 * 32;
  p.chunk_keys = choose_chunk_keys(L * Hkv, T);
  p.n_chunks = static_cast<int32_t>(ceil_div(T, p.chunk_keys));
  p.partial_bytes = static_cast<size_t>(L * Hkv) * p.n_chunks * p.Mpad * sizeof(float2);
  p.partial_bytes = (p.partial_bytes + 255) / 256 * 256;
  p.bias_bytes = static_cast<size_t>(L * Hkv) * p.Mpad * sizeof(float);
  return p;
}

template <bool PASS_B>
void launch_pass(int qt_per_wave, dim3 grid, hipStream_t st, const ScoreArgs& a) {
  switch (qt_per_wave) {
    case 1: score_kernel<1, PASS_B><<<grid, kThreads, 0, st>>>(a); break;
    case 2: score_kernel<2, PASS_B><<<grid, kThreads, 0, st>>>(a); break;
    case 3: score_kernel<3, PASS_B><<<grid, kThreads, 0, st>>>(a); break;
    default: score_kernel<4, PASS_B><<<grid, kThreads, 0, st>>>(a); break;
  }
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
  a.Hkv = static_cast<int32_t>(Hkv); a.M = p.M; a.Mpad = p.Mpad;
  a.chunk_keys = p.chunk_keys; a.n_chunks = p.n_chunks;
  a.causal = causal ? 1 : 0; a.force_window = force_window ? 1 : 0;
  a.scale2 = kLog2e / sqrtf(static_cast<float>(kHeadDim));
  a.partial = static_cast<float2*>(ws);
  a.bias = reinterpret_cast<float*>(static_cast<char*>(ws) + p.partial_bytes);
  a.scores = scores;

  const int qt_per_wave = static_cast<int>(ceil_div(p.Mpad / 32, kWavesPerBlock));
  const dim3 grid(static_cast<unsigned>(p.n_chunks), static_cast<unsigned>(L * Hkv));
  launch_pass<false>(qt_per_wave, grid, st, a);
  combine_kernel<<<dim3(static_cast<unsigned>(L * Hkv)), 256, 0, st>>>(a);
  launch_pass<true>(qt_per_wave, grid, st, a);
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
