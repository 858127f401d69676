// CPU oracle for the KV-cache compress / decompress hot path of EvicPress
// (arxiv 2512.14946).
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
// single-threaded, obviously-correct definition of what each operation
// computes.  Only the tests, the smoke check and the benchmark's cpu_baseline
// leg may call it.  It shares no code, header, table or helper with the HIP
// library, and neither includes the other.
//
// The paper names the operations but gives no formula for the quantization
// category (Background, KV cache compression: entries stored at a lower bit
// width; Related work: uniform quantization) and one sentence for the
// attention-score token dropping (Evaluation, Baselines, snapkv: the earlier
// context is scored by the attention it gets from the tokens next to the query,
// and the lowest-scored tokens go).  The concrete arithmetic below is therefore a
// stated reading (symmetric abs-max scaling, IEEE binary32 division,
// round-half-to-even, lowest-index tie-break, keep count ceil(ratio*T)); each
// reading is stated again at the function it governs.
//
// Parity status:
//   oracle_quantize / oracle_dequantize_paged / oracle_select_topk: pinned by
//     hand-exact examples, exact rational arithmetic, invariants and brute
//     force (tests/test_oracle_*.py).
//   oracle_quantize_asym / oracle_dequantize_paged_asym: pinned the same way (hand-exact
//     examples, exact rational arithmetic, invariants).
//   oracle_quantize_channel / oracle_dequantize_paged_channel: hand-exact examples, reduction to the
//     per-token quantizers on a transposed tile, exact rational arithmetic, invariants.
//   oracle_dequantize_paged_scatter: composition with the compact dequantizers plus a brute-force
//     address check.  oracle_smooth_scores: library pooling, closed forms, brute force.
//   oracle_score_keys (knorm, keydiff): pinned by closed forms (3-4-5 norms, identical / orthogonal /
//     antipodal keys), scale invariance and a library float64 normalize + matmul.
//   oracle_score_tokens / oracle_eval_configs: pinned by closed forms (zero
//     queries, one dominant key), the row-sum invariant, a library float64
//     softmax / einsum recomputation on random inputs of small shape and a
//     brute force written from the formulas (tests/test_oracle_select_score.py,
//     tests/test_oracle_eval.py).  The paper prints no numeric value of either
//     quantity, so there is no golden figure of its own to compare with.
//
// Precision: binary32 exactly where results are graded bit-exactly (scales,
// codes, dequantized bf16), double where results are graded to a tolerance
// (token scores, quality-loss proxy).
//
// Build: g++ -O2 -std=c++17 -fno-fast-math -ffp-contract=off -shared -fPIC

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

namespace {

// bf16 is the upper half of a binary32: widening is exact.
inline float bf16_to_f32(uint16_t h) {
  uint32_t u = static_cast<uint32_t>(h) << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return f;
}

// binary32 -> bf16, round to nearest, ties to even.  Inputs are finite by
// contract; a NaN is kept a NaN (quiet bit forced) so nothing silently turns
// into infinity.
inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  std::memcpy(&u, &f, sizeof u);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
  const uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  return static_cast<uint16_t>(u >> 16);
}

inline int qmax_of(int bits) { return (1 << (bits - 1)) - 1; }  // 127, 7, 1

inline bool quant_args_ok(int bits, int group, int64_t D) {
  if (bits != 8 && bits != 4 && bits != 2) return false;
  if (group <= 0 || D <= 0 || D % group != 0) return false;
  if ((D * bits) % 8 != 0) return false;
  return true;
}

// One row (one token of one head of one layer): D bf16 values -> D*bits/8
// packed bytes and D/group binary32 scales.
//
// Per group of `group` consecutive channels:
//   amax  = max |x|                       (exact)
//   scale = amax / qmax                   (one binary32 division)
//   q     = clamp(rint(x / scale), -qmax, qmax), 0 when scale == 0
//           (one binary32 division per element, rint = half-to-even)
// Packing is little-endian inside a byte, two's complement truncated to
// `bits` bits, bytes in channel order.
void quantize_row(const uint16_t* x, int64_t D, int bits, int group, uint8_t* codes, float* scales) {
  const int qmax = qmax_of(bits);
  const int per_byte = 8 / bits;
  const uint32_t field_mask = (1u << bits) - 1u;
  std::vector<int> q(static_cast<size_t>(D));
  for (int64_t g0 = 0; g0 < D; g0 += group) {
    float amax = 0.0f;
    for (int64_t c = 0; c < group; ++c) amax = std::max(amax, std::fabs(bf16_to_f32(x[g0 + c])));
    const float scale = amax / static_cast<float>(qmax);
    scales[g0 / group] = scale;
    for (int64_t c = 0; c < group; ++c) {
      int v = 0;
      if (scale != 0.0f) {
        const float r = std::rint(bf16_to_f32(x[g0 + c]) / scale);
        v = static_cast<int>(r);
        v = std::min(qmax, std::max(-qmax, v));
      }
      q[static_cast<size_t>(g0 + c)] = v;
    }
  }
  for (int64_t m = 0; m < D / per_byte; ++m) {
    uint32_t byte = 0;
    for (int i = 0; i < per_byte; ++i)
      byte |= (static_cast<uint32_t>(q[static_cast<size_t>(m * per_byte + i)]) & field_mask) << (bits * i);
    codes[m] = static_cast<uint8_t>(byte);
  }
}

// The inverse direction for one row: unpack, sign-extend, one binary32
// multiply by the group's scale, round to bf16 (nearest even).
void dequantize_row(const uint8_t* codes, const float* scales, int64_t D, int bits, int group, uint16_t* out) {
  const int per_byte = 8 / bits;
  const uint32_t field_mask = (1u << bits) - 1u;
  const int sign_bit = 1 << (bits - 1);
  for (int64_t c = 0; c < D; ++c) {
    const uint32_t byte = codes[c / per_byte];
    int v = static_cast<int>((byte >> (bits * (c % per_byte))) & field_mask);
    if (v & sign_bit) v -= (1 << bits);
    const float y = static_cast<float>(v) * scales[c / group];
    out[c] = f32_to_bf16_rne(y);
  }
}

// Asymmetric (min / scale) variant of the row quantizer: every one of the 2^bits levels is used,
// which matters most at 2 bits (the uniform quantization with zero point that the paper's Related
// work cites as the uniform method).  Per group:
//   mn = min x, mx = max x                      (exact)
//   scale = fl32(fl32(mx - mn) / (2^bits - 1))  (one binary32 subtraction, one division)
//   q = clamp(rint(fl32(fl32(x - mn) / scale)), 0, 2^bits - 1), 0 when scale == 0   (unsigned fields)
// and back: y = bf16_rne(fl32(fl32(q * scale) + mn))   (a multiply and an add, not fused).
void quantize_row_asym(const uint16_t* x, int64_t D, int bits, int group, uint8_t* codes, float* scales, float* mins) {
  const int levels = (1 << bits) - 1;
  const int per_byte = 8 / bits;
  std::vector<int> q(static_cast<size_t>(D));
  for (int64_t g0 = 0; g0 < D; g0 += group) {
    float mn = bf16_to_f32(x[g0]), mx = mn;
    for (int64_t c = 1; c < group; ++c) {
      const float v = bf16_to_f32(x[g0 + c]);
      mn = std::min(mn, v);
      mx = std::max(mx, v);
    }
    if (mn == 0.0f) mn = 0.0f;  // -0 and +0 compare equal: a zero extreme is taken as +0, so that the
    if (mx == 0.0f) mx = 0.0f;  // stored minimum and a zero range (hence scale) have unique bytes
    const float range = mx - mn;
    const float scale = range / static_cast<float>(levels);
    scales[g0 / group] = scale;
    mins[g0 / group] = mn;
    for (int64_t c = 0; c < group; ++c) {
      int v = 0;
      if (scale != 0.0f) {
        const float d = bf16_to_f32(x[g0 + c]) - mn;
        v = static_cast<int>(std::rint(d / scale));
        v = std::min(levels, std::max(0, v));
      }
      q[static_cast<size_t>(g0 + c)] = v;
    }
  }
  for (int64_t m = 0; m < D / per_byte; ++m) {
    uint32_t byte = 0;
    for (int i = 0; i < per_byte; ++i) byte |= static_cast<uint32_t>(q[static_cast<size_t>(m * per_byte + i)]) << (bits * i);
    codes[m] = static_cast<uint8_t>(byte);
  }
}

void dequantize_row_asym(const uint8_t* codes, const float* scales, const float* mins, int64_t D, int bits, int group,
                         uint16_t* out) {
  const int per_byte = 8 / bits;
  const uint32_t field_mask = (1u << bits) - 1u;
  for (int64_t c = 0; c < D; ++c) {
    const uint32_t v = (codes[c / per_byte] >> (bits * (c % per_byte))) & field_mask;
    const float prod = static_cast<float>(v) * scales[c / group];
    const float y = prod + mins[c / group];
    out[c] = f32_to_bf16_rne(y);
  }
}

struct View {  // strided bf16 tensor [L][T][H][D], innermost D contiguous
  const uint16_t* p;
  int64_t sl, st, sh;
  const uint16_t* row(int64_t l, int64_t t, int64_t h) const { return p + l * sl + t * st + h * sh; }
};

// Window-query x key attention probabilities of one (layer, kv head):
// P[u][w][t] for the G query heads u of kv head h and the W window rows, in
// double.  Window row w sits at absolute position T - W + w.  `allowed` (or
// null = all tokens) restricts the softmax to a key subset.  Keys that the
// causal mask or the subset removes get probability 0.
void window_probs(const View& q, const View& k, int64_t l, int64_t h, int64_t G, int64_t W, int64_t T,
                  int64_t D, bool causal, const uint8_t* allowed, std::vector<double>& P) {
  const double inv_sqrt_d = 1.0 / std::sqrt(static_cast<double>(D));
  P.assign(static_cast<size_t>(G * W * T), 0.0);
  std::vector<double> s(static_cast<size_t>(T));
  for (int64_t u = 0; u < G; ++u) {
    for (int64_t w = 0; w < W; ++w) {
      const uint16_t* qr = q.row(l, w, h * G + u);
      const int64_t pos = T - W + w;
      double mx = -std::numeric_limits<double>::infinity();
      for (int64_t t = 0; t < T; ++t) {
        const bool masked = (causal && t > pos) || (allowed && !allowed[t]);
        if (masked) {
          s[static_cast<size_t>(t)] = -std::numeric_limits<double>::infinity();
          continue;
        }
        const uint16_t* kr = k.row(l, t, h);
        double dot = 0.0;
        for (int64_t c = 0; c < D; ++c)
          dot += static_cast<double>(bf16_to_f32(qr[c])) * static_cast<double>(bf16_to_f32(kr[c]));
        s[static_cast<size_t>(t)] = dot * inv_sqrt_d;
        mx = std::max(mx, s[static_cast<size_t>(t)]);
      }
      double* prow = &P[static_cast<size_t>((u * W + w) * T)];
      if (!(mx > -std::numeric_limits<double>::infinity())) continue;  // every key masked: row of zeros
      double z = 0.0;
      for (int64_t t = 0; t < T; ++t) {
        const double e = std::exp(s[static_cast<size_t>(t)] - mx);  // exp(-inf) = 0
        prow[t] = e;
        z += e;
      }
      for (int64_t t = 0; t < T; ++t) prow[t] /= z;
    }
  }
}

void scores_from_probs(const std::vector<double>& P, int64_t GW, int64_t T, int64_t W, bool force_window,
                       float* out) {
  for (int64_t t = 0; t < T; ++t) {
    double acc = 0.0;
    for (int64_t r = 0; r < GW; ++r) acc += P[static_cast<size_t>(r * T + t)];
    out[t] = static_cast<float>(acc);
  }
  if (force_window)
    for (int64_t t = std::max<int64_t>(0, T - W); t < T; ++t) out[t] = std::numeric_limits<float>::infinity();
}

// The k largest scores of one row: stable sort by score descending (equal
// scores stay in ascending index order, so the lowest index wins a tie), take
// k, emit ascending.
void topk_row(const float* s, int64_t T, int64_t k, int32_t* out) {
  std::vector<int32_t> order(static_cast<size_t>(T));
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [s](int32_t a, int32_t b) { return s[a] > s[b]; });
  std::vector<int32_t> kept(order.begin(), order.begin() + k);
  std::sort(kept.begin(), kept.end());
  std::copy(kept.begin(), kept.end(), out);
}

}  // namespace

extern "C" {

// Group-wise quantization of a strided bf16 plane x[L][T][H][D] (strides in
// elements) into codes[L][Tp][H][D*bits/8] and scales[L][Tp][H][D/group].
// With keep_idx (host, [L][H][k], ascending) slot i of head h holds token
// keep_idx[l][h][i] and the slot count is k; otherwise slot i is token i and
// the slot count is T.  Slots from the slot count up to Tp are zero codes and
// zero scales.  Returns 0, or -1 on a bad argument.
int oracle_quantize(const uint16_t* x, int64_t L, int64_t T, int64_t H, int64_t D, int64_t stride_l,
                    int64_t stride_t, int64_t stride_h, const int32_t* keep_idx, int64_t k, int bits,
                    int group, int64_t Tp, uint8_t* codes, float* scales) {
  if (!x || !codes || !scales || !quant_args_ok(bits, group, D)) return -1;
  const int64_t n_slots = keep_idx ? k : T;
  if (n_slots < 0 || n_slots > Tp || L < 0 || T < 0 || H <= 0) return -1;
  const int64_t cb = D * bits / 8, ns = D / group;
  const View v{x, stride_l, stride_t, stride_h};
  for (int64_t l = 0; l < L; ++l)
    for (int64_t i = 0; i < Tp; ++i)
      for (int64_t h = 0; h < H; ++h) {
        uint8_t* c = codes + ((l * Tp + i) * H + h) * cb;
        float* s = scales + ((l * Tp + i) * H + h) * ns;
        if (i >= n_slots) {
          std::memset(c, 0, static_cast<size_t>(cb));
          for (int64_t j = 0; j < ns; ++j) s[j] = 0.0f;
          continue;
        }
        int64_t t = i;
        if (keep_idx) {
          t = keep_idx[(l * H + h) * k + i];
          if (t < 0 || t >= T) return -1;
        }
        quantize_row(v.row(l, t, h), D, bits, group, c, s);
      }
  return 0;
}

// Same as oracle_quantize, the source being a paged pool
// pool[L][num_blocks][bs][H][D] (layer stride pool_stride_l elements) read
// through block_table[ceil(T/bs)]: token t lives in physical block
// block_table[t / bs] at slot t % bs.
int oracle_quantize_paged_src(const uint16_t* pool, const int32_t* block_table, int64_t L, int64_t num_blocks,
                              int64_t bs, int64_t H, int64_t D, int64_t T, int64_t pool_stride_l,
                              const int32_t* keep_idx, int64_t k, int bits, int group, int64_t Tp,
                              uint8_t* codes, float* scales) {
  if (!pool || !block_table || !codes || !scales || !quant_args_ok(bits, group, D) || bs <= 0) return -1;
  const int64_t n_slots = keep_idx ? k : T;
  if (n_slots < 0 || n_slots > Tp) return -1;
  const int64_t cb = D * bits / 8, ns = D / group;
  for (int64_t l = 0; l < L; ++l)
    for (int64_t i = 0; i < Tp; ++i)
      for (int64_t h = 0; h < H; ++h) {
        uint8_t* c = codes + ((l * Tp + i) * H + h) * cb;
        float* s = scales + ((l * Tp + i) * H + h) * ns;
        if (i >= n_slots) {
          std::memset(c, 0, static_cast<size_t>(cb));
          for (int64_t j = 0; j < ns; ++j) s[j] = 0.0f;
          continue;
        }
        int64_t t = i;
        if (keep_idx) {
          t = keep_idx[(l * H + h) * k + i];
          if (t < 0 || t >= T) return -1;
        }
        const int64_t blk = block_table[t / bs];
        if (blk < 0 || blk >= num_blocks) return -1;
        const uint16_t* row = pool + l * pool_stride_l + ((blk * bs + t % bs) * H + h) * D;
        quantize_row(row, D, bits, group, c, s);
      }
  return 0;
}

// Dequantize codes/scales (layout as written by oracle_quantize) into the
// paged bf16 pool: pool[l][block_table[t/bs]][t%bs][h][:] for t < T.  Page
// slots at or beyond T and pages the table does not name are left untouched.
int oracle_dequantize_paged(const uint8_t* codes, const float* scales, int bits, int group, int64_t L,
                            int64_t T, int64_t Tp, int64_t H, int64_t D, const int32_t* block_table,
                            int64_t num_blocks, int64_t bs, uint16_t* pool, int64_t pool_stride_l) {
  if (!codes || !scales || !block_table || !pool || !quant_args_ok(bits, group, D) || bs <= 0 || T > Tp)
    return -1;
  const int64_t cb = D * bits / 8, ns = D / group;
  for (int64_t l = 0; l < L; ++l)
    for (int64_t t = 0; t < T; ++t) {
      const int64_t blk = block_table[t / bs];
      if (blk < 0 || blk >= num_blocks) return -1;
      for (int64_t h = 0; h < H; ++h) {
        const uint8_t* c = codes + ((l * Tp + t) * H + h) * cb;
        const float* s = scales + ((l * Tp + t) * H + h) * ns;
        uint16_t* row = pool + l * pool_stride_l + ((blk * bs + t % bs) * H + h) * D;
        dequantize_row(c, s, D, bits, group, row);
      }
    }
  return 0;
}

// Asymmetric variants: same layouts as oracle_quantize / oracle_dequantize_paged plus
// mins[L][Tp][H][D/group]; codes are unsigned fields.  Flat strided source, optional keep list.
int oracle_quantize_asym(const uint16_t* x, int64_t L, int64_t T, int64_t H, int64_t D, int64_t stride_l,
                         int64_t stride_t, int64_t stride_h, const int32_t* keep_idx, int64_t k, int bits, int group,
                         int64_t Tp, uint8_t* codes, float* scales, float* mins) {
  if (!x || !codes || !scales || !mins || !quant_args_ok(bits, group, D)) return -1;
  const int64_t n_slots = keep_idx ? k : T;
  if (n_slots < 0 || n_slots > Tp || L < 0 || T < 0 || H <= 0) return -1;
  const int64_t cb = D * bits / 8, ns = D / group;
  const View v{x, stride_l, stride_t, stride_h};
  for (int64_t l = 0; l < L; ++l)
    for (int64_t i = 0; i < Tp; ++i)
      for (int64_t h = 0; h < H; ++h) {
        uint8_t* c = codes + ((l * Tp + i) * H + h) * cb;
        float* s = scales + ((l * Tp + i) * H + h) * ns;
        float* m = mins + ((l * Tp + i) * H + h) * ns;
        if (i >= n_slots) {
          std::memset(c, 0, static_cast<size_t>(cb));
          for (int64_t j = 0; j < ns; ++j) s[j] = m[j] = 0.0f;
          continue;
        }
        int64_t t = i;
        if (keep_idx) {
          t = keep_idx[(l * H + h) * k + i];
          if (t < 0 || t >= T) return -1;
        }
        quantize_row_asym(v.row(l, t, h), D, bits, group, c, s, m);
      }
  return 0;
}

int oracle_dequantize_paged_asym(const uint8_t* codes, const float* scales, const float* mins, int bits, int group,
                                 int64_t L, int64_t T, int64_t Tp, int64_t H, int64_t D, const int32_t* block_table,
                                 int64_t num_blocks, int64_t bs, uint16_t* pool, int64_t pool_stride_l) {
  if (!codes || !scales || !mins || !block_table || !pool || !quant_args_ok(bits, group, D) || bs <= 0 || T > Tp)
    return -1;
  const int64_t cb = D * bits / 8, ns = D / group;
  for (int64_t l = 0; l < L; ++l)
    for (int64_t t = 0; t < T; ++t) {
      const int64_t blk = block_table[t / bs];
      if (blk < 0 || blk >= num_blocks) return -1;
      for (int64_t h = 0; h < H; ++h) {
        const int64_t r = (l * Tp + t) * H + h;
        uint16_t* row = pool + l * pool_stride_l + ((blk * bs + t % bs) * H + h) * D;
        dequantize_row_asym(codes + r * cb, scales + r * ns, mins + r * ns, D, bits, group, row);
      }
    }
  return 0;
}

// Per-channel grouping (the KIVI-style key quantizer the paper's Related work names): a group is
// `group` consecutive token slots of ONE channel of one head, instead of `group` channels of one
// token.  Slots are tokens, or kept tokens when a keep list is given; the last group of a plane
// holds the n_slots % group remaining slots and padding slots never enter a minimum or maximum.
// The per-element formulas are those of quantize_row (asym == 0) and quantize_row_asym (asym != 0).
//   codes  [L][Tp][H][D*bits/8]   (same plane as the per-token codec)
//   scales [L][ceil(Tp/group)][H][D], mins likewise (asym only)
int oracle_quantize_channel(const uint16_t* x, int64_t L, int64_t T, int64_t H, int64_t D, int64_t stride_l,
                            int64_t stride_t, int64_t stride_h, const int32_t* keep_idx, int64_t k, int bits,
                            int group, int asym, int64_t Tp, uint8_t* codes, float* scales, float* mins) {
  if (!x || !codes || !scales || (asym && !mins)) return -1;
  if ((bits != 8 && bits != 4 && bits != 2) || group <= 0 || D <= 0 || (D * bits) % 8 != 0) return -1;
  const int64_t n_slots = keep_idx ? k : T;
  if (n_slots < 0 || n_slots > Tp || L < 0 || T < 0 || H <= 0) return -1;
  const int64_t cb = D * bits / 8, n_groups = (Tp + group - 1) / group;
  const int per_byte = 8 / bits;
  const uint32_t field_mask = (1u << bits) - 1u;
  const int qmax = qmax_of(bits), levels = (1 << bits) - 1;
  const View v{x, stride_l, stride_t, stride_h};
  std::memset(codes, 0, static_cast<size_t>(L * Tp * H * cb));
  for (int64_t l = 0; l < L; ++l)
    for (int64_t g = 0; g < n_groups; ++g)
      for (int64_t h = 0; h < H; ++h)
        for (int64_t c = 0; c < D; ++c) {
          const int64_t i0 = g * group, i1 = std::min<int64_t>(i0 + group, n_slots);
          std::vector<float> member;
          for (int64_t i = i0; i < i1; ++i) {
            int64_t t = i;
            if (keep_idx) {
              t = keep_idx[(l * H + h) * k + i];
              if (t < 0 || t >= T) return -1;
            }
            member.push_back(bf16_to_f32(v.row(l, t, h)[c]));
          }
          float scale = 0.0f, mn = 0.0f;
          if (!member.empty()) {
            if (asym) {
              float mx = member[0];
              mn = member[0];
              for (float f : member) {
                mn = std::min(mn, f);
                mx = std::max(mx, f);
              }
              if (mn == 0.0f) mn = 0.0f;  // a zero extreme is taken as +0
              if (mx == 0.0f) mx = 0.0f;
              const float range = mx - mn;
              scale = range / static_cast<float>(levels);
            } else {
              float amax = 0.0f;
              for (float f : member) amax = std::max(amax, std::fabs(f));
              scale = amax / static_cast<float>(qmax);
            }
          }
          const int64_t so = ((l * n_groups + g) * H + h) * D + c;
          scales[so] = scale;
          if (asym) mins[so] = mn;
          for (size_t j = 0; j < member.size(); ++j) {
            int q = 0;
            if (scale != 0.0f) {
              if (asym) {
                const float d = member[j] - mn;
                q = static_cast<int>(std::rint(d / scale));
                q = std::min(levels, std::max(0, q));
              } else {
                q = static_cast<int>(std::rint(member[j] / scale));
                q = std::min(qmax, std::max(-qmax, q));
              }
            }
            const int64_t i = i0 + static_cast<int64_t>(j);
            uint8_t* byte = codes + ((l * Tp + i) * H + h) * cb + c / per_byte;
            *byte = static_cast<uint8_t>(*byte | ((static_cast<uint32_t>(q) & field_mask) << (bits * (c % per_byte))));
          }
        }
  return 0;
}

// Inverse of oracle_quantize_channel into the paged pool: y = bf16_rne(q * scale) or, asym,
// bf16_rne(fl32(fl32(q * scale) + mn)), with the scale (and minimum) of slot t's group and channel.
int oracle_dequantize_paged_channel(const uint8_t* codes, const float* scales, const float* mins, int bits, int group,
                                    int asym, int64_t L, int64_t T, int64_t Tp, int64_t H, int64_t D,
                                    const int32_t* block_table, int64_t num_blocks, int64_t bs, uint16_t* pool,
                                    int64_t pool_stride_l) {
  if (!codes || !scales || (asym && !mins) || !block_table || !pool || bs <= 0 || T > Tp || group <= 0) return -1;
  if ((bits != 8 && bits != 4 && bits != 2) || D <= 0 || (D * bits) % 8 != 0) return -1;
  const int64_t cb = D * bits / 8, n_groups = (Tp + group - 1) / group;
  const int per_byte = 8 / bits;
  const uint32_t field_mask = (1u << bits) - 1u;
  const int sign_bit = 1 << (bits - 1);
  for (int64_t l = 0; l < L; ++l)
    for (int64_t t = 0; t < T; ++t) {
      const int64_t blk = block_table[t / bs];
      if (blk < 0 || blk >= num_blocks) return -1;
      for (int64_t h = 0; h < H; ++h)
        for (int64_t c = 0; c < D; ++c) {
          const uint8_t byte = codes[((l * Tp + t) * H + h) * cb + c / per_byte];
          int q = static_cast<int>((byte >> (bits * (c % per_byte))) & field_mask);
          if (!asym && (q & sign_bit)) q -= (1 << bits);
          const int64_t so = ((l * n_groups + t / group) * H + h) * D + c;
          float y = static_cast<float>(q) * scales[so];
          if (asym) y = y + mins[so];
          pool[l * pool_stride_l + ((blk * bs + t % bs) * H + h) * D + c] = f32_to_bf16_rne(y);
        }
    }
  return 0;
}

// Attention-score token importance: for each layer and kv head, the softmax
// probabilities of the G*W window-query rows (G = Hq / Hkv query heads of that
// kv head, W last positions of the context) over all T keys, logits scaled by
// 1/sqrt(D), causal mask inside the window when `causal`, summed over the G*W
// rows; window positions are forced to +inf when `force_window` so they are
// always kept.  q is [L][W][Hq][D], k is [L][T][Hkv][D], strides in elements.
// scores is [L][Hkv][T] binary32.
int oracle_score_tokens(const uint16_t* q, int64_t W, int64_t Hq, int64_t q_sl, int64_t q_st, int64_t q_sh,
                        const uint16_t* k, int64_t L, int64_t T, int64_t Hkv, int64_t D, int64_t k_sl,
                        int64_t k_st, int64_t k_sh, int causal, int force_window, float* scores) {
  if (!q || !k || !scores || Hkv <= 0 || Hq % Hkv != 0 || W <= 0 || W > T || D <= 0) return -1;
  const int64_t G = Hq / Hkv;
  const View qv{q, q_sl, q_st, q_sh}, kv{k, k_sl, k_st, k_sh};
  std::vector<double> P;
  for (int64_t l = 0; l < L; ++l)
    for (int64_t h = 0; h < Hkv; ++h) {
      window_probs(qv, kv, l, h, G, W, T, D, causal != 0, nullptr, P);
      scores_from_probs(P, G * W, T, W, force_window != 0, scores + (l * Hkv + h) * T);
    }
  return 0;
}

// Restore of a dropped-and-quantized plane at the ORIGINAL token positions: slot i of head h of a
// compressed plane with k slots came from token keep_idx[l][h][i] (see oracle_quantize with a keep
// list) and is written back to that token's place in a paged pool that spans all T tokens,
//   pool[l][block_table[t / bs]][t % bs][h][:] = dequantized slot i,  t = keep_idx[l][h][i];
// positions of dropped tokens are left untouched.  Any of the four codecs: asym (unsigned codes plus
// minimum) or not, group_axis 0 (groups of channels, scales [L][Tp][H][D/group]) or 1 (groups of
// token slots, scales [L][ceil(Tp/group)][H][D]).  One binary32 multiply (and one add), bf16 RNE.
int oracle_dequantize_paged_scatter(const uint8_t* codes, const float* scales, const float* mins, int bits, int group,
                                    int asym, int group_axis, int64_t L, int64_t k, int64_t Tp, int64_t H, int64_t D,
                                    const int32_t* keep_idx, int64_t T, const int32_t* block_table,
                                    int64_t num_blocks, int64_t bs, uint16_t* pool, int64_t pool_stride_l) {
  if (!codes || !scales || (asym && !mins) || !keep_idx || !block_table || !pool) return -1;
  if ((bits != 8 && bits != 4 && bits != 2) || group <= 0 || D <= 0 || (D * bits) % 8 != 0) return -1;
  if (group_axis == 0 && D % group != 0) return -1;
  if (k < 0 || k > Tp || k > T || bs <= 0) return -1;
  const int64_t cb = D * bits / 8;
  const int per_byte = 8 / bits;
  const uint32_t field_mask = (1u << bits) - 1u;
  const int sign_bit = 1 << (bits - 1);
  const int64_t n_groups = (Tp + group - 1) / group;
  for (int64_t l = 0; l < L; ++l)
    for (int64_t h = 0; h < H; ++h)
      for (int64_t i = 0; i < k; ++i) {
        const int64_t t = keep_idx[(l * H + h) * k + i];
        if (t < 0 || t >= T) return -1;
        const int64_t blk = block_table[t / bs];
        if (blk < 0 || blk >= num_blocks) return -1;
        for (int64_t c = 0; c < D; ++c) {
          const uint8_t byte = codes[((l * Tp + i) * H + h) * cb + c / per_byte];
          int q = static_cast<int>((byte >> (bits * (c % per_byte))) & field_mask);
          if (!asym && (q & sign_bit)) q -= (1 << bits);
          const int64_t so = group_axis == 0 ? ((l * Tp + i) * H + h) * (D / group) + c / group
                                             : ((l * n_groups + i / group) * H + h) * D + c;
          float y = static_cast<float>(q) * scales[so];
          if (asym) y = y + mins[so];
          pool[l * pool_stride_l + ((blk * bs + t % bs) * H + h) * D + c] = f32_to_bf16_rne(y);
        }
      }
  return 0;
}

// Score smoothing before the selection (the published snapkv method that the paper's Baselines
// evaluate pools the summed attention votes along the token axis, so that neighbours of an
// important token are kept with it).  For the prefix positions t < T - window:
//   mode 0 (average): out[t] = (sum of scores[u], |u - t| <= kernel/2, 0 <= u < T - window) / kernel
//                     (positions outside the prefix count as zeros: the divisor is always `kernel`)
//   mode 1 (maximum): out[t] = max of the same in-range scores
// The last `window` positions (the observation window, kept unconditionally) are copied unchanged
// and never leak into the prefix.  kernel is odd.  Sums are formed in double.
int oracle_smooth_scores(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t window,
                         int kernel, int mode, float* out, int64_t out_stride) {
  if (!scores || !out || n_rows < 0 || T <= 0 || window < 0 || window > T) return -1;
  if (kernel < 1 || kernel % 2 == 0 || (mode != 0 && mode != 1)) return -1;
  const int64_t P = T - window, r = kernel / 2;
  for (int64_t row = 0; row < n_rows; ++row) {
    const float* in = scores + row * row_stride;
    float* o = out + row * out_stride;
    for (int64_t t = 0; t < P; ++t) {
      const int64_t u0 = std::max<int64_t>(0, t - r), u1 = std::min<int64_t>(P - 1, t + r);
      if (mode == 0) {
        double sum = 0.0;
        for (int64_t u = u0; u <= u1; ++u) sum += static_cast<double>(in[u]);
        o[t] = static_cast<float>(sum / static_cast<double>(kernel));
      } else {
        float m = in[u0];
        for (int64_t u = u0 + 1; u <= u1; ++u) m = std::max(m, in[u]);
        o[t] = m;
      }
    }
    for (int64_t t = P; t < T; ++t) o[t] = in[t];
  }
  return 0;
}

// Per-row top-k keep-set: indices of the k largest scores of each row, ties
// toward the lowest index, written ascending.  scores is n_rows rows of T
// floats, row_stride floats apart; idx_out is [n_rows][k] int32.
int oracle_select_topk(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                       int32_t* idx_out) {
  if (!scores || (!idx_out && k > 0) || k < 0 || k > T || T <= 0 || row_stride < T) return -1;
  for (int64_t r = 0; r < n_rows; ++r) topk_row(scores + r * row_stride, T, k, idx_out + r * k);
  return 0;
}

// Quality-loss proxy of every candidate configuration (bits, group, keep_k) of
// one context: relative L2 error of the window queries' attention output
// softmax(Q K^T / sqrt(D)) V when K, V are replaced by dequantize(quantize())
// at (bits, group) (bits == 16: unquantized) and the keys are restricted to
// the top-keep_k keep-set of the unquantized-score ranking (keep_k == T: no
// dropping).  loss[c] = sqrt(num_c / den), num_c and den summed over layers,
// query heads, window rows and channels.  partial (may be null) receives
// [L][n_cfgs][2] = (num, den) per layer.
int oracle_eval_configs(const uint16_t* q, int64_t W, int64_t Hq, int64_t q_sl, int64_t q_st, int64_t q_sh,
                        const uint16_t* k, int64_t k_sl, int64_t k_st, int64_t k_sh, const uint16_t* v,
                        int64_t v_sl, int64_t v_st, int64_t v_sh, int64_t L, int64_t T, int64_t Hkv, int64_t D,
                        const int32_t* cfg_bits, const int32_t* cfg_group, const int64_t* cfg_keep,
                        int32_t n_cfgs, float* loss, double* partial) {
  if (!q || !k || !v || !loss || !cfg_bits || !cfg_group || !cfg_keep) return -1;
  if (Hkv <= 0 || Hq % Hkv != 0 || W <= 0 || W > T || D <= 0 || n_cfgs < 0) return -1;
  for (int32_t c = 0; c < n_cfgs; ++c) {
    if (cfg_bits[c] != 16 && !quant_args_ok(cfg_bits[c], cfg_group[c], D)) return -1;
    if (cfg_keep[c] < 1 || cfg_keep[c] > T) return -1;
  }
  const int64_t G = Hq / Hkv, GW = G * W;
  const View qv{q, q_sl, q_st, q_sh}, kv{k, k_sl, k_st, k_sh}, vv{v, v_sl, v_st, v_sh};
  std::vector<double> num(static_cast<size_t>(n_cfgs), 0.0);
  double den = 0.0;
  std::vector<double> P, Pc, o_full(static_cast<size_t>(GW * D)), o_c(static_cast<size_t>(GW * D));
  std::vector<float> sc(static_cast<size_t>(T));
  std::vector<int32_t> keep(static_cast<size_t>(T));
  std::vector<uint8_t> allowed(static_cast<size_t>(T));
  std::vector<uint16_t> kh(static_cast<size_t>(T * D)), vh(static_cast<size_t>(T * D));
  std::vector<uint8_t> codes(static_cast<size_t>(D));
  std::vector<float> scl(static_cast<size_t>(D));

  for (int64_t l = 0; l < L; ++l) {
    std::vector<double> num_l(static_cast<size_t>(n_cfgs), 0.0);
    double den_l = 0.0;
    for (int64_t h = 0; h < Hkv; ++h) {
      // reference output and the ranking, both from the unquantized keys
      window_probs(qv, kv, l, h, G, W, T, D, true, nullptr, P);
      for (int64_t r = 0; r < GW; ++r)
        for (int64_t c = 0; c < D; ++c) {
          double acc = 0.0;
          for (int64_t t = 0; t < T; ++t)
            acc += P[static_cast<size_t>(r * T + t)] * static_cast<double>(bf16_to_f32(vv.row(l, t, h)[c]));
          o_full[static_cast<size_t>(r * D + c)] = acc;
          den_l += acc * acc;
        }
      scores_from_probs(P, GW, T, W, true, sc.data());

      for (int32_t ci = 0; ci < n_cfgs; ++ci) {
        const int bits = cfg_bits[ci], group = cfg_group[ci];
        const int64_t kk = cfg_keep[ci];
        // K-hat, V-hat: what decoding would read back, as bf16 values
        for (int64_t t = 0; t < T; ++t) {
          const uint16_t* kr = kv.row(l, t, h);
          const uint16_t* vr = vv.row(l, t, h);
          if (bits == 16) {
            std::copy(kr, kr + D, &kh[static_cast<size_t>(t * D)]);
            std::copy(vr, vr + D, &vh[static_cast<size_t>(t * D)]);
          } else {
            quantize_row(kr, D, bits, group, codes.data(), scl.data());
            dequantize_row(codes.data(), scl.data(), D, bits, group, &kh[static_cast<size_t>(t * D)]);
            quantize_row(vr, D, bits, group, codes.data(), scl.data());
            dequantize_row(codes.data(), scl.data(), D, bits, group, &vh[static_cast<size_t>(t * D)]);
          }
        }
        topk_row(sc.data(), T, kk, keep.data());
        std::fill(allowed.begin(), allowed.end(), 0);
        for (int64_t i = 0; i < kk; ++i) allowed[static_cast<size_t>(keep[static_cast<size_t>(i)])] = 1;
        // head-local views: q indexes the G heads of this kv head
        const View qh{qv.row(l, 0, h * G), 0, q_st, q_sh};
        const View khv{kh.data(), 0, D, 0};
        window_probs(qh, khv, 0, 0, G, W, T, D, true, allowed.data(), Pc);
        for (int64_t r = 0; r < GW; ++r)
          for (int64_t c = 0; c < D; ++c) {
            double acc = 0.0;
            for (int64_t t = 0; t < T; ++t)
              if (allowed[static_cast<size_t>(t)])
                acc += Pc[static_cast<size_t>(r * T + t)] *
                       static_cast<double>(bf16_to_f32(vh[static_cast<size_t>(t * D + c)]));
            const double d = acc - o_full[static_cast<size_t>(r * D + c)];
            num_l[static_cast<size_t>(ci)] += d * d;
          }
      }
    }
    den += den_l;
    for (int32_t ci = 0; ci < n_cfgs; ++ci) {
      num[static_cast<size_t>(ci)] += num_l[static_cast<size_t>(ci)];
      if (partial) {
        partial[(l * n_cfgs + ci) * 2 + 0] = num_l[static_cast<size_t>(ci)];
        partial[(l * n_cfgs + ci) * 2 + 1] = den_l;
      }
    }
  }
  for (int32_t ci = 0; ci < n_cfgs; ++ci)
    loss[ci] = static_cast<float>(std::sqrt(num[static_cast<size_t>(ci)] / den));
  return 0;
}

// Key-only token importance of the paper's two other token-dropping methods (Evaluation, Baselines):
//   method 0, knorm:   tokens whose key has a small L2 norm are dropped
//                      score[t] = ||k_t||_2                              (keep the largest)
//   method 1, keydiff: tokens whose key is, on average, most similar (cosine) to all other keys are dropped
//                      score[t] = - mean over t' != t of cos(k_t, k_t')  (keep the largest)
// written out as the plain definitions (keydiff is the O(T^2 D) double loop).  A zero key has cosine
// 0 with everything; T == 1 gives score 0.  With `tokens` (n of them) only those tokens are scored
// (out has n entries per (layer, head)); otherwise all T (out is [L][H][T]).
int oracle_score_keys(const uint16_t* k, int64_t L, int64_t T, int64_t H, int64_t D, int64_t k_sl, int64_t k_st,
                      int64_t k_sh, int method, const int32_t* tokens, int64_t n, float* out) {
  if (!k || !out || L < 0 || T <= 0 || H <= 0 || D <= 0 || (method != 0 && method != 1)) return -1;
  const View kv{k, k_sl, k_st, k_sh};
  const int64_t n_out = tokens ? n : T;
  std::vector<double> norm(static_cast<size_t>(T));
  for (int64_t l = 0; l < L; ++l)
    for (int64_t h = 0; h < H; ++h) {
      for (int64_t t = 0; t < T; ++t) {
        double ss = 0.0;
        const uint16_t* r = kv.row(l, t, h);
        for (int64_t c = 0; c < D; ++c) ss += static_cast<double>(bf16_to_f32(r[c])) * bf16_to_f32(r[c]);
        norm[static_cast<size_t>(t)] = std::sqrt(ss);
      }
      for (int64_t i = 0; i < n_out; ++i) {
        const int64_t t = tokens ? tokens[i] : i;
        if (t < 0 || t >= T) return -1;
        double score;
        if (method == 0) {
          score = norm[static_cast<size_t>(t)];
        } else {
          double acc = 0.0;
          const uint16_t* a = kv.row(l, t, h);
          for (int64_t u = 0; u < T; ++u) {
            if (u == t) continue;
            const double nn = norm[static_cast<size_t>(t)] * norm[static_cast<size_t>(u)];
            if (nn == 0.0) continue;
            const uint16_t* b = kv.row(l, u, h);
            double dot = 0.0;
            for (int64_t c = 0; c < D; ++c) dot += static_cast<double>(bf16_to_f32(a[c])) * bf16_to_f32(b[c]);
            acc += dot / nn;
          }
          score = T > 1 ? -acc / static_cast<double>(T - 1) : 0.0;
        }
        out[(l * H + h) * n_out + i] = static_cast<float>(score);
      }
    }
  return 0;
}

// Number of tokens kept at a keep-ratio: ceil(ratio * T) in double, clamped to [1, T].
int64_t oracle_keep_count(double ratio, int64_t T) {
  int64_t k = static_cast<int64_t>(std::ceil(ratio * static_cast<double>(T)));
  return std::min<int64_t>(T, std::max<int64_t>(1, k));
}

// Scalar conversions exposed so the tests can pin them against a library.
uint16_t oracle_f32_to_bf16(float f) { return f32_to_bf16_rne(f); }
float oracle_bf16_to_f32(uint16_t h) { return bf16_to_f32(h); }

}  // extern "C"
