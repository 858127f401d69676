// Launchers shared between translation units of libkvp (not part of the C ABI).
#pragma once

#include "kvp_common.h"

namespace kvp {

// kvp_score_tokens on an explicit stream (validates like the public entry point).
int32_t score_tokens_impl(const kvp_view* q_win, const kvp_view* k, int32_t causal, int32_t force_window,
                          float* scores, void* ws, size_t ws_bytes, hipStream_t st);

// kvp_select_topk's kernel launches; arguments already validated, n_rows > 0, 0 < k <= T; ws holds at least
// select_workspace_bytes(n_rows, T) bytes, 16-byte aligned (may be null when that is 0).
size_t select_workspace_bytes(int64_t n_rows, int64_t T);
void select_topk_launch(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                        int32_t* idx_out, void* ws, hipStream_t st);

// Validated arguments of kvp_quantize as the kernels take them.
enum SrcMode { kLinear = 0, kStrided = 1, kPaged = 2 };
struct QuantArgs {
  const uint16_t* src;         // view base or page pool
  int64_t stride_l, stride_t, stride_h;  // elements (view); stride_l also for the pool
  const int32_t* block_table;  // paged source only
  const int32_t* keep_idx;     // [L][H][k] or null
  int64_t k;                   // row length of keep_idx
  uint32_t n_slots;            // valid slots per layer (T, or k when gathered)
  uint32_t T;                  // source tokens per layer
  uint32_t num_blocks;         // paged source only
  uint32_t rows_per_layer;     // Tp * H
  uint32_t H, bs;
  FastDiv div_h, div_bs;
  uint8_t* codes;
  float* scales;
  float* mins;   // asymmetric codec only
};

// Validated arguments of kvp_dequantize_paged.
struct DequantArgs {
  const uint8_t* codes;
  const float* scales;
  const float* mins;   // asymmetric codec only
  uint16_t* pool;
  const int32_t* block_table;
  int64_t pool_stride_l;   // elements
  int64_t Tp;
  uint32_t T, H, bs, num_blocks;   // T: slots of the compressed plane to restore
  // scatter restore only: slot i of head h goes to token keep_idx[l][h][i] of a pool that spans T_full tokens
  const int32_t* keep_idx;
  int64_t k;
  uint32_t T_full;
  FastDiv div_h, div_bs;
};

// Destination row of the scatter restore: source row r of a block whose first slot is t0.
__device__ __forceinline__ uint16_t* scatter_row(const DequantArgs& a, uint32_t l, uint32_t t0, uint32_t r) {
  const uint32_t di = a.div_h.quot(r), h = r - di * a.H;
  // an out-of-contract index is clamped so that a bad keep list cannot fault the GPU
  const uint32_t t = min(static_cast<uint32_t>(a.keep_idx[(static_cast<int64_t>(l) * a.H + h) * a.k + t0 + di]), a.T_full - 1);
  const uint32_t pg = a.div_bs.quot(t);
  const int64_t blk = min(static_cast<uint32_t>(a.block_table[pg]), a.num_blocks - 1);
  return a.pool + static_cast<int64_t>(l) * a.pool_stride_l + ((blk * a.bs + (t - pg * a.bs)) * a.H + h) * kHeadDim;
}

// Groups along the token axis (KVP_GROUP_TOKENS): kernel launches for validated arguments.
void quantize_channel_launch(const QuantArgs& a, int bits, int group, int mode, int64_t L, hipStream_t st);
void dequantize_channel_launch(const DequantArgs& a, int bits, int group, int64_t L, hipStream_t st);  // scatter if a.keep_idx

}  // namespace kvp
