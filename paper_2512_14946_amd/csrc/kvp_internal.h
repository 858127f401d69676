// Launchers shared between translation units of libkvp (not part of the C ABI).
#pragma once

#include "kvp_common.h"

namespace kvp {

// kvp_score_tokens on an explicit stream (validates like the public entry point).
int32_t score_tokens_impl(const kvp_view* q_win, const kvp_view* k, int32_t causal, int32_t force_window,
                          float* scores, void* ws, size_t ws_bytes, hipStream_t st);

// kvp_select_topk's kernel launch; arguments already validated, n_rows > 0, 0 < k <= T.
void select_topk_launch(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                        int32_t* idx_out, hipStream_t st);

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
  uint32_t T, H, bs, num_blocks;
};

// Groups along the token axis (KVP_GROUP_TOKENS): kernel launches for validated arguments.
void quantize_channel_launch(const QuantArgs& a, int bits, int group, int mode, int64_t L, hipStream_t st);
void dequantize_channel_launch(const DequantArgs& a, int bits, int group, int64_t L, hipStream_t st);

}  // namespace kvp
