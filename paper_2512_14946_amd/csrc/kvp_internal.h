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

}  // namespace kvp
