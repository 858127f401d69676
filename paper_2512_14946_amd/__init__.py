"""MI355X-native KV-cache compress / decompress hot path (after EvicPress, arxiv 2512.14946).

The work is done by libkvp.so (hand-written HIP for gfx950, C ABI in include/kvp.h); this
package only marshals torch tensors into that ABI.  There is no CPU fallback: if the library is
not built, importing the binding raises.
"""
from .kvp import (  # noqa: F401
    KVPError, PagedKV, QPlane, alloc_paged, alloc_qplane, kvp_copy_bytes, kvp_selftest_reciprocal, kvp_dequantize_paged,
    kvp_dequantize_paged_scatter,
    kvp_eval_configs, kvp_eval_workspace_bytes, kvp_keep_count, kvp_quantize, kvp_score_tokens,
    kvp_score_tokens_static, KVP_SCORE_STATIC_SCRATCH_BYTES,
    KVP_EVAL_PV_MATRIX_CORES, KVP_EVAL_PV_FP32, KVP_OP_COMPRESS, KVP_OP_EVICT, KVP_OP_INSERT, kvp_policy_insert, kvp_utility_table,
    KVP_SCORE_KEYDIFF, KVP_SCORE_KNORM, kvp_score_keys, kvp_score_keys_workspace_bytes,
    kvp_score_workspace_bytes, kvp_select_topk, kvp_select_workspace_bytes, kvp_smooth_scores, kvp_strerror,
    kvp_version, kvp_workspace_bytes, KVP_WS_SCORE_TOKENS, KVP_WS_SCORE_KEYS, KVP_WS_SELECT_TOPK, KVP_WS_EVAL_CONFIGS,
    library_path,
)
