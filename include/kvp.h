/*
 * kvp.h -- C ABI of libkvp: the KV-cache compress / decompress hot path of
 * EvicPress (arxiv 2512.14946) on one MI355X (gfx950).
 *
 * The paper's system keeps several compressed versions of a context's KV cache
 * (different methods and ratios), scores every version, and on a cache hit
 * loads the chosen version back into the serving engine's paged GPU memory (System design: profiler module, utility function; Implementation:
 * lookup / retrieve / store / manage).  This library is the data-parallel part
 * of that: quantize, dequantize into pages, score tokens, select a keep-set,
 * and evaluate a quality-loss proxy for every candidate configuration.
 *
 * Conventions for every call
 *   - All tensor pointers are DEVICE pointers unless a comment says "host".
 *     The structs themselves and kvp_config arrays are read on the HOST.
 *   - The caller owns every buffer.  The library never allocates, frees or
 *     keeps a pointer after the call returns.  Scratch memory comes from the
 *     caller as (ws, ws_bytes); the size needed is returned by the matching
 *     kvp_*_workspace_bytes call.
 *   - Calls validate their arguments on the host, enqueue kernels on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and return
 *     without synchronizing.  A call that fails validation enqueues nothing.
 *   - Device pointers must be 16-byte aligned and strides must keep every row
 *     of D elements 16-byte aligned.  head_dim D must be 128.
 *   - Results are deterministic: the same inputs give the same bytes.
 *   - Return value: KVP_OK or a negative KVP_ERR_* code; kvp_strerror() names it.
 */
#ifndef KVP_H_
#define KVP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  KVP_OK = 0,
  KVP_ERR_NULL = -1,        /* a required pointer is NULL */
  KVP_ERR_ALIGN = -2,       /* a pointer or stride breaks the 16-byte row alignment */
  KVP_ERR_SHAPE = -3,       /* sizes inconsistent (k > T, W > T, Hq % Hkv != 0, D % group != 0, ...) */
  KVP_ERR_UNSUPPORTED = -4, /* bits not in {8,4,2} (16 allowed in kvp_config), group not in {32,64,128}, D != 128 */
  KVP_ERR_WORKSPACE = -5,   /* ws is NULL or ws_bytes is smaller than kvp_*_workspace_bytes() */
  KVP_ERR_LAUNCH = -6       /* the HIP runtime refused a launch */
};

/* Strided bf16 tensor [L][T][H][D], innermost D contiguous; strides in elements. */
typedef struct {
  const void* ptr; /* device, bf16 */
  int64_t L, T, H, D;
  int64_t stride_l, stride_t, stride_h;
} kvp_view;

/* Paged bf16 plane (K or V) in the serving engine's page pool (Background:
 * PagedAttention's page-like blocks; Implementation: retrieve fills the
 * engine's paged GPU memory).  Token t of layer l lives at
 * pool[l][block_table[t / bs]][t % bs][h][:].  One block table per context,
 * shared by all layers.  Entries must lie in [0, num_blocks). */
typedef struct {
  void* pool;                 /* device, bf16 [L][num_blocks][bs][H][D], layers stride_l elements apart */
  const int32_t* block_table; /* device, int32 [ceil(T / bs)] */
  int64_t L, num_blocks, bs, H, D, T;
  int64_t stride_l;
} kvp_paged;

/* Compressed plane: packed codes and one fp32 scale per group.  Slot s of head
 * h holds one token's D channels: D*bits/8 bytes, channel order, fields packed
 * little-endian inside a byte, two's complement truncated to `bits`.  Slots
 * T <= s < Tp are padding (zero codes, zero scales) so that the plane splits
 * into whole pages of the compressed store; Tp >= T. */
typedef struct {
  uint8_t* codes; /* device [L][Tp][H][D*bits/8] */
  float* scales;  /* device [L][Tp][H][D/group] */
  float* mins;    /* NULL: symmetric codec.  Else device [L][Tp][H][D/group]: asymmetric codec (see kvp_quantize) */
  int32_t bits, group;
  int64_t L, T, Tp, H, D;
  int32_t group_axis; /* KVP_GROUP_CHANNELS (0) or KVP_GROUP_TOKENS (1), see kvp_quantize */
} kvp_qplane;

/* What a quantization group runs over.  KVP_GROUP_CHANNELS: `group` consecutive channels of one
 * token (the layouts above).  KVP_GROUP_TOKENS: `group` consecutive slots of ONE channel of one
 * head ("per-channel" key quantization); scales (and mins) are then device
 * [L][ceil(Tp/group)][H][D], the codes plane is unchanged, the last group of a plane holds the
 * T % group remaining slots, and padding slots never enter a minimum or maximum. */
enum { KVP_GROUP_CHANNELS = 0, KVP_GROUP_TOKENS = 1 };

/* One candidate configuration of the utility table: quantization (bits = 16
 * means none; group is then ignored) and the number of tokens kept
 * (keep_k = T means no token dropping). */
typedef struct {
  int32_t bits, group;
  int64_t keep_k;
} kvp_config;

/* Group-wise symmetric quantization (Background, KV cache compression: the
 * quantization category stores KV entries at a lower bit width; Related work:
 * uniform quantization; Limitations: a method pool that joins token dropping
 * with quantization).  For every group of `group` consecutive channels
 * of one token's head vector:
 *     scale = max|x| / qmax   (qmax = 2^(bits-1) - 1; IEEE binary32 division)
 *     code  = clamp(rint(x / scale), -qmax, qmax)   (binary32 division,
 *             round-half-to-even; code 0 when scale == 0)
 * Exactly one of `src` (strided view) and `src_paged` is non-NULL.  With
 * `keep_idx` (device int32 [L][H][k], ascending, values in [0, T)) slot i of
 * head h takes source token keep_idx[l][h][i] and dst->T must equal k;
 * otherwise slot i is token i, k is ignored and dst->T must equal the source
 * T.  Writes dst->codes and dst->scales in full, padding slots included.
 * With dst->mins != NULL the asymmetric variant is used instead (uniform quantization with a
 * zero point, all 2^bits levels): per group mn = min x (a zero minimum or maximum is taken as +0), scale = fl32(fl32(max x - mn) / (2^bits - 1)),
 * code = clamp(rint(fl32(fl32(x - mn) / scale)), 0, 2^bits - 1) as an UNSIGNED field, mins = mn;
 * kvp_dequantize_paged then returns bf16_rne(fl32(fl32(code * scale) + mn)).
 * With dst->group_axis == KVP_GROUP_TOKENS the same formulas apply to groups of dst->group slots
 * of one channel (Related work: KIVI / KVQuant style per-channel key quantizers); group is 32, 64
 * or 128 slots, slots being kept tokens when keep_idx is given.
 * Limits: D = 128; L <= 65535; T, Tp * H and num_blocks below 2^31.  Entries of keep_idx and of a source
 * block table that lie outside their range are clamped into it (the call cannot fault on them; the slots
 * they feed are then meaningless): KVP_ERR_SHAPE is for sizes, not for table contents, which stay on the device. */
int32_t kvp_quantize(const kvp_view* src, const kvp_paged* src_paged, const int32_t* keep_idx, int64_t k,
                     const kvp_qplane* dst, void* stream);

/* Inverse direction, into the paged pool (Background: quantization methods
 * pay a decompression step; Implementation: retrieve).  For t < src->T:
 *     pool[l][block_table[t/bs]][t%bs][h][c] = bf16_rne((float)code * scale)
 * (one binary32 multiply, then round-to-nearest-even to bf16).  Page slots at
 * or beyond T and blocks the table does not name are not written.  dst->T
 * must equal src->T; L, H, D must match.  Planes grouped along tokens
 * (KVP_GROUP_TOKENS) need src->group to be a multiple of dst->bs, so that a
 * page lies inside one group (KVP_ERR_UNSUPPORTED otherwise).
 * Limits: D = 128; L <= 65535; T, bs * H and num_blocks below 2^31.  Block-table entries outside
 * [0, num_blocks) are clamped into it, as in kvp_quantize. */
int32_t kvp_dequantize_paged(const kvp_qplane* src, const kvp_paged* dst, void* stream);

/* Restore of a dropped-and-quantized plane at the ORIGINAL token positions (Limitations: the pool
 * that joins token dropping with quantization; Implementation: retrieve into paged GPU memory).  src holds k = src->T slots per head, written by kvp_quantize with the same keep_idx
 * (device int32 [L][H][k], values in [0, dst->T)); slot i of head h is dequantized as in
 * kvp_dequantize_paged and stored at token t = keep_idx[l][h][i] of the pool, which spans
 * dst->T >= k tokens:  pool[l][block_table[t/bs]][t%bs][h][:].  Rows of dropped tokens are not
 * written.  keep_idx doubles as the position ids of the restored rows.  Limits as for
 * kvp_dequantize_paged; keep_idx entries outside [0, dst->T) are clamped into it. */
int32_t kvp_dequantize_paged_scatter(const kvp_qplane* src, const int32_t* keep_idx, const kvp_paged* dst,
                                     void* stream);

/* Attention-score token importance (Evaluation, Baselines: snapkv scores the
 * earlier context by the attention it receives from the tokens next to the
 * query).  q_win is [L][W][Hq][D]: the queries of the last W positions
 * (T-W .. T-1) of the context; k is [L][T][Hkv][D]; G = Hq / Hkv query heads
 * share kv head h (heads h*G .. h*G+G-1).  For each (l, h):
 *     scores[l][h][t] = sum over the G*W window rows of softmax_t(q.k / sqrt(D))
 * with keys after a row's own position masked when `causal`, and positions
 * t >= T-W set to +inf when `force_window` (window tokens are always kept).
 * bf16 inputs, fp32 accumulation.  scores is device fp32 [L][Hkv][T].
 * Limits: D = 128; G * W <= 512 window rows per kv head (KVP_ERR_UNSUPPORTED beyond); L * Hkv <= 65535;
 * W <= T < 2^30 (KVP_ERR_SHAPE). */
int32_t kvp_score_tokens(const kvp_view* q_win, const kvp_view* k, int32_t causal, int32_t force_window,
                         float* scores, void* ws, size_t ws_bytes, void* stream);
size_t kvp_score_workspace_bytes(int64_t L, int64_t Hkv, int64_t Hq, int64_t W, int64_t T);

/* kvp_score_tokens for callers that cannot allocate device memory or carry a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels and the
 * same results, bit for bit, with the scratch in a fixed device array inside the library
 * (KVP_SCORE_STATIC_SCRATCH_BYTES per GPU, held until the process ends).  The call allocates and
 * frees nothing and calls no allocating routine.  Shapes whose kvp_score_workspace_bytes() exceeds
 * the array return KVP_ERR_WORKSPACE and enqueue nothing (4 MiB covers one layer of every shape up
 * to Hkv = 8, G*W = 512, T = 131072, and whole small contexts).  All calls on one GPU share the one
 * array: calls that may overlap on that GPU (different streams, different host threads) race and
 * must be ordered by the caller; calls on one stream are ordered by the stream.  The array keeps
 * the previous call's contents; every word a call reads it has written itself first. */
#define KVP_SCORE_STATIC_SCRATCH_BYTES (4u << 20)
int32_t kvp_score_tokens_static(const kvp_view* q_win, const kvp_view* k, int32_t causal, int32_t force_window,
                                float* scores, void* stream);

/* Key-only token importance of the paper's two other token-dropping methods
 * (Evaluation, Baselines): knorm scores a token by the L2 norm of its key (low
 * norms are dropped); keydiff by the average cosine similarity of its key to
 * the keys of all other tokens (similar tokens are dropped).  scores (device
 * fp32 [L][H][T]) are "keep the largest" scores for kvp_select_topk:
 *     KVP_SCORE_KNORM    scores[l][h][t] = ||k_t||_2
 *     KVP_SCORE_KEYDIFF  scores[l][h][t] = - mean over t' != t of cos(k_t, k_t')
 * A zero key has cosine 0 with every key; T == 1 gives 0.  bf16 input, fp32
 * arithmetic.  No window is forced.  knorm needs no workspace. */
enum { KVP_SCORE_KNORM = 0, KVP_SCORE_KEYDIFF = 1 };
int32_t kvp_score_keys(const kvp_view* k, int32_t method, float* scores, void* ws, size_t ws_bytes, void* stream);
size_t kvp_score_keys_workspace_bytes(int64_t L, int64_t H, int64_t T, int32_t method);

/* Per-row top-k keep-set (Evaluation, Baselines: the tokens with the lowest
 * attention scores are dropped; IMPRESS keeps the top X %).  For each
 * of n_rows rows of T fp32 scores (row_stride floats apart): the indices of the
 * k largest, equal scores resolved toward the lowest index, written ascending
 * to idx_out [n_rows][k] (device int32).  NaN scores are out of contract.
 * 0 <= k <= T; T < 2^30.  Rows longer than 16384 and up to 2^18 scores are split over several
 * workgroups and need scratch: kvp_select_workspace_bytes(n_rows, T, k) bytes (16 bytes for two
 * pivots and a flag per row, two counts per 16384-score span, 64 KiB of candidate slots per
 * row), 16-byte aligned; it returns 0 for other lengths, for which ws may be NULL.  A missing
 * or short workspace: KVP_ERR_WORKSPACE. */
int32_t kvp_select_topk(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t k,
                        int32_t* idx_out, void* ws, size_t ws_bytes, void* stream);
size_t kvp_select_workspace_bytes(int64_t n_rows, int64_t T, int64_t k);

/* Score smoothing before the selection (Evaluation, Baselines: snapkv; the published method pools
 * the summed attention votes along the token axis so that the neighbours of an important token are
 * kept with it).  Rows as in kvp_select_topk; P = T - window is the prefix length.  For t < P:
 *     KVP_SMOOTH_AVG: out[t] = (sum of scores[u], |u - t| <= kernel/2, 0 <= u < P) / kernel
 *                     (taps outside the prefix count as zeros; fp32 sum, left to right)
 *     KVP_SMOOTH_MAX: out[t] = max of the same in-range scores
 * and out[t] = scores[t] for the `window` last positions, which never enter a prefix tap (with
 * kvp_score_tokens(force_window=1) they hold +inf).  kernel is odd, 1 <= kernel <= 63;
 * 0 <= window <= T; out (device fp32, rows out_stride floats apart) must not overlap scores. */
enum { KVP_SMOOTH_AVG = 0, KVP_SMOOTH_MAX = 1 };
int32_t kvp_smooth_scores(const float* scores, int64_t n_rows, int64_t T, int64_t row_stride, int64_t window,
                          int32_t kernel, int32_t mode, float* out, int64_t out_stride, void* stream);

/* Quality-loss proxy for every candidate configuration of ONE context
 * (System design, profiler module: every KV cache is compressed with each
 * method and ratio of the pool and every version is scored; utility function:
 * the quality term).  For config c = (bits, group, keep_k):
 *     O_full = softmax(Q K^T / sqrt(D)) V          (causal, the W window rows)
 *     O_c    = the same with K, V replaced by dequantize(quantize(.)) at
 *              (bits, group) and the keys restricted to the top-keep_k keep-set
 *              of kvp_score_tokens(causal=1, force_window=1) on the unquantized K
 *     loss[c] = sqrt( sum (O_c - O_full)^2 / sum O_full^2 )
 * sums over layers, query heads, window rows and channels.  cfgs is a HOST
 * array; loss is device fp32 [n_cfgs]; partial is NULL or device fp32
 * [L][n_cfgs][2] = (numerator, denominator) per layer.  At most 64 configurations and 8 distinct
 * keep_k values per call (KVP_ERR_UNSUPPORTED beyond), and the limits of kvp_score_tokens.  The workspace holds the scores, the keep lists and one fp32 output
 * (64 KiB per 128 window rows) per (layer, kv head, distinct codec, keep level): about 1.5 GB for
 * 40 configurations of a 32-layer, 8-kv-head context; ask kvp_eval_workspace_bytes. */
int32_t kvp_eval_configs(const kvp_view* q_win, const kvp_view* k, const kvp_view* v, const kvp_config* cfgs,
                         int32_t n_cfgs, float* loss, float* partial, void* ws, size_t ws_bytes, void* stream);
size_t kvp_eval_workspace_bytes(int64_t L, int64_t Hkv, int64_t Hq, int64_t W, int64_t T, int32_t n_cfgs);

/* The same computation with implementation flags (0 = kvp_eval_configs).  The flags choose how the P.V
 * product of the proxy is formed; logits, softmax statistics and accumulation are fp32 in every mode.
 * 0 (default): vector ALU with 16-bit operands: the probabilities rounded to fp16 (nearest even; the row sums
 *   use the rounded values) and V-hat as fp16, two tokens per v_dot2_f32_f16.  V-hat is a bf16 value and exact in
 *   fp16 for 2^-14 <= |v| <= 65504; smaller magnitudes round to multiples of 2^-24 and larger ones become infinite
 *   (the losses then come out non-finite), so caches with |V| beyond that range need one of the other modes.  Losses agree with KVP_EVAL_PV_FP32 within
 *   1e-4 relative (3e-5 measured on the 40-configuration sweep).
 * KVP_EVAL_PV_FP32: vector ALU with fp32 probabilities and V-hat, one fma per token and output; 1.2x slower.
 * KVP_EVAL_PV_MATRIX_CORES: on the matrix cores (P as the sum of two bf16 terms, relative error 2^-18); the
 *   fastest; agrees with KVP_EVAL_PV_FP32 within 1e-5 relative.  Not the default because the scope of this
 *   library reserves the matrix cores for the query-window x key contraction.
 * The two flags exclude each other; both set, or unknown flag bits: KVP_ERR_UNSUPPORTED. */
enum { KVP_EVAL_PV_MATRIX_CORES = 1, KVP_EVAL_PV_FP32 = 2 };
int32_t kvp_eval_configs_ex(const kvp_view* q_win, const kvp_view* k, const kvp_view* v, const kvp_config* cfgs,
                            int32_t n_cfgs, float* loss, float* partial, void* ws, size_t ws_bytes, uint32_t flags,
                            void* stream);

/* One sizing call for every entry point that takes (ws, ws_bytes): the bytes the call needs for the
 * sizes in `dims` (fields an operation does not use are ignored), 0 if it needs none or the sizes
 * are invalid.  The kvp_*_workspace_bytes helpers above return the same numbers. */
enum {
  KVP_WS_SCORE_TOKENS = 0, /* L, Hkv, Hq, W, T */
  KVP_WS_SCORE_KEYS = 1,   /* L, Hkv (= H), T, method */
  KVP_WS_SELECT_TOPK = 2,  /* n_rows, T, k */
  KVP_WS_EVAL_CONFIGS = 3  /* L, Hkv, Hq, W, T, n_cfgs */
};
typedef struct {
  int64_t L, Hkv, Hq, W, T; /* layers, kv heads, query heads, window rows, tokens */
  int64_t n_rows, k;        /* kvp_select_topk */
  int32_t n_cfgs;           /* kvp_eval_configs */
  int32_t method;           /* kvp_score_keys */
} kvp_dims;
size_t kvp_workspace_bytes(int32_t op, const kvp_dims* dims);

/* ---- policy layer on the HOST (all pointers below are host pointers; no kernel is launched) ----
 *
 * Utility of a stored configuration (System design, "Utility function"):
 *     Util(config, tier) = (alpha * quality - TTFT) * frequency,  TTFT = bytes / tier bandwidth
 * quality is 1 - loss of kvp_eval_configs (or any quality score in [0, 1]). */
typedef struct {
  double capacity_bytes;        /* negative = unbounded */
  double bandwidth_bytes_per_s; /* loading bandwidth towards the GPU, > 0 */
} kvp_tier;

/* util[tier][cfg] for one context.  quality, bytes: [n_cfg]; util: [n_tiers][n_cfg]. */
int32_t kvp_utility_table(const double* quality, const double* bytes, int32_t n_cfg, const kvp_tier* tiers,
                          int32_t n_tiers, double alpha, double frequency, double* util);

enum { KVP_OP_INSERT = 0, KVP_OP_COMPRESS = 1, KVP_OP_EVICT = 2 };
typedef struct {
  int32_t ctx, cfg, tier, op; /* context, its configuration after the operation, the tier it is on after it
                                 (-1: evicted from the last tier, no longer stored) */
} kvp_policy_op;

/* Greedy placement (appendix, Policy Optimizer; "Eviction-compression configuration selection
 * module").  Context `incoming` enters tier 0 with its highest-quality configuration (fewest
 * bytes, then lowest index, among equals).  Then every bounded tier, first to last, is brought
 * under its capacity by repeatedly applying the operation with the least utility drop among: re-
 * compressing a cache on the tier to a configuration with fewer bytes, or evicting it: unchanged to
 * the next tier, or, from the last tier, out of storage (tier -1 in the operation and in ctx_tier;
 * a cache that is not stored earns utility 0, so the drop is its current utility).  Ties: lowest
 * context, compress before evict, lowest configuration.  This is the appendix algorithm's pair of
 * single operations; the wider option set of the selection-module text (any method and ratio
 * combined with a move to any lower tier in one step) is not searched.
 * bytes, quality: [n_ctx][n_cfg]; frequency: [n_ctx]; ctx_tier (-1 = not stored) and ctx_cfg:
 * [n_ctx], updated in place.  The operations are written to ops (at most max_ops) and counted in
 * *n_ops.  Every bounded tier fits on return.
 * KVP_ERR_WORKSPACE if max_ops is too small (the state then reflects the operations written). */
int32_t kvp_policy_insert(int32_t n_ctx, int32_t n_cfg, const double* bytes, const double* quality,
                          const double* frequency, const kvp_tier* tiers, int32_t n_tiers, double alpha,
                          int32_t* ctx_tier, int32_t* ctx_cfg, int32_t incoming, kvp_policy_op* ops,
                          int32_t max_ops, int32_t* n_ops);

/* Host helper: tokens kept at a keep-ratio = ceil(ratio * T) in double, clamped to [1, T]. */
int64_t kvp_keep_count(double ratio, int64_t T);

/* Plain device-to-device copy kernel (nbytes a multiple of 16, both pointers
 * 16-byte aligned).  Not part of the method: it is the yardstick the benchmark
 * and the hardware-counter calibration compare the streaming kernels with. */
int32_t kvp_copy_bytes(void* dst, const void* src, size_t nbytes, void* stream);

/* Self-test of an arithmetic identity of this build: the asymmetric quantizer forms fl32(1 / scale) as the
 * hardware reciprocal estimate plus one fma correction step instead of a division.  The call compares that with
 * the IEEE quotient 1.0f / s for every binary32 s in [2^-60, 2^61) (2^23 significands x 121 exponents, about
 * 0.3 s of GPU time) and ADDS the number of operands that differ to *mismatches (device memory, 8-byte aligned,
 * cleared by the caller).  0 on gfx950; a GPU test asserts it, so a part or a compiler that rounds differently
 * is noticed before any code depends on it. */
int32_t kvp_selftest_reciprocal(uint64_t* mismatches, void* stream);

const char* kvp_strerror(int32_t code);
/* 0x00MMmmpp.  1.3: kvp_qplane carries mins and group_axis; scatter restore, score smoothing and
 * kvp_eval_configs_ex exist.  1.4: kvp_select_topk uses its workspace for long rows; kvp_dims,
 * kvp_workspace_bytes and kvp_score_tokens_static exist.  1.5: KVP_EVAL_PV_FP32, tier -1 in kvp_policy_op,
 * kvp_selftest_reciprocal. */
uint32_t kvp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KVP_H_ */
