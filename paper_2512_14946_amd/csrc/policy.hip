// Host-side policy layer that consumes the quality-loss table (paper: System design, "Utility
// function: Balancing quality and loading delay"; "Eviction-compression configuration selection
// module"; appendix, Policy Optimizer).  Scalar work on host arrays: no kernel is launched.
//
//   Util(config, tier) = (alpha * quality - TTFT) * frequency,  TTFT = bytes / tier bandwidth
//
// kvp_policy_insert stores one incoming cache and then, tier by tier, applies the operation with
// the least utility drop (re-compress on the tier, or evict: unchanged to the next tier, or out of
// storage from the last tier, where the cache's utility becomes 0) until the tier fits, as the paper's
// greedy loop does.  Occupancy is kept incrementally; the candidate scan
// is O(contexts x configs) per operation.

#include <vector>

#include "kvp_common.h"

namespace {

inline double util_of(double alpha, double quality, double bytes, double bandwidth, double frequency) {
  return (alpha * quality - bytes / bandwidth) * frequency;
}

}  // namespace

extern "C" int32_t kvp_utility_table(const double* quality, const double* bytes, int32_t n_cfg, const kvp_tier* tiers,
                                     int32_t n_tiers, double alpha, double frequency, double* util) {
  if (!quality || !bytes || !tiers || !util) return KVP_ERR_NULL;
  if (n_cfg < 0 || n_tiers <= 0) return KVP_ERR_SHAPE;
  for (int32_t d = 0; d < n_tiers; ++d) {
    if (!(tiers[d].bandwidth_bytes_per_s > 0.0)) return KVP_ERR_SHAPE;
    for (int32_t c = 0; c < n_cfg; ++c)
      util[static_cast<int64_t>(d) * n_cfg + c] = util_of(alpha, quality[c], bytes[c], tiers[d].bandwidth_bytes_per_s, frequency);
  }
  return KVP_OK;
}

extern "C" int32_t kvp_policy_insert(int32_t n_ctx, int32_t n_cfg, const double* bytes, const double* quality,
                                     const double* frequency, const kvp_tier* tiers, int32_t n_tiers, double alpha,
                                     int32_t* ctx_tier, int32_t* ctx_cfg, int32_t incoming, kvp_policy_op* ops,
                                     int32_t max_ops, int32_t* n_ops) {
  if (!bytes || !quality || !frequency || !tiers || !ctx_tier || !ctx_cfg || !ops || !n_ops) return KVP_ERR_NULL;
  if (n_ctx <= 0 || n_cfg <= 0 || n_tiers <= 0 || incoming < 0 || incoming >= n_ctx || max_ops < 1) return KVP_ERR_SHAPE;
  for (int32_t d = 0; d < n_tiers; ++d)
    if (!(tiers[d].bandwidth_bytes_per_s > 0.0)) return KVP_ERR_SHAPE;
  for (int32_t j = 0; j < n_ctx; ++j)
    if (ctx_tier[j] >= n_tiers || (ctx_tier[j] >= 0 && (ctx_cfg[j] < 0 || ctx_cfg[j] >= n_cfg))) return KVP_ERR_SHAPE;
  auto B = [&](int32_t j, int32_t c) { return bytes[static_cast<int64_t>(j) * n_cfg + c]; };
  auto Q = [&](int32_t j, int32_t c) { return quality[static_cast<int64_t>(j) * n_cfg + c]; };

  // the incoming cache enters the first tier at its best quality (fewest bytes among equals)
  int32_t best = 0;
  for (int32_t c = 1; c < n_cfg; ++c)
    if (Q(incoming, c) > Q(incoming, best) || (Q(incoming, c) == Q(incoming, best) && B(incoming, c) < B(incoming, best)))
      best = c;
  ctx_tier[incoming] = 0;
  ctx_cfg[incoming] = best;
  int32_t count = 0;
  ops[count++] = kvp_policy_op{incoming, best, 0, KVP_OP_INSERT};

  std::vector<int32_t> members;
  for (int32_t d = 0; d < n_tiers; ++d) {
    const double cap = tiers[d].capacity_bytes;
    if (cap < 0.0) continue;  // unbounded
    const double bw = tiers[d].bandwidth_bytes_per_s;
    const bool has_next = d + 1 < n_tiers;
    members.clear();
    for (int32_t j = 0; j < n_ctx; ++j)
      if (ctx_tier[j] == d) members.push_back(j);
    for (;;) {
      // summed in context order on every round, as the definition does (no drift from running updates)
      double occupied = 0.0;
      for (int32_t j : members) occupied += B(j, ctx_cfg[j]);
      if (occupied <= cap) break;
      bool found = false;
      double best_drop = 0.0;
      int32_t best_j = -1, best_c = -1, best_op = -1;
      for (int32_t j : members) {
        const int32_t cur = ctx_cfg[j];
        const double u_now = util_of(alpha, Q(j, cur), B(j, cur), bw, frequency[j]);
        for (int32_t c = 0; c < n_cfg; ++c) {
          if (!(B(j, c) < B(j, cur))) continue;  // keeps the cache here without saving space
          const double drop = u_now - util_of(alpha, Q(j, c), B(j, c), bw, frequency[j]);
          if (!found || drop < best_drop) {
            found = true; best_drop = drop; best_j = j; best_c = c; best_op = KVP_OP_COMPRESS;
          }
        }
        {
          // evict: to the next tier unchanged, or, from the last tier, out of storage (the appendix's evict sets the
          // stored ratio to 0: the cache leaves the queue; a cache that is not stored earns no utility)
          const double u_after =
              has_next ? util_of(alpha, Q(j, cur), B(j, cur), tiers[d + 1].bandwidth_bytes_per_s, frequency[j]) : 0.0;
          const double drop = u_now - u_after;
          if (!found || drop < best_drop) {
            found = true; best_drop = drop; best_j = j; best_c = cur; best_op = KVP_OP_EVICT;
          }
        }
      }
      if (!found) { *n_ops = count; return KVP_ERR_SHAPE; }        // over capacity with no member: negative sizes
      if (count == max_ops) { *n_ops = count; return KVP_ERR_WORKSPACE; }
      if (best_op == KVP_OP_COMPRESS) {
        ctx_cfg[best_j] = best_c;
        ops[count++] = kvp_policy_op{best_j, best_c, d, KVP_OP_COMPRESS};
      } else {
        const int32_t to = has_next ? d + 1 : -1;
        ctx_tier[best_j] = to;
        ops[count++] = kvp_policy_op{best_j, best_c, to, KVP_OP_EVICT};
        for (size_t i = 0; i < members.size(); ++i)
          if (members[i] == best_j) { members.erase(members.begin() + static_cast<long>(i)); break; }
      }
    }
  }
  *n_ops = count;
  return KVP_OK;
}
