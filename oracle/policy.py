"""CPU oracle of the policy layer that consumes the quality-loss table: the utility function and the
greedy placement (paper: System design, "Utility function"; "Eviction-compression configuration
selection module"; appendix "Pseudo Code for Algorithm", Policy Optimizer).

TEST INFRASTRUCTURE ONLY, plain Python loops, no code shared with the library.

Readings (the paper leaves them open):
  * TTFT of a stored configuration = its bytes / the tier's loading bandwidth (the delay term of
    the utility "is computed with estimated latency to fetch a (compressed) KV cache"; the worked
    two-context figure adds such terms).  The prefill of the new query is the same for every
    configuration and is left out.
  * An incoming cache enters the first tier with its highest-quality configuration (fewest bytes,
    then lowest index, among equals).
  * While a tier is over capacity, the operation with the least utility drop is applied: either
    re-compress a cache on that tier to a configuration with fewer bytes, or evict it: unchanged to
    the next tier, or, from the last tier, out of storage (the appendix's evict sets the stored ratio
    to 0; a cache that is not stored has utility 0; tier -1).  Ties: lowest context index, compress
    before evict, lowest configuration index.
  * Tiers are settled from the first to the last; a negative capacity means unbounded.
Parity status: pinned by the paper's printed utility examples and its two-context figure
(tests/golden/policy_examples.txt), plus hand-worked cascades for the tie order and the last-tier eviction.
"""
from __future__ import annotations

INSERT, COMPRESS, EVICT = 0, 1, 2


def ttft(nbytes: float, bandwidth: float) -> float:
    return nbytes / bandwidth


def utility(alpha: float, quality: float, delay: float, frequency: float) -> float:
    """Util = (alpha * quality - TTFT) * frequency."""
    return (alpha * quality - delay) * frequency


def utility_table(quality, nbytes, tiers, alpha, frequency):
    """tiers: [(capacity_bytes, bandwidth_bytes_per_s)] -> util[tier][cfg]."""
    return [[utility(alpha, quality[c], ttft(nbytes[c], bw), frequency) for c in range(len(quality))]
            for (_, bw) in tiers]


def insert(nbytes, quality, frequency, tiers, alpha, ctx_tier, ctx_cfg, incoming):
    """Store context `incoming`; returns the list of (ctx, cfg, tier, op).  ctx_tier / ctx_cfg are updated in place."""
    n_cfg = len(nbytes[incoming])
    best = 0
    for c in range(1, n_cfg):
        if (quality[incoming][c] > quality[incoming][best] or
                (quality[incoming][c] == quality[incoming][best] and nbytes[incoming][c] < nbytes[incoming][best])):
            best = c
    ctx_tier[incoming], ctx_cfg[incoming] = 0, best
    ops = [(incoming, best, 0, INSERT)]
    for d in range(len(tiers)):
        cap, bw = tiers[d]
        if cap < 0:
            continue
        while True:
            occupied = 0.0
            for j in range(len(ctx_tier)):
                if ctx_tier[j] == d:
                    occupied += nbytes[j][ctx_cfg[j]]
            if occupied <= cap:
                break
            choice = None  # (drop, ctx, op, cfg)
            for j in range(len(ctx_tier)):
                if ctx_tier[j] != d:
                    continue
                cur = ctx_cfg[j]
                u_now = utility(alpha, quality[j][cur], ttft(nbytes[j][cur], bw), frequency[j])
                for c in range(len(nbytes[j])):
                    if nbytes[j][c] < nbytes[j][cur]:
                        drop = u_now - utility(alpha, quality[j][c], ttft(nbytes[j][c], bw), frequency[j])
                        if choice is None or drop < choice[0]:
                            choice = (drop, j, COMPRESS, c)
                if d + 1 < len(tiers):
                    u_after = utility(alpha, quality[j][cur], ttft(nbytes[j][cur], tiers[d + 1][1]), frequency[j])
                else:
                    u_after = 0.0          # leaves storage
                drop = u_now - u_after
                if choice is None or drop < choice[0]:
                    choice = (drop, j, EVICT, cur)
            if choice is None:
                raise ValueError("over capacity with nothing stored")
            _, j, op, c = choice
            if op == COMPRESS:
                ctx_cfg[j] = c
                ops.append((j, c, d, COMPRESS))
            else:
                to = d + 1 if d + 1 < len(tiers) else -1
                ctx_tier[j] = to
                ops.append((j, c, to, EVICT))
    return ops
