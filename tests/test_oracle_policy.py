"""Pins for the policy oracle (utility function and greedy placement) against the numbers the
paper prints (tests/golden/policy_examples.txt)."""
import os

import pytest

from oracle import policy

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "policy_examples.txt")
GB = 1e9


def _rows(kind):
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            parts = [p.strip() for p in line.split("|")]
            if parts[0] == kind:
                out.append(parts[1:])
    return out


def test_printed_utility_values():
    vals = []
    for alpha, q, t, printed in _rows("utility"):
        u = policy.utility(float(alpha), float(q), float(t), 1.0)
        assert abs(u - float(printed)) <= 0.01
        vals.append(u)
    assert vals[0] < vals[1]                 # the lower-quality configuration at equal TTFT is strictly worse
    assert policy.utility(1.0, 0.65, 0.05, 3.0) == pytest.approx(3 * vals[0])   # frequency scales the score


def test_alpha_trade_off():
    (qa, ta, qb, tb), = _rows("tradeoff")
    qa, ta, qb, tb = map(float, (qa, ta, qb, tb))
    for alpha in (0.0, 0.1, 0.3):
        assert policy.utility(alpha, qa, ta, 1.0) > policy.utility(alpha, qb, tb, 1.0)
    for alpha in (0.41, 0.5, 1.0, 5.0):
        assert policy.utility(alpha, qa, ta, 1.0) < policy.utility(alpha, qb, tb, 1.0)


def _figure_instance():
    # configs per context: kept fraction 1.0, 0.5, 0.05
    nbytes = [[4 * GB, 2 * GB, 0.2 * GB], [8 * GB, 4 * GB, 0.4 * GB]]
    quality = [[1.0, 1.0, 1.0], [1.0, 0.5, 0.5]]
    tiers = [(8 * GB, 20 * GB), (-1.0, 2 * GB)]
    return nbytes, quality, tiers


def test_two_context_figure_arithmetic_and_greedy_outcome():
    nbytes, quality, tiers = _figure_instance()
    want = {r[0]: (float(r[1]), float(r[2])) for r in _rows("figure")}
    fast, slow = tiers[0][1], tiers[1][1]
    # the three schemes of the figure, straight from bytes / bandwidth
    t = policy.ttft(nbytes[0][1], fast) + policy.ttft(nbytes[1][1], fast)
    assert t == pytest.approx(want["compress_only"][0]) and (quality[0][1] + quality[1][1]) / 2 == want["compress_only"][1]
    t = policy.ttft(nbytes[0][0], slow) + policy.ttft(nbytes[1][0], fast)
    assert t == pytest.approx(want["evict_only"][0])
    t = policy.ttft(nbytes[0][2], slow) + policy.ttft(nbytes[1][0], fast)
    assert t == pytest.approx(want["joint"][0])
    # the greedy placement reaches the joint scheme
    ctx_tier, ctx_cfg = [-1, -1], [0, 0]
    ops = policy.insert(nbytes, quality, [1.0, 1.0], tiers, 1.0, ctx_tier, ctx_cfg, 0)
    assert ops == [(0, 2, 0, policy.INSERT)]          # all three versions keep 100 %: the smallest enters
    ops = policy.insert(nbytes, quality, [1.0, 1.0], tiers, 1.0, ctx_tier, ctx_cfg, 1)
    assert ops == [(1, 0, 0, policy.INSERT), (0, 2, 1, policy.EVICT)]
    # starting from both caches uncompressed in fast memory (the figure's starting point) the loop
    # first compresses the insensitive cache, then evicts it
    ctx_tier, ctx_cfg = [0, -1], [0, 0]
    ops = policy.insert(nbytes, quality, [1.0, 1.0], tiers, 1.0, ctx_tier, ctx_cfg, 1)
    assert ops == [(1, 0, 0, policy.INSERT), (0, 2, 0, policy.COMPRESS), (0, 2, 1, policy.EVICT)]
    assert ctx_tier == [1, 0] and ctx_cfg == [2, 0]
    total = sum(policy.ttft(nbytes[j][ctx_cfg[j]], tiers[ctx_tier[j]][1]) for j in range(2))
    mean_q = sum(quality[j][ctx_cfg[j]] for j in range(2)) / 2
    assert total == pytest.approx(want["joint"][0]) and mean_q == want["joint"][1]


def test_unbounded_first_tier_needs_no_operation_and_overfull_last_tier_evicts_out_of_storage():
    nbytes, quality, _ = _figure_instance()
    ctx_tier, ctx_cfg = [-1, -1], [0, 0]
    for i in range(2):
        ops = policy.insert(nbytes, quality, [1.0, 1.0], [(-1.0, 20 * GB)], 1.0, ctx_tier, ctx_cfg, i)
        assert len(ops) == 1 and ops[0][3] == policy.INSERT
    # a single bounded tier that nothing fits: the cache is compressed as far as that lowers the drop, then leaves
    ctx_tier, ctx_cfg = [-1, -1], [0, 0]
    ops = policy.insert(nbytes, quality, [1.0, 1.0], [(0.1 * GB, 20 * GB)], 1.0, ctx_tier, ctx_cfg, 0)
    assert ops[-1][2] == -1 and ops[-1][3] == policy.EVICT and ctx_tier == [-1, -1]


def _golden_ops(kind):
    return [tuple(int(x) for x in r) for r in _rows(kind)]


def test_three_tier_cascade_and_tie_order_worked_by_hand():
    # the instance and every candidate's utility drop are written out in the golden file
    nbytes = [[4 * GB, 2 * GB], [4 * GB, 2 * GB], [4 * GB, 2 * GB], [2 * GB, 1 * GB]]
    quality = [[1.0, 0.5], [1.0, 0.5], [1.0, 0.25], [1.0, 0.5]]
    tiers = [(8 * GB, 8 * GB), (3 * GB, 4 * GB), (-1.0, 1 * GB)]
    ctx_tier, ctx_cfg = [0, 0, -1, 1], [0, 0, 0, 0]
    ops = policy.insert(nbytes, quality, [1.0] * 4, tiers, 1.0, ctx_tier, ctx_cfg, 2)
    assert ops == _golden_ops("three_tiers")
    assert ctx_tier == [1, 0, 0, 1] and ctx_cfg == [1, 0, 0, 1]
    # the drops the derivation lists, from the utility function alone
    u = policy.utility
    assert u(1.0, 1.0, policy.ttft(4 * GB, 8 * GB), 1.0) - u(1.0, 0.5, policy.ttft(2 * GB, 8 * GB), 1.0) == 0.25
    assert u(1.0, 0.5, policy.ttft(2 * GB, 8 * GB), 1.0) - u(1.0, 0.5, policy.ttft(2 * GB, 4 * GB), 1.0) == 0.25
    assert u(1.0, 1.0, policy.ttft(2 * GB, 4 * GB), 1.0) - u(1.0, 1.0, policy.ttft(2 * GB, 1 * GB), 1.0) == 1.5


def test_eviction_from_the_last_tier_worked_by_hand():
    nbytes, quality = [[2 * GB, 1 * GB], [4 * GB, 2 * GB]], [[1.0, 0.5], [1.0, 0.5]]
    ctx_tier, ctx_cfg = [0, -1], [0, 0]
    ops = policy.insert(nbytes, quality, [2.0, 1.0], [(2 * GB, 4 * GB)], 1.0, ctx_tier, ctx_cfg, 1)
    assert ops == _golden_ops("last_tier_evict")
    assert ctx_tier == [0, -1] and ctx_cfg == [0, 1]
    u = policy.utility                                  # the drops of the derivation, from the utility function alone
    assert u(1.0, 1.0, policy.ttft(2 * GB, 4 * GB), 2.0) == 1.0
    assert u(1.0, 1.0, policy.ttft(2 * GB, 4 * GB), 2.0) - u(1.0, 0.5, policy.ttft(1 * GB, 4 * GB), 2.0) == 0.5
    assert u(1.0, 1.0, policy.ttft(4 * GB, 4 * GB), 1.0) == 0.0 and u(1.0, 0.5, policy.ttft(2 * GB, 4 * GB), 1.0) == 0.0


def test_equal_drops_inside_one_context_compress_first_lowest_configuration():
    nbytes, quality = [[4 * GB, 2 * GB, 2 * GB]], [[1.0, 0.25, 0.25]]
    tiers = [(3 * GB, 8 * GB), (-1.0, 4 * GB)]
    ctx_tier, ctx_cfg = [-1], [0]
    ops = policy.insert(nbytes, quality, [1.0], tiers, 1.0, ctx_tier, ctx_cfg, 0)
    assert ops == _golden_ops("one_context_tie")
    assert ctx_tier == [0] and ctx_cfg == [1]
