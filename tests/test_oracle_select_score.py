"""Pins for the oracle's token scoring and top-k keep-set (CPU only).

The paper describes attention-score token dropping in one sentence
(Evaluation, Baselines: snapkv; IMPRESS keeps the top X% by attention score).
The pins: brute force and a library stable sort for the selection; closed
forms, the row-sum invariant and a library float64 softmax for the scores.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import bits_to_f32, to_bf16_bits, torch_bits


# ---------------------------------------------------------------- top-k

def _brute_topk(s: np.ndarray, k: int):
    """k rounds of 'largest remaining score, lowest index among equals', then ascending."""
    alive = list(range(len(s)))
    out = []
    for _ in range(k):
        best = alive[0]
        for i in alive[1:]:
            if s[i] > s[best]:
                best = i
        out.append(best)
        alive.remove(best)
    return sorted(out)


@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force_and_stable_sort(seed):
    rng = np.random.default_rng(seed)
    T = int(rng.integers(1, 33))
    kinds = [rng.standard_normal(T), rng.integers(0, 3, T).astype(float), np.zeros(T), np.arange(T, dtype=float),
             -np.arange(T, dtype=float)]
    for s in kinds:
        s = s.astype(np.float32)
        if T > 4:
            s[-2:] = np.inf                       # forced-window style +inf run
        for k in sorted({0, 1, T // 2, max(T - 1, 0), T}):
            got = oracle.select_topk(s.reshape(1, T), k)[0].tolist()
            assert got == _brute_topk(s, k)
            lib = np.sort(np.argsort(-s.astype(np.float64), kind="stable")[:k]).tolist()
            assert got == lib


def test_topk_properties_and_ties():
    s = workloads.make_scores(5, 1000, seed=1, levels=3).numpy()
    s[0, :] = 1.0                                  # all equal: keeps the first k indices
    for k in (1, 333, 334, 999, 1000):
        idx = oracle.select_topk(s, k)
        assert idx.shape == (5, k)
        assert idx[0].tolist() == list(range(k))
        for r in range(5):
            kept = idx[r]
            assert np.all(np.diff(kept) > 0)                       # ascending, distinct
            mask = np.zeros(1000, bool)
            mask[kept] = True
            if k < 1000:
                thr = s[r][mask].min()
                assert thr >= s[r][~mask].max()                    # every kept >= every dropped
                # among scores equal to the threshold the kept ones are the lowest-indexed
                eq = np.flatnonzero(s[r] == thr)
                kept_eq = eq[mask[eq]]
                assert np.array_equal(kept_eq, eq[: len(kept_eq)])


def test_topk_strided_rows_and_tie_run_boundaries():
    base = np.zeros((3, 64), dtype=np.float32)
    base[:, 10:20] = 2.0
    base[:, 30:50] = 1.0
    view = base[:, :48]                            # row stride 64, T = 48
    for k, want in [(9, list(range(10, 19))), (10, list(range(10, 20))), (11, list(range(10, 20)) + [30]),
                    (28, list(range(10, 20)) + list(range(30, 48))), (29, [0] + list(range(10, 20)) + list(range(30, 48)))]:
        got = oracle.select_topk(view, k)
        assert all(row.tolist() == sorted(want) for row in got)


# ---------------------------------------------------------------- scores

def _rand_qk(L, W, G, H, T, D, seed):
    K, _ = workloads.make_kv(L, T, H, D, seed=seed)
    Q = workloads.make_q(L, W, G * H, D, seed=seed)
    return torch_bits(Q), torch_bits(K)


def test_scores_row_sum_invariant():
    L, W, G, H, T, D = 2, 4, 2, 2, 50, 32
    q, k = _rand_qk(L, W, G, H, T, D, 0)
    for causal in (True, False):
        s = oracle.score_tokens(q, k, causal=causal, force_window=False)
        assert np.allclose(s.sum(-1), G * W, rtol=1e-5)
        assert np.all(s >= 0)
    # the causal mask removes exactly the keys after each window row's position
    s = oracle.score_tokens(q, k, causal=True, force_window=False)
    s_nc = oracle.score_tokens(q, k, causal=False, force_window=False)
    assert not np.allclose(s, s_nc)
    f = oracle.score_tokens(q, k, causal=True, force_window=True)
    assert np.all(np.isposinf(f[..., T - W:])) and np.array_equal(f[..., :T - W], s[..., :T - W])


def test_scores_closed_form_zero_queries():
    # Q = 0: every allowed key gets the same probability 1/(T-W+w+1) in window row w
    L, W, G, H, T, D = 1, 5, 3, 2, 23, 16
    _, k = _rand_qk(L, W, G, H, T, D, 1)
    q = np.zeros((L, W, G * H, D), dtype=np.uint16)
    s = oracle.score_tokens(q, k, causal=True, force_window=False)
    want = np.zeros(T)
    for t in range(T):
        for w in range(W):
            if t <= T - W + w:
                want[t] += G / (T - W + w + 1)
    assert np.allclose(s[0, 0], want, rtol=1e-6) and np.allclose(s[0, 1], want, rtol=1e-6)
    s_nc = oracle.score_tokens(q, k, causal=False, force_window=False)
    assert np.allclose(s_nc, G * W / T, rtol=1e-6)


def test_scores_peaked_key():
    # one key aligned with every query (30 x the unit query), all other keys zero
    L, W, G, H, T, D = 1, 3, 2, 1, 40, 64
    rng = np.random.default_rng(0)
    qdir = rng.standard_normal(D).astype(np.float32)
    qdir = qdir / np.linalg.norm(qdir) * np.sqrt(D)
    q = np.broadcast_to(to_bf16_bits(qdir), (L, W, G * H, D)).copy()
    kf = np.zeros((L, T, H, D), dtype=np.float32)
    kf[0, 7, 0] = 30.0 * bits_to_f32(q[0, 0, 0]) / np.sqrt(D)
    s = oracle.score_tokens(q, to_bf16_bits(kf).reshape(L, T, H, D), causal=True, force_window=False)
    assert abs(s[0, 0, 7] - G * W) < 1e-6 * G * W
    assert s[0, 0].sum() - s[0, 0, 7] < 1e-6


@pytest.mark.parametrize("causal", [True, False])
def test_scores_match_library_softmax(causal):
    L, W, G, H, T, D = 2, 4, 2, 3, 37, 32
    q, k = _rand_qk(L, W, G, H, T, D, 2)
    s = oracle.score_tokens(q, k, causal=causal, force_window=False)
    qf = torch.from_numpy(bits_to_f32(q)).double()
    kf = torch.from_numpy(bits_to_f32(k)).double()
    for l in range(L):
        for h in range(H):
            logits = torch.einsum("wud,td->uwt", qf[l][:, h * G:(h + 1) * G], kf[l][:, h]) / D ** 0.5
            if causal:
                pos = (T - W + torch.arange(W)).view(1, W, 1)
                logits = logits.masked_fill(torch.arange(T).view(1, 1, T) > pos, float("-inf"))
            want = torch.softmax(logits, dim=-1).sum((0, 1)).numpy()
            assert np.allclose(s[l, h], want, rtol=1e-6, atol=1e-9)


def test_scores_strided_views_and_window_equals_context():
    L, W, G, H, T, D = 1, 6, 2, 2, 6, 16          # W == T: every row is a window row
    q, k = _rand_qk(L, W, G, H, T, D, 3)
    s = oracle.score_tokens(q, k, causal=True, force_window=True)
    assert np.all(np.isposinf(s))
    big = np.zeros((L, T, H + 1, D), dtype=np.uint16)
    big[:, :, :H] = k
    a = oracle.score_tokens(q, big[:, :, :H], causal=True, force_window=False)
    b = oracle.score_tokens(q, k, causal=True, force_window=False)
    assert np.array_equal(a, b)
