"""GPU parity: kvp_select_topk (bit-exact on identical score buffers) and kvp_score_tokens
(1e-2 relative, +inf exact) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import torch_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _kvp():
    import paper_2512_14946_amd as kvp
    return kvp


def _say(*a):
    print("[case]", *a, flush=True)


# ---------------------------------------------------------------- top-k

def _check_topk(s: np.ndarray, k: int, view=None):
    kvp = _kvp()
    t = torch.from_numpy(s).to(DEV) if view is None else view
    got = kvp.kvp_select_topk(t, k)
    torch.cuda.synchronize()
    want = oracle.select_topk(s, k)
    assert np.array_equal(got.cpu().numpy(), want)


@pytest.mark.parametrize("T", [1, 7, 64, 1000, 4096, 5003, 16384])
def test_topk_random_and_ties(T):
    _say("topk", T)
    for seed, levels in [(0, None), (1, 3), (2, 1)]:
        s = workloads.make_scores(5, T, seed=seed, levels=levels).numpy()
        if T > 40:
            s[:, T - 32:] = np.inf                                    # forced window
        if levels is None and T > 8:
            s[1, ::3] = -s[1, ::3]                                    # negative scores
            s[2, 1::2] = 0.0
            s[2, 0::4] = -0.0                                         # signed zeros tie
            s[3, :] = np.float32(1e-42) * np.arange(T, dtype=np.float32)  # subnormals
        for k in sorted({0, 1, T // 3, T // 2, max(T - 1, 0), T}):
            _check_topk(s, k)


def test_topk_strided_rows_unaligned():
    _say("topk strided")
    kvp = _kvp()
    base = workloads.make_scores(6, 1031, seed=4, levels=5).to(DEV)
    view = base[:, :1001]                                             # row stride 1031: rows not 16 B aligned
    got = kvp.kvp_select_topk(view, 400)
    torch.cuda.synchronize()
    want = oracle.select_topk(base.cpu().numpy()[:, :1001], 400)
    assert np.array_equal(got.cpu().numpy(), want)


@pytest.mark.parametrize("T", [9, 3000, 8195, 16384])
def test_topk_many_rows(T):
    """More rows than the chip holds wide blocks for: the narrower block shape (8 items per thread)."""
    _say("topk many rows", T)
    rows = 530
    s = workloads.make_scores(rows, T, seed=T).numpy()
    s[1::7] = np.round(s[1::7] * 8) / 8                                # rows with heavy ties
    s[2::7, ::2] = 0.0
    if T > 40:
        s[::3, T - 32:] = np.inf
    for k in sorted({1, T // 3, T - 1, T}):
        _check_topk(s, k)


def test_topk_long_rows_many_ties():
    _say("topk long")
    T = 131072
    s = workloads.make_scores(3, T, seed=5).numpy()
    s[1] = np.round(s[1] * 4) / 4                                     # heavy ties
    s[:, T - 32:] = np.inf
    _check_topk(s, 13108)
    _check_topk(s, T - 5)


def _long_rows(T, seed):
    """Rows that take every branch of the split-row path: plain random scores, few ties, heavy ties at the
    threshold (more candidates than a span's slice holds: the row is redone by the streaming kernel), one value
    only, sorted both ways, negative scores with signed zeros, a forced +inf window."""
    s = workloads.make_scores(9, T, seed=seed).numpy()
    s[1] = np.round(s[1] * 64) / 64                                   # a few hundred levels
    s[2] = np.round(s[2] * 2) / 2                                     # a handful of levels: huge tie classes
    s[3] = 0.25                                                       # all equal
    s[4] = np.sort(s[4])                                              # ascending: the kept tokens are the last ones
    s[5] = np.sort(s[5])[::-1]                                        # descending
    s[6] = -s[6]
    s[6, ::5] = 0.0
    s[6, 1::5] = -0.0
    s[7, T - 64:] = np.inf
    s[8, : T // 2] = 1e-30                                            # half the row in one bin, far below the rest
    return s


@pytest.mark.parametrize("T", [16385, 20000, 49999, 131072 + 5])
def test_topk_split_rows(T):
    _say("topk split rows", T)
    s = _long_rows(T, seed=T)
    for k in sorted({1, 7, T // 10, T // 2 + 1, T - T // 10, T - 1, T}):
        _check_topk(s, k)


def test_topk_split_rows_strided_unaligned_and_many_rows():
    _say("topk split rows strided")
    kvp = _kvp()
    T = 33001
    base = workloads.make_scores(70, T + 30, seed=11).to(DEV)
    view = base[:, 1:T + 1]                                           # rows neither 16-byte aligned nor contiguous
    got = kvp.kvp_select_topk(view, 9000)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.select_topk(base.cpu().numpy()[:, 1:T + 1], 9000))


def test_topk_rows_beyond_the_split_limit():
    _say("topk 2^20 + 3")
    T = (1 << 20) + 3
    s = workloads.make_scores(2, T, seed=12).numpy()
    s[1] = np.round(s[1] * 16) / 16
    _check_topk(s, T // 7)


def test_topk_workspace_is_validated():
    kvp = _kvp()
    T = 40000
    s = workloads.make_scores(3, T, seed=1).to(DEV)
    need = kvp.kvp_select_workspace_bytes(3, T, 100)
    assert need > 0 and kvp.kvp_select_workspace_bytes(3, 16384, 100) == 0
    with pytest.raises(kvp.KVPError) as e:
        kvp.kvp_select_topk(s, 100, ws=torch.empty(need - 256, dtype=torch.uint8, device=DEV))
    assert e.value.code == -5
    # a caller-owned workspace, reused across calls with different k
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    for k in (100, 20000):
        got = kvp.kvp_select_topk(s, k, ws=ws)
        torch.cuda.synchronize()
        assert np.array_equal(got.cpu().numpy(), oracle.select_topk(s.cpu().numpy(), k))


def test_topk_errors():
    kvp = _kvp()
    s = torch.zeros(2, 10, device=DEV)
    with pytest.raises(kvp.KVPError):
        kvp.kvp_select_topk(s, 11)


# ---------------------------------------------------------------- scores

def _score_case(L, W, G, H, T, seed, causal=True, force=True, outlier=8.0):
    kvp = _kvp()
    D = 128
    _say("score", dict(L=L, W=W, G=G, H=H, T=T, causal=causal, force=force))
    K, _ = workloads.make_kv(L, T, H, D, seed=seed, outlier_scale=outlier)
    Q = workloads.make_q(L, W, G * H, D, seed=seed)
    got = kvp.kvp_score_tokens(Q.to(DEV), K.to(DEV), causal=causal, force_window=force)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    ref = oracle.score_tokens(torch_bits(Q), torch_bits(K), causal=causal, force_window=force)
    inf = np.isinf(ref)
    assert np.array_equal(np.isinf(got), inf)
    tol = 1e-2 * np.abs(ref[~inf]) + 1e-4 * (G * W / T)
    assert np.all(np.abs(got[~inf] - ref[~inf]) <= tol)
    return got, ref


@pytest.mark.parametrize("shape", [
    dict(L=2, W=32, G=4, H=2, T=700),       # M = 128: one query tile per wave, ragged key tail
    dict(L=1, W=32, G=7, H=2, T=1100),      # M = 224: padded last tile
    dict(L=1, W=64, G=8, H=1, T=640),       # M = 512: four tiles per wave
    dict(L=1, W=8, G=1, H=3, T=100),        # M = 8: a single partly filled tile
    dict(L=1, W=32, G=4, H=1, T=32),        # W == T: every key sits in the window
])
def test_scores_match_oracle(shape):
    _score_case(seed=1, **shape)


def test_scores_flags_and_chunking():
    _score_case(1, 32, 4, 2, 5000, seed=2, causal=False, force=False)
    got, ref = _score_case(1, 32, 4, 2, 5000, seed=2, causal=True, force=False)
    # each softmax row sums to one
    assert np.allclose(got.sum(-1), 4 * 32, rtol=1e-3)


def test_score_then_select_overlap():
    # end-to-end keep-set: GPU scores -> GPU select; compared with the oracle pipeline as an overlap
    # fraction (scores differ in the last bits, so ties at the threshold may resolve differently)
    kvp = _kvp()
    L, W, G, H, T, D = 1, 32, 4, 8, 4096, 128
    _say("score->select", T)
    K, _ = workloads.make_kv(L, T, H, D, seed=0)
    Q = workloads.make_q(L, W, G * H, D, seed=0)
    s = kvp.kvp_score_tokens(Q.to(DEV), K.to(DEV))
    k = kvp.kvp_keep_count(0.5, T)
    idx = kvp.kvp_select_topk(s.view(L * H, T), k)
    torch.cuda.synchronize()
    # bit-exact against the oracle's selector on the very same (GPU) scores
    assert np.array_equal(idx.cpu().numpy(), oracle.select_topk(s.view(L * H, T).cpu().numpy(), k))
    ref_idx = oracle.select_topk(oracle.score_tokens(torch_bits(Q), torch_bits(K)).reshape(L * H, T), k)
    overlap = np.mean([len(set(a) & set(b)) / k for a, b in zip(idx.cpu().numpy(), ref_idx)])
    assert overlap > 0.99


@pytest.mark.parametrize("T,window,kernel", [(203, 0, 1), (4096, 32, 7), (5003, 64, 13), (16384, 64, 5), (2049, 5, 63),
                                             (40, 40, 3), (70, 69, 7)])
def test_smooth_scores_match_oracle(T, window, kernel):
    kvp = _kvp()
    _say("smooth", T, window, kernel)
    rows = 6
    big = workloads.make_scores(rows, T + 9, seed=T + kernel, device="cpu")
    s = big[:, :T]                                                  # strided rows
    s[:, T - window:] = float("inf")
    sg = big.to(DEV)[:, :T]
    s_np = s.numpy()
    for mode in ("avg", "max"):
        got = kvp.kvp_smooth_scores(sg, window, kernel, mode)
        torch.cuda.synchronize()
        ref = oracle.smooth_scores(s_np, window, kernel, mode)
        g = got.cpu().numpy()
        P = T - window
        assert np.array_equal(g[:, P:], ref[:, P:])
        if mode == "max":
            assert np.array_equal(g, ref)
        else:   # fp32 left-to-right sum of <= 63 non-negative terms against a double sum
            assert np.all(np.abs(g[:, :P] - ref[:, :P]) <= 1e-5 * np.abs(ref[:, :P]) + 1e-30)
        # the pipeline the method runs: smooth, then select; selection is exact on the GPU's own rows
        k = max(1, min(T, window + (T - window) // 3))
        idx = kvp.kvp_select_topk(got, k)
        torch.cuda.synchronize()
        assert np.array_equal(idx.cpu().numpy(), oracle.select_topk(g, k))


def test_smooth_scores_errors():
    kvp = _kvp()
    _say("smooth errors")
    s = torch.zeros(2, 64, device=DEV)
    for bad_kernel in (0, 4, 65):
        with pytest.raises(kvp.KVPError) as e:
            kvp.kvp_smooth_scores(s, 4, bad_kernel)
        assert e.value.code == -4
    with pytest.raises(kvp.KVPError):
        kvp.kvp_smooth_scores(s, 65, 3)                              # window longer than the row
    with pytest.raises(kvp.KVPError):
        kvp.kvp_smooth_scores(s, 4, 3, out=s)                        # in place
    torch.cuda.synchronize()
