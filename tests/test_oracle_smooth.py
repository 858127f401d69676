"""Pins for the oracle's score smoothing (1-D pooling of the prefix scores before the top-k).

Library routines (torch's avg_pool1d / max_pool1d with zero / -inf padding) on the prefix, closed
forms (constant rows, an impulse), the window pass-through, and a brute-force loop.
"""
import numpy as np
import pytest
import torch

import oracle


@pytest.mark.parametrize("kernel", [1, 3, 7, 13])
@pytest.mark.parametrize("window", [0, 5, 32])
def test_matches_library_pooling_on_the_prefix(kernel, window):
    rng = np.random.default_rng(kernel * 100 + window)
    rows, T = 5, 211
    s = rng.random((rows, T)).astype(np.float32) * 10
    s[:, T - window:] = np.inf                                   # forced window entries
    P = T - window
    x = torch.from_numpy(s[:, :P].astype(np.float64)).unsqueeze(1)
    want_avg = torch.nn.functional.avg_pool1d(x, kernel, stride=1, padding=kernel // 2, count_include_pad=True)[:, 0].numpy()
    want_max = torch.nn.functional.max_pool1d(x, kernel, stride=1, padding=kernel // 2)[:, 0].numpy()
    got_avg = oracle.smooth_scores(s, window, kernel, "avg")
    got_max = oracle.smooth_scores(s, window, kernel, "max")
    assert np.array_equal(got_avg[:, :P], want_avg.astype(np.float32))    # fp64 sum, one rounding: same value
    assert np.array_equal(got_max[:, :P], want_max.astype(np.float32))
    assert np.all(np.isinf(got_avg[:, P:])) and np.all(np.isinf(got_max[:, P:]))
    assert np.all(np.isfinite(got_avg[:, :P])) and np.all(np.isfinite(got_max[:, :P]))   # the window never leaks


def test_closed_forms():
    T, W, k = 40, 4, 5
    s = np.full((1, T), 3.0, dtype=np.float32)
    out = oracle.smooth_scores(s, W, k, "avg")[0]
    P = T - W
    assert np.all(out[2:P - 2] == 3.0)
    assert out[0] == np.float32(9.0 / 5) and out[1] == np.float32(12.0 / 5)          # 3 and 4 in-range taps
    assert out[P - 1] == np.float32(9.0 / 5) and out[P - 2] == np.float32(12.0 / 5)  # the window is not a tap
    assert np.all(out[P:] == 3.0)
    # impulse -> a box of 1/kernel (avg) or 1 (max) of width kernel
    s = np.zeros((1, T), dtype=np.float32)
    s[0, 10] = 1.0
    a = oracle.smooth_scores(s, W, k, "avg")[0]
    m = oracle.smooth_scores(s, W, k, "max")[0]
    assert np.array_equal(np.nonzero(a)[0], np.arange(8, 13)) and np.all(a[8:13] == np.float32(0.2))
    assert np.array_equal(np.nonzero(m)[0], np.arange(8, 13)) and np.all(m[8:13] == 1.0)
    # kernel 1 is the identity; mass is preserved away from the edges
    r = np.random.default_rng(0).random((2, T)).astype(np.float32)
    assert np.array_equal(oracle.smooth_scores(r, W, 1, "avg"), r)
    assert np.array_equal(oracle.smooth_scores(r, W, 1, "max"), r)


def test_brute_force_strided_rows():
    rng = np.random.default_rng(3)
    big = rng.standard_normal((4, 64)).astype(np.float32)
    s = big[:, :37]                                              # strided rows
    W, k = 6, 7
    got = oracle.smooth_scores(s, W, k, "avg")
    P = 37 - W
    for row in range(4):
        for t in range(37):
            if t >= P:
                assert got[row, t] == s[row, t]
                continue
            acc = 0.0
            for u in range(t - 3, t + 4):
                if 0 <= u < P:
                    acc += float(s[row, u])
            assert got[row, t] == np.float32(acc / k)


def test_smoothing_keeps_neighbours_of_a_peak():
    # the point of the pooling: after it, the top-k around an isolated peak is a contiguous run
    T, W = 128, 8
    s = np.random.default_rng(1).random((1, T)).astype(np.float32) * 0.01
    s[0, 50] = 5.0
    s[0, T - W:] = np.inf
    idx = oracle.select_topk(oracle.smooth_scores(s, W, 7, "max"), W + 7)[0]
    assert np.array_equal(idx[:7], np.arange(47, 54))
