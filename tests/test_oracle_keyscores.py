"""Pins for the oracle's key-only importance scores (CPU only): knorm and keydiff, the two other
token-dropping methods the paper evaluates (Evaluation, Baselines)."""
import numpy as np
import torch

import oracle
import workloads
from helpers import bits_to_f32, to_bf16_bits, torch_bits


def _keys(rows):
    a = np.asarray(rows, dtype=np.float32)
    return to_bf16_bits(a).reshape(1, a.shape[0], 1, a.shape[1])


def test_knorm_closed_forms():
    k = _keys([[3, 4, 0, 0], [0, 0, 0, 0], [1, 1, 1, 1], [-2, 0, 0, 0], [0.5, -0.5, 0.5, -0.5]])
    s = oracle.score_keys(k, oracle.KNORM)[0, 0]
    assert np.allclose(s, [5.0, 0.0, 2.0, 2.0, 1.0], rtol=1e-7)


def test_keydiff_closed_forms():
    # identical directions: every cosine is 1 -> score -1, whatever the lengths
    k = _keys([[1, 2, 3, 4], [2, 4, 6, 8], [0.5, 1, 1.5, 2]])
    assert np.allclose(oracle.score_keys(k, oracle.KEYDIFF)[0, 0], -1.0, rtol=1e-6)
    # orthogonal one-hot keys: every cosine is 0
    assert np.allclose(oracle.score_keys(_keys(np.eye(4)), oracle.KEYDIFF)[0, 0], 0.0, atol=1e-12)
    # two antipodal pairs {a, a, -a}: token 0 sees cosines (1, -1) -> 0; token 2 sees (-1, -1) -> +1
    k = _keys([[1, 1, 0, 0], [2, 2, 0, 0], [-1, -1, 0, 0]])
    assert np.allclose(oracle.score_keys(k, oracle.KEYDIFF)[0, 0], [0.0, 0.0, 1.0], atol=1e-7)
    # a zero key has cosine 0 with everything; the others average over T - 1 tokens including it
    k = _keys([[1, 0, 0, 0], [0, 0, 0, 0], [1, 0, 0, 0]])
    assert np.allclose(oracle.score_keys(k, oracle.KEYDIFF)[0, 0], [-0.5, 0.0, -0.5], atol=1e-7)
    # a single token has nobody to compare with
    assert oracle.score_keys(_keys([[1, 2, 3, 4]]), oracle.KEYDIFF)[0, 0, 0] == 0.0


def test_keydiff_matches_library_and_is_scale_invariant():
    L, T, H, D = 2, 70, 3, 32
    K, _ = workloads.make_kv(L, T, H, D, seed=0)
    kb = torch_bits(K)
    s = oracle.score_keys(kb, oracle.KEYDIFF)
    kf = torch.from_numpy(bits_to_f32(kb)).double()
    for l in range(L):
        for h in range(H):
            x = torch.nn.functional.normalize(kf[l, :, h], dim=-1)
            cos = x @ x.T
            want = -(cos.sum(1) - cos.diagonal()) / (T - 1)
            assert np.allclose(s[l, h], want.numpy(), rtol=1e-5, atol=1e-8)
    # doubling one token's key (exact in bf16) changes its norm score but not any keydiff score
    kb2 = kb.copy()
    kb2[0, 5, 1] = to_bf16_bits(bits_to_f32(kb[0, 5, 1]) * 2.0)
    assert np.allclose(oracle.score_keys(kb2, oracle.KEYDIFF), s, rtol=1e-6, atol=1e-9)
    n1, n2 = oracle.score_keys(kb, oracle.KNORM), oracle.score_keys(kb2, oracle.KNORM)
    assert np.isclose(n2[0, 1, 5], 2 * n1[0, 1, 5], rtol=1e-6)
    # the sampled form returns the same numbers
    toks = np.array([0, 5, 69], dtype=np.int32)
    assert np.array_equal(oracle.score_keys(kb, oracle.KEYDIFF, tokens=toks), s[..., toks])
    # strided view (one head of a wider tensor)
    assert np.array_equal(oracle.score_keys(kb[:, :, 1:2], oracle.KNORM), n1[:, 1:2])


def test_knorm_matches_library():
    K, _ = workloads.make_kv(1, 50, 2, 128, seed=1)
    kb = torch_bits(K)
    want = torch.from_numpy(bits_to_f32(kb)).double().norm(dim=-1).permute(0, 2, 1).numpy()
    assert np.allclose(oracle.score_keys(kb, oracle.KNORM), want, rtol=1e-6)
