"""GPU parity: kvp_score_keys (knorm, keydiff) against the CPU oracle.

Tolerances: knorm is an fp32 sum of 128 squares and a square root: 1e-5 relative.  keydiff is a
difference of O(1) quantities divided by T - 1, from an fp32 sum of T unit vectors:
|gpu - ref| <= 1e-3 |ref| + 2e-5 / (T - 1)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import bits_to_torch, torch_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _kvp():
    import paper_2512_14946_amd as kvp
    return kvp


def _check(kb, kd, T, tokens=None):
    kvp = _kvp()
    n = kvp.kvp_score_keys(kd, kvp.KVP_SCORE_KNORM)
    d = kvp.kvp_score_keys(kd, kvp.KVP_SCORE_KEYDIFF)
    torch.cuda.synchronize()
    n, d = n.cpu().numpy(), d.cpu().numpy()
    rn = oracle.score_keys(kb, oracle.KNORM, tokens=tokens)
    rd = oracle.score_keys(kb, oracle.KEYDIFF, tokens=tokens)
    if tokens is not None:
        n, d = n[..., tokens], d[..., tokens]
    assert np.all(np.abs(n - rn) <= 1e-5 * np.abs(rn))
    assert np.all(np.abs(d - rd) <= 1e-3 * np.abs(rd) + 2e-5 / max(T - 1, 1)), np.abs(d - rd).max()
    return n, d


@pytest.mark.parametrize("shape", [(2, 1000, 3), (1, 67, 8), (1, 1, 2), (3, 2, 1), (1, 2500, 2)])
def test_key_scores_match_oracle(shape):
    L, T, H = shape
    print("[case] key scores", shape, flush=True)
    K, _ = workloads.make_kv(L, T, H, 128, seed=3)
    kb = torch_bits(K).copy()
    if T > 10:
        kb[0, 3, 0] = 0                                     # a zero key
        kb[0, 4, 0] = kb[0, 5, 0]                           # a duplicated key
    _check(kb, bits_to_torch(kb, DEV), T)


def test_key_scores_strided_view_and_feed_select():
    kvp = _kvp()
    print("[case] key scores strided", flush=True)
    L, T, H = 2, 300, 6
    K, _ = workloads.make_kv(L, T, H, 128, seed=4)
    kd = K.to(DEV)[:, :, 2:5]
    kb = np.ascontiguousarray(torch_bits(K)[:, :, 2:5])
    _check(kb, kd, T)
    s = kvp.kvp_score_keys(kd, kvp.KVP_SCORE_KEYDIFF)
    idx = kvp.kvp_select_topk(s.view(L * 3, T), 100)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy(), oracle.select_topk(s.view(L * 3, T).cpu().numpy(), 100))


def test_key_scores_full_size_sampled():
    print("[case] key scores full size", flush=True)
    c = workloads.CONFIGS["llama3_8b_int4_paged"]
    L, T, H = 8, c["T"], c["H"]                              # 8 of the 32 layers: same per-layer grid
    K, _ = workloads.make_kv(L, T, H, 128, seed=0, device=DEV)
    toks = np.unique(np.concatenate([[0, 1, T - 1], np.random.default_rng(0).integers(0, T, 40)])).astype(np.int32)
    n, d = _check(torch_bits(K), K, T, tokens=toks)
    assert np.all(n > 0)


def test_key_scores_errors():
    kvp = _kvp()
    k = torch.zeros(1, 8, 2, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(kvp.KVPError):
        kvp.kvp_score_keys(k, 7)
    with pytest.raises(kvp.KVPError):
        kvp.kvp_score_keys(k, kvp.KVP_SCORE_KEYDIFF, ws=torch.empty(16, dtype=torch.uint8, device=DEV))
