"""kvp_score_tokens_static (the entry point that allocates nothing: its scratch is a fixed device array of the
library) against kvp_score_tokens with a caller workspace: same kernels, so the scores must agree bit for bit,
on two calls in a row, the second on a smaller input (the array still holds the first call's statistics)."""
import ctypes

import numpy as np
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pair(kvp, L, T, H, G, W, seed, causal=True, force_window=True):
    print("[case] score static", L, T, H, G, W, seed, flush=True)
    K, _ = workloads.make_kv(L, T, H, 128, seed=seed, device=DEV)
    Q = workloads.make_q(L, W, G * H, 128, seed=seed, device=DEV)
    want = kvp.kvp_score_tokens(Q, K, causal=causal, force_window=force_window)
    got = torch.full((L, H, T), float("nan"), dtype=torch.float32, device=DEV)
    # the call itself must not allocate: torch's allocator statistics do not move across it
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    kvp.kvp_score_tokens_static(Q, K, got, causal=causal, force_window=force_window)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32))


def test_static_scratch_matches_workspace_entry_point_twice():
    import paper_2512_14946_amd as kvp
    # first call: several chunks, ragged tail, M = 224 (7 query tiles); 1.8 MiB of the 4 MiB array
    assert kvp.kvp_score_workspace_bytes(2, 4, 28, 32, 9000) <= kvp.KVP_SCORE_STATIC_SCRATCH_BYTES
    _pair(kvp, 2, 9000, 4, 7, 32, seed=3)
    # second call: smaller in every dimension, so most of the array keeps stale statistics
    _pair(kvp, 1, 777, 2, 2, 16, seed=4)
    # and the first shape again, non-causal without the forced window
    _pair(kvp, 2, 9000, 4, 7, 32, seed=5, causal=False, force_window=False)


def test_static_scratch_rejects_oversized_shapes():
    import paper_2512_14946_amd as kvp
    L, T, H, G, W = 80, 16384, 8, 8, 64
    assert kvp.kvp_score_workspace_bytes(L, H, G * H, W, T) > kvp.KVP_SCORE_STATIC_SCRATCH_BYTES
    # validation reads sizes only: small stand-in tensors with the big shape's strides are never dereferenced
    K = torch.empty(128, dtype=torch.bfloat16, device=DEV).as_strided((L, T, H, 128), (0, 0, 0, 1))
    Q = torch.empty(128, dtype=torch.bfloat16, device=DEV).as_strided((L, W, G * H, 128), (0, 0, 0, 1))
    out = torch.empty(4, dtype=torch.float32, device=DEV)
    with pytest.raises(kvp.KVPError) as e:
        # the binding checks `scores` for contiguity first: call the C entry point directly
        from paper_2512_14946_amd import kvp as binding
        qv, kv = binding._view(Q), binding._view(K)
        binding._check(binding._lib.kvp_score_tokens_static(ctypes.byref(qv), ctypes.byref(kv), 1, 1, out.data_ptr(),
                                                            None), "kvp_score_tokens_static")
    assert e.value.code == -5
