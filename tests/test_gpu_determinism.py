"""GPU: the boundary's determinism promise.  The same inputs give the same bytes, call after call, with other work
in between, on the current stream or on a stream of the caller's (no order-dependent floating-point atomics
anywhere on the path)."""
import pytest
import torch

import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _kvp():
    import paper_2512_14946_amd as kvp
    return kvp


def _same(a: torch.Tensor, b: torch.Tensor) -> bool:
    return bool((a.contiguous().view(torch.uint8) == b.contiguous().view(torch.uint8)).all())


def test_repeated_calls_are_bit_identical():
    kvp = _kvp()
    L, T, H, D, G, W = 3, 5000, 4, 128, 7, 32
    print("[case] determinism", (L, T, H, D, G, W), flush=True)
    K, V = workloads.make_kv(L, T, H, D, seed=11, device=DEV)
    Q = workloads.make_q(L, W, G * H, D, seed=11, device=DEV)
    cfgs = [(16, 0, T), (8, 64, T), (4, 32, 2500), (2, 128, 1250), (4, 128, 1250)]
    side = torch.cuda.Stream()

    def run_all(stream):
        out = {}
        out["scores"] = kvp.kvp_score_tokens(Q, K, stream=stream)
        out["knorm"] = kvp.kvp_score_keys(K, kvp.KVP_SCORE_KNORM, stream=stream)
        out["keydiff"] = kvp.kvp_score_keys(K, kvp.KVP_SCORE_KEYDIFF, stream=stream)
        out["smooth"] = kvp.kvp_smooth_scores(out["scores"].view(L * H, T), W, 7, "avg", stream=stream)
        out["idx"] = kvp.kvp_select_topk(out["smooth"], 1500, stream=stream)
        out["loss"], out["partial"] = kvp.kvp_eval_configs(Q, K, V, cfgs, want_partial=True, stream=stream)
        out["loss_mx"], out["partial_mx"] = kvp.kvp_eval_configs(Q, K, V, cfgs, want_partial=True, pv_matrix_cores=True,
                                                               stream=stream)
        qp = kvp.alloc_qplane(L, T, H, D, 4, 64, DEV, asymmetric=True)
        kvp.kvp_quantize(V, qp, stream=stream)
        out["codes"], out["scales"], out["mins"] = qp.codes, qp.scales, qp.mins
        return out

    first = run_all(None)
    torch.cuda.synchronize()
    # unrelated work in between, then again on the current stream and on a side stream
    junk = torch.randn(4096, 4096, device=DEV) @ torch.randn(4096, 4096, device=DEV)
    second = run_all(None)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        third = run_all(side)
    side.synchronize()
    del junk
    for name, ref in first.items():
        assert _same(ref, second[name]), name
        assert _same(ref, third[name]), name
