"""GPU: the token-dropping pipeline and the configuration proxy replayed from a HIP graph.

The library allocates nothing and never synchronizes, so every entry point can be captured when the caller supplies
the workspaces.  Each replay must reproduce the eager result bit for bit, with eager work and synchronizations
between the replays; the eager result itself is checked against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import torch_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_score_select_gather_quantize_and_eval_replay_from_a_graph():
    import paper_2512_14946_amd as kvp
    L, T, H, D, G, W = 2, 700, 2, 128, 4, 32
    print("[case] graph pipeline", dict(L=L, T=T, H=H, G=G, W=W), flush=True)
    inputs = []
    for seed in (21, 22):
        K, V = workloads.make_kv(L, T, H, D, seed=seed)
        Q = workloads.make_q(L, W, G * H, D, seed=seed)
        inputs.append((Q.to(DEV), K.to(DEV), V.to(DEV)))
    k = kvp.kvp_keep_count(0.3, T)
    cfgs = [(16, 0, T), (8, 32, T), (4, 64, k), (2, 32, k)]
    # everything the captured calls touch is allocated up front
    q, kk, v = (torch.empty_like(t) for t in inputs[0])
    scores = torch.empty(L, H, T, dtype=torch.float32, device=DEV)
    ws_score = torch.empty(kvp.kvp_score_workspace_bytes(L, H, G * H, W, T) + 16, dtype=torch.uint8, device=DEV)
    idx = torch.empty(L * H, k, dtype=torch.int32, device=DEV)
    qp = kvp.alloc_qplane(L, k, H, D, 4, 32, DEV)
    loss = torch.empty(len(cfgs), dtype=torch.float32, device=DEV)
    ws_eval = torch.empty(kvp.kvp_eval_workspace_bytes(L, H, G * H, W, T, len(cfgs)) + 16, dtype=torch.uint8, device=DEV)

    def step():
        kvp.kvp_score_tokens(q, kk, scores, ws=ws_score)
        kvp.kvp_select_topk(scores.view(L * H, T), k, idx)
        kvp.kvp_quantize(kk, qp, keep_idx=idx.view(L, H, k))
        kvp.kvp_eval_configs(q, kk, v, cfgs, loss=loss, ws=ws_eval)

    def load(i):
        for dst, src in zip((q, kk, v), inputs[i]):
            dst.copy_(src)

    load(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep, i in enumerate([0, 1, 0, 1]):
        load(i)                                  # eager work between the replays
        scores.fill_(float("nan"))
        idx.fill_(-1)
        qp.codes.fill_(0xEE)
        loss.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        got = (scores.clone(), idx.clone(), qp.codes.clone(), qp.scales.clone(), loss.clone())
        step()                                   # the eager result for the same input
        torch.cuda.synchronize()
        want = (scores, idx, qp.codes, qp.scales, loss)
        for a, b in zip(got, want):
            assert torch.equal(a.view(torch.uint8) if a.dtype == torch.uint8 else a.view(torch.int32), 
                               b.view(torch.uint8) if b.dtype == torch.uint8 else b.view(torch.int32)), rep
    # the last eager result (inputs[1]) against the oracle
    Q, K, V = inputs[1]
    ref_scores = oracle.score_tokens(torch_bits(Q.cpu()), torch_bits(K.cpu()))
    s = scores.cpu().numpy()
    fin = np.isfinite(ref_scores)
    assert np.array_equal(np.isfinite(s), fin)
    assert np.all(np.abs(s[fin] - ref_scores[fin]) <= 1e-2 * np.abs(ref_scores[fin]) + 1e-4 * G * W / T)
    assert np.array_equal(idx.cpu().numpy(), oracle.select_topk(s.reshape(L * H, T), k))
    ref_loss, _ = oracle.eval_configs(torch_bits(Q.cpu()), torch_bits(K.cpu()), torch_bits(V.cpu()), cfgs)
    assert np.all(np.abs(loss.cpu().numpy() - ref_loss) <= 1e-2 * np.abs(ref_loss) + 1e-5)
