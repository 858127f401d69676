"""Pins for the oracle's batched quality-loss proxy (CPU only).

The paper's profiler scores every (method, ratio) configuration of a context
(Profiler module; utility function); its quality metric needs model weights,
so the proxy here is the relative L2 error of the window queries' attention
output.  Pins: identities (unquantized + keep-all gives exactly 0; nested
keep-sets; monotone in bits), a float64 library recomputation on a tiny
shape, and an independent from-the-formula brute force.
"""
import numpy as np
import torch

import oracle
import workloads
from helpers import bits_to_f32, torch_bits


def _inputs(L, W, G, H, T, D, seed):
    K, V = workloads.make_kv(L, T, H, D, seed=seed)
    Q = workloads.make_q(L, W, G * H, D, seed=seed)
    return torch_bits(Q), torch_bits(K), torch_bits(V)


def test_identity_and_orderings():
    L, W, G, H, T, D = 2, 4, 2, 2, 64, 128
    q, k, v = _inputs(L, W, G, H, T, D, 0)
    cfgs = [(16, 0, T), (8, 32, T), (4, 32, T), (2, 32, T), (8, 128, T), (4, 128, T), (2, 128, T),
            (16, 0, 48), (16, 0, 32), (16, 0, 16)]
    loss, partial = oracle.eval_configs(q, k, v, cfgs)
    assert loss[0] == 0.0                                   # identity row
    assert 0 < loss[1] < loss[2] < loss[3]                  # fewer bits, larger loss (group 32)
    assert 0 < loss[4] < loss[5] < loss[6]                  # ... and at group 128
    assert loss[1] < loss[4] and loss[2] < loss[5]          # outlier channels: smaller groups help
    assert 0 < loss[7] < loss[8] < loss[9]                  # dropping more tokens, larger loss
    # loss = sqrt(sum num / sum den) over layers; den does not depend on the config
    assert np.allclose(partial[:, 0, 1], partial[:, 3, 1])
    want = np.sqrt(partial[:, :, 0].sum(0) / partial[:, :, 1].sum(0))
    assert np.allclose(loss, want, rtol=1e-6)


def test_keep_sets_are_nested():
    L, W, G, H, T, D = 1, 4, 2, 1, 64, 32
    q, k, _ = _inputs(L, W, G, H, T, D, 1)
    s = oracle.score_tokens(q, k, causal=True, force_window=True)[0]
    sets = [set(oracle.select_topk(s, kk)[0].tolist()) for kk in (16, 32, 48, 64)]
    assert sets[0] < sets[1] < sets[2] < sets[3]
    assert all(set(range(T - W, T)) <= st for st in sets)


def _library_loss(q, k, v, cfgs, G):
    """float64 torch recomputation; K-hat / V-hat and keep-sets come from oracle pieces pinned elsewhere."""
    L, W, Hq, D = q.shape
    _, T, H, _ = k.shape
    qf = torch.from_numpy(bits_to_f32(q)).double()
    scores = oracle.score_tokens(q, k, causal=True, force_window=True)
    pos = (T - W + torch.arange(W)).view(1, W, 1)
    causal = torch.arange(T).view(1, 1, T) > pos
    out = []
    for bits, group, kk in cfgs:
        num = den = 0.0
        for l in range(L):
            for h in range(H):
                def attn(kb, vb, allowed):
                    kf = torch.from_numpy(bits_to_f32(kb)).double()
                    vf = torch.from_numpy(bits_to_f32(vb)).double()
                    logits = torch.einsum("wud,td->uwt", qf[l][:, h * G:(h + 1) * G], kf) / D ** 0.5
                    logits = logits.masked_fill(causal | ~allowed.view(1, 1, T), float("-inf"))
                    return torch.softmax(logits, -1) @ vf
                full = attn(k[l, :, h], v[l, :, h], torch.ones(T, dtype=torch.bool))
                if bits == 16:
                    kh, vh = k[l, :, h], v[l, :, h]
                else:
                    bt = np.arange((T + 15) // 16, dtype=np.int32)
                    def roundtrip(x):
                        c, s = oracle.quantize(np.ascontiguousarray(x).reshape(1, T, 1, D), bits, group)
                        return oracle.dequantize_paged(c, s, bits, group, T, bt, len(bt), 16).reshape(-1, D)[:T]
                    kh, vh = roundtrip(k[l, :, h]), roundtrip(v[l, :, h])
                allowed = torch.zeros(T, dtype=torch.bool)
                allowed[torch.from_numpy(oracle.select_topk(scores[l, h:h + 1], kk)[0].astype(np.int64))] = True
                o = attn(kh, vh, allowed)
                num += float(((o - full) ** 2).sum())
                den += float((full ** 2).sum())
        out.append(np.sqrt(num / den))
    return np.array(out)


def test_matches_library_recomputation():
    L, W, G, H, T, D = 2, 3, 2, 2, 40, 32
    q, k, v = _inputs(L, W, G, H, T, D, 2)
    cfgs = [(16, 0, T), (8, 32, T), (4, 16, 30), (2, 32, 20), (16, 0, 10), (8, 8, 3)]
    loss, _ = oracle.eval_configs(q, k, v, cfgs)
    want = _library_loss(q, k, v, cfgs, G)
    assert np.allclose(loss, want, rtol=1e-5, atol=1e-9)


def test_tiny_brute_force_from_the_formula():
    # T = 8, W = 2, D = 32 (one group), one layer, one kv head, one query head: everything from first
    # principles in float64 numpy, including the abs-max quantizer and the score ranking.
    L, W, G, H, T, D = 1, 2, 1, 1, 8, 32
    q, k, v = _inputs(L, W, G, H, T, D, 4)
    qf, kf, vf = (bits_to_f32(a).astype(np.float64)[0, :, 0] for a in (q, k, v))

    def probs(keys, allowed):
        P = np.zeros((W, T))
        for w in range(W):
            ok = [t for t in range(T) if t <= T - W + w and allowed[t]]
            lg = np.array([qf[w] @ keys[t] / np.sqrt(D) for t in ok])
            e = np.exp(lg - lg.max())
            P[w, ok] = e / e.sum()
        return P

    def fake_quant(x, qmax):  # float64 stand-in; exact here because the data avoids rounding boundaries
        s = np.float32(np.abs(x).max(axis=1, keepdims=True).astype(np.float32) / np.float32(qmax))
        qv = np.rint((x.astype(np.float32) / s).astype(np.float32))
        y = (qv.astype(np.float32) * s).astype(np.float32)
        return bits_to_f32(torch_bits(torch.from_numpy(y).to(torch.bfloat16))).astype(np.float64)

    P_full = probs(kf, np.ones(T, bool))
    o_full = P_full @ vf
    score = P_full.sum(0)
    score[T - W:] = np.inf
    order = sorted(range(T), key=lambda t: (-score[t], t))
    cfgs = [(16, 0, 8), (4, 32, 8), (16, 0, 5), (2, 32, 4)]
    want = []
    for bits, group, kk in cfgs:
        allowed = np.zeros(T, bool)
        allowed[order[:kk]] = True
        kh, vh = (kf, vf) if bits == 16 else (fake_quant(kf, 2 ** (bits - 1) - 1), fake_quant(vf, 2 ** (bits - 1) - 1))
        o = probs(kh, allowed) @ vh
        want.append(np.sqrt(((o - o_full) ** 2).sum() / (o_full ** 2).sum()))
    loss, _ = oracle.eval_configs(q, k, v, cfgs)
    assert np.allclose(loss, np.array(want), rtol=1e-5, atol=1e-9)
