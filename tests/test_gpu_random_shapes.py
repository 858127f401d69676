"""GPU parity on seeded random shapes: every entry point of the compress / decompress path against the oracle on
shapes nobody picked by hand (ragged tails, odd head counts, window sizes that do not divide a tile, keep counts
anywhere between 1 and T, spare blocks in the pool)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import torch_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
D = 128


def _kvp():
    import paper_2512_14946_amd as kvp
    return kvp


def _shape(seed):
    rng = np.random.default_rng(1000 + seed)
    L = int(rng.integers(1, 4))
    H = int(rng.choice([1, 2, 3, 4, 8]))
    T = int(rng.choice([rng.integers(1, 40), rng.integers(40, 700), rng.integers(700, 3000)]))
    G = int(rng.choice([1, 2, 4, 7, 8]))
    W = int(min(T, rng.integers(1, 65), 512 // G))
    return rng, L, H, T, G, W


@pytest.mark.parametrize("seed", range(10))
def test_quantize_dequantize_random(seed):
    kvp = _kvp()
    rng, L, H, T, _, _ = _shape(seed)
    bits = int(rng.choice([8, 4, 2]))
    group = int(rng.choice([32, 64, 128]))
    asym, per_channel = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    bs = int(rng.choice([1, 4, 8, 16, 32]))                     # page size (a per-channel group holds whole pages)
    print("[case] random quantize", dict(seed=seed, L=L, H=H, T=T, bits=bits, group=group, asym=asym,
                                         per_channel=per_channel, bs=bs), flush=True)
    K, _ = workloads.make_kv(L, T, H, D, seed=seed, outlier_scale=float(rng.choice([1.0, 8.0, 16.0])))
    Kd = K.to(DEV)
    qp = kvp.alloc_qplane(L, T, H, D, bits, group, DEV, page=bs, asymmetric=asym, per_channel=per_channel)
    kvp.kvp_quantize(Kd, qp)
    n_pages = (T + bs - 1) // bs
    nb = n_pages + int(rng.integers(0, 5))                      # spare blocks stay untouched
    bt = torch.from_numpy(rng.permutation(nb)[:n_pages].astype(np.int32)).to(DEV)
    pg = kvp.alloc_paged(L, T, H, D, bt, nb, bs, fill_nan=True)
    kvp.kvp_dequantize_paged(qp, pg)
    torch.cuda.synchronize()
    x, btn = torch_bits(K), bt.cpu().numpy()
    if per_channel:
        oc, os_, om = oracle.quantize_channel(x, bits, group, asym=asym, Tp=qp.Tp)
        od = oracle.dequantize_paged_channel(oc, os_, om, bits, group, T, btn, nb, bs)
    elif asym:
        oc, os_, om = oracle.quantize_asym(x, bits, group, Tp=qp.Tp)
        od = oracle.dequantize_paged_asym(oc, os_, om, bits, group, T, btn, nb, bs)
    else:
        oc, os_ = oracle.quantize(x, bits, group, Tp=qp.Tp)
        om = None
        od = oracle.dequantize_paged(oc, os_, bits, group, T, btn, nb, bs)
    assert np.array_equal(qp.codes.cpu().numpy(), oc)
    assert np.array_equal(qp.scales.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    if om is not None:
        assert np.array_equal(qp.mins.cpu().numpy().view(np.uint32), om.view(np.uint32))
    assert np.array_equal(torch_bits(pg.pool), od)              # untouched slots keep the same NaN pattern


@pytest.mark.parametrize("seed", range(10))
def test_score_smooth_select_random(seed):
    kvp = _kvp()
    rng, L, H, T, G, W = _shape(seed)
    causal, force = bool(rng.integers(0, 2)), bool(rng.integers(0, 2))
    print("[case] random score/select", dict(seed=seed, L=L, H=H, T=T, G=G, W=W, causal=causal, force=force), flush=True)
    K, _ = workloads.make_kv(L, T, H, D, seed=seed)
    Q = workloads.make_q(L, W, G * H, D, seed=seed)
    got = kvp.kvp_score_tokens(Q.to(DEV), K.to(DEV), causal=causal, force_window=force)
    torch.cuda.synchronize()
    ref = oracle.score_tokens(torch_bits(Q), torch_bits(K), causal=causal, force_window=force)
    g = got.cpu().numpy()
    inf = np.isinf(ref)
    assert np.array_equal(np.isinf(g), inf)
    assert np.all(np.abs(g[~inf] - ref[~inf]) <= 1e-2 * np.abs(ref[~inf]) + 1e-4 * (G * W / T))
    # smoothing and selection are checked on the GPU's own scores (bit-exact from there on)
    rows = got.view(L * H, T)
    kernel = int(rng.choice([1, 3, 7, 13]))
    mode = str(rng.choice(["avg", "max"]))
    sm = kvp.kvp_smooth_scores(rows, W, kernel, mode)
    k = int(rng.integers(1, T + 1))
    idx = kvp.kvp_select_topk(sm, k)
    torch.cuda.synchronize()
    ref_sm = oracle.smooth_scores(rows.cpu().numpy(), W, kernel, mode)
    sm_np = sm.cpu().numpy()
    fin = np.isfinite(ref_sm)
    assert np.array_equal(np.isfinite(sm_np), fin)
    if mode == "max":
        assert np.array_equal(sm_np[fin], ref_sm[fin])
    else:
        assert np.all(np.abs(sm_np[fin] - ref_sm[fin]) <= 1e-5 * np.abs(ref_sm[fin]))
    assert np.array_equal(idx.cpu().numpy(), oracle.select_topk(sm_np, k))


@pytest.mark.parametrize("seed", range(6))
def test_gather_quantize_and_scatter_restore_random(seed):
    kvp = _kvp()
    rng, L, H, T, _, _ = _shape(seed + 50)
    bits, group = int(rng.choice([8, 4, 2])), int(rng.choice([32, 64, 128]))
    asym = bool(rng.integers(0, 2))
    k = int(rng.integers(1, T + 1))
    print("[case] random gather/scatter", dict(seed=seed, L=L, H=H, T=T, k=k, bits=bits, group=group, asym=asym), flush=True)
    K, _ = workloads.make_kv(L, T, H, D, seed=seed)
    keep = np.stack([np.stack([np.sort(rng.permutation(T)[:k]) for _ in range(H)]) for _ in range(L)]).astype(np.int32)
    keep_d = torch.from_numpy(keep).to(DEV)
    bs = int(rng.choice([2, 8, 16, 64]))
    n_pages = (T + bs - 1) // bs
    bt = torch.from_numpy(rng.permutation(n_pages).astype(np.int32)).to(DEV)
    # the source is the serving engine's paged pool (same block table), gathered through the keep lists
    src_pool = torch.zeros(L, n_pages, bs, H, D, dtype=torch.bfloat16, device=DEV)
    tok = torch.arange(T, device=DEV)
    src_pool[:, bt.long()[tok // bs], tok % bs] = K.to(DEV)
    qp = kvp.alloc_qplane(L, k, H, D, bits, group, DEV, page=bs, asymmetric=asym)
    kvp.kvp_quantize(kvp.PagedKV(src_pool, bt, T), qp, keep_idx=keep_d)
    pool = torch.full((L, n_pages, bs, H, D), 3.0, dtype=torch.bfloat16, device=DEV)
    kvp.kvp_dequantize_paged_scatter(qp, keep_d, kvp.PagedKV(pool, bt, T))
    torch.cuda.synchronize()
    x = torch_bits(K)
    if asym:
        oc, os_, om = oracle.quantize_asym(x, bits, group, keep_idx=keep, Tp=qp.Tp)
    else:
        oc, os_ = oracle.quantize(x, bits, group, keep_idx=keep, Tp=qp.Tp)
        om = None
    assert np.array_equal(qp.codes.cpu().numpy(), oc)
    assert np.array_equal(qp.scales.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    three = int(torch_bits(torch.tensor([3.0], dtype=torch.bfloat16))[0])
    ref_pool = np.full((L, n_pages, bs, H, D), three, dtype=np.uint16)
    oracle.dequantize_paged_scatter(oc, os_, om, bits, group, keep, T, bt.cpu().numpy(), n_pages, bs, pool=ref_pool)
    assert np.array_equal(torch_bits(pool), ref_pool)


@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("pv", ["pv_dot2_fp16", "pv_fp32", "pv_matrix_cores"])
def test_eval_configs_random(seed, pv):
    pv_kw = {"pv_dot2_fp16": {}, "pv_fp32": {"pv_fp32": True}, "pv_matrix_cores": {"pv_matrix_cores": True}}[pv]
    kvp = _kvp()
    rng, L, H, T, G, W = _shape(seed + 100)
    T = min(max(T, 2), 600)                                   # the oracle is O(configs x rows x T x D)
    L = min(L, 2)
    W = max(1, min(W, T, 32))
    n = int(rng.integers(1, 9))
    cfgs = []
    for _ in range(n):
        bits = int(rng.choice([16, 8, 4, 2]))
        group = 0 if bits == 16 else int(rng.choice([32, 64, 128]))
        cfgs.append((bits, group, int(rng.choice([T, rng.integers(1, T + 1)]))))
    # at most 8 distinct keep levels
    levels = sorted({c[2] for c in cfgs})[:8]
    cfgs = [c for c in cfgs if c[2] in levels]
    print("[case] random eval", dict(seed=seed, L=L, H=H, T=T, G=G, W=W, cfgs=cfgs, pv=pv), flush=True)
    K, V = workloads.make_kv(L, T, H, D, seed=seed)
    Q = workloads.make_q(L, W, G * H, D, seed=seed)
    loss = kvp.kvp_eval_configs(Q.to(DEV), K.to(DEV), V.to(DEV), cfgs, **pv_kw)
    torch.cuda.synchronize()
    ref, _ = oracle.eval_configs(torch_bits(Q), torch_bits(K), torch_bits(V), cfgs)
    loss = loss.cpu().numpy()
    assert np.all(np.abs(loss - ref) <= 1e-2 * np.abs(ref) + 1e-5), (loss, ref)
