"""GPU parity: quantization groups along the token axis (per-channel codec), bit for bit against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import bits_to_torch, torch_bits
from test_gpu_quant import _asym_special_rows, _special_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _kvp():
    import paper_2512_14946_amd as kvp
    return kvp


def _say(*a):
    print("[case]", *a, flush=True)


def _check_plane(qp, ref):
    oc, os_, om = ref
    assert np.array_equal(qp.scales.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    if om is not None:
        assert np.array_equal(qp.mins.cpu().numpy().view(np.uint32), om.view(np.uint32))
    assert np.array_equal(qp.codes.cpu().numpy(), oc)


@pytest.mark.parametrize("asym", [False, True])
@pytest.mark.parametrize("group", [32, 64, 128])
@pytest.mark.parametrize("bits", [8, 4, 2])
def test_channel_quantize_dequantize_bit_exact(bits, group, asym):
    kvp = _kvp()
    L, T, H, D, bs = 2, 203, 8, 128, 16          # 203 slots: a ragged last group and a ragged last page
    _say("channel quant/dequant", bits, group, asym, (L, T, H, D))
    K, _ = workloads.make_kv(L, T, H, D, seed=bits * 10 + group + asym)
    xb = torch_bits(K).copy()
    sp = torch_bits(torch.from_numpy(np.concatenate([_special_rows(D), _asym_special_rows(D)])).to(torch.bfloat16))
    n = sp.shape[0]
    xb[0, :128, 0, :n] = sp.T                     # each special row runs along the tokens of one channel
    xb[1, T - 128:, 7, D - n:] = sp.T             # and again across the ragged tail
    x = bits_to_torch(xb, DEV)
    qp = kvp.alloc_qplane(L, T, H, D, bits, group, DEV, asymmetric=asym, per_channel=True)
    qp.codes.fill_(0xEE)
    qp.scales.fill_(float("nan"))
    if asym:
        qp.mins.fill_(float("nan"))
    kvp.kvp_quantize(x, qp)
    torch.cuda.synchronize()
    ref = oracle.quantize_channel(xb, bits, group, Tp=qp.Tp, asym=asym)
    _check_plane(qp, ref)

    bt, nb = workloads.make_block_table(T, bs, seed=5, spare=3, device=DEV)
    pg = kvp.alloc_paged(L, T, H, D, bt, nb, bs, fill_nan=True)
    kvp.kvp_dequantize_paged(qp, pg)
    torch.cuda.synchronize()
    opool = oracle.dequantize_paged_channel(*ref, bits, group, T, bt.cpu().numpy(), nb, bs,
                                            pool=torch_bits(torch.full((L, nb, bs, H, D), float("nan"),
                                                                       dtype=torch.bfloat16)).copy())
    assert np.array_equal(torch_bits(pg.pool), opool)


@pytest.mark.parametrize("H,bits,group,asym", [(4, 4, 32, True), (3, 2, 64, False), (12, 8, 128, True), (1, 4, 32, False),
                                               (12, 4, 64, False), (16, 2, 128, True)])
def test_channel_head_counts_strided_gathered_and_paged_sources(H, bits, group, asym):
    kvp = _kvp()
    L, T, D, bs = 2, 150, 128, 16
    _say("channel sources", H, bits, group, asym)
    K, _ = workloads.make_kv(L, T, H + 2, D, seed=13 + H)
    xb_full = torch_bits(K)
    xv = K.to(DEV)[:, :, 1:1 + H]                                            # strided view: heads 1..H of H+2
    xc = np.ascontiguousarray(xb_full[:, :, 1:1 + H])
    qp = kvp.alloc_qplane(L, T, H, D, bits, group, DEV, asymmetric=asym, per_channel=True)
    kvp.kvp_quantize(xv, qp)
    ref = oracle.quantize_channel(xc, bits, group, Tp=qp.Tp, asym=asym)
    torch.cuda.synchronize()
    _check_plane(qp, ref)
    # dequantize (exercises the per-row scale reload when H does not divide 16)
    bt, nb = workloads.make_block_table(T, bs, seed=H, spare=2, device=DEV)
    pg = kvp.alloc_paged(L, T, H, D, bt, nb, bs, fill_nan=True)
    kvp.kvp_dequantize_paged(qp, pg)
    torch.cuda.synchronize()
    opool = oracle.dequantize_paged_channel(*ref, bits, group, T, bt.cpu().numpy(), nb, bs,
                                            pool=torch_bits(torch.full((L, nb, bs, H, D), float("nan"),
                                                                       dtype=torch.bfloat16)).copy())
    assert np.array_equal(torch_bits(pg.pool), opool)
    # gathered, from the view and from a paged source
    rng = np.random.default_rng(7)
    k = 77
    keep = np.stack([[np.sort(rng.choice(T, k, replace=False)) for _ in range(H)] for _ in range(L)]).astype(np.int32)
    refg = oracle.quantize_channel(xc, bits, group, keep_idx=keep, Tp=80, asym=asym)
    qg = kvp.alloc_qplane(L, k, H, D, bits, group, DEV, asymmetric=asym, per_channel=True)
    assert qg.Tp == 80
    kvp.kvp_quantize(xv, qg, keep_idx=torch.from_numpy(keep).to(DEV))
    btn, nbs = workloads.make_block_table(T, bs, seed=21, spare=1)
    pool = np.zeros((L, nbs, bs, H, D), dtype=np.uint16)
    b = btn.numpy()
    for t in range(T):
        pool[:, b[t // bs], t % bs] = xc[:, t]
    src = kvp.PagedKV(bits_to_torch(pool, DEV), btn.to(DEV), T)
    qpg = kvp.alloc_qplane(L, k, H, D, bits, group, DEV, asymmetric=asym, per_channel=True)
    kvp.kvp_quantize(src, qpg, keep_idx=torch.from_numpy(keep).to(DEV))
    qpf = kvp.alloc_qplane(L, T, H, D, bits, group, DEV, asymmetric=asym, per_channel=True)
    kvp.kvp_quantize(src, qpf)
    torch.cuda.synchronize()
    _check_plane(qg, refg)
    _check_plane(qpg, refg)
    _check_plane(qpf, ref)


def test_channel_argument_errors():
    kvp = _kvp()
    _say("channel argument errors")
    L, T, H, D = 1, 128, 8, 128
    x = torch.zeros(L, T, H, D, dtype=torch.bfloat16, device=DEV)
    qp = kvp.alloc_qplane(L, T, H, D, 4, 32, DEV, per_channel=True)
    kvp.kvp_quantize(x, qp)
    bt, nb = workloads.make_block_table(T, 64, seed=0, device=DEV)
    pg = kvp.alloc_paged(L, T, H, D, bt, nb, 64)
    with pytest.raises(kvp.KVPError) as e:          # a 64-token page would straddle two 32-slot groups
        kvp.kvp_dequantize_paged(qp, pg)
    assert e.value.code == -4
    bad = kvp.QPlane(qp.codes, qp.scales, 4, 32, T, None, 2)
    with pytest.raises((kvp.KVPError, ValueError)):
        kvp.kvp_quantize(x, bad)
    torch.cuda.synchronize()


@pytest.mark.parametrize("bits,group,asym,per_channel,H", [(4, 64, False, False, 8), (2, 32, True, False, 3),
                                                           (8, 128, False, True, 8), (4, 32, True, True, 5),
                                                           (8, 32, True, False, 12), (2, 64, False, True, 4)])
def test_scatter_restore_to_original_positions(bits, group, asym, per_channel, H):
    kvp = _kvp()
    L, T, D, bs, k = 2, 333, 128, 16, 141
    _say("scatter restore", bits, group, asym, per_channel, H)
    K, _ = workloads.make_kv(L, T, H, D, seed=31 + H)
    xb = torch_bits(K)
    x = K.to(DEV)
    rng = np.random.default_rng(H)
    keep = np.stack([[np.sort(rng.choice(T, k, replace=False)) for _ in range(H)] for _ in range(L)]).astype(np.int32)
    keep_g = torch.from_numpy(keep).to(DEV)
    qp = kvp.alloc_qplane(L, k, H, D, bits, group, DEV, asymmetric=asym, per_channel=per_channel)
    kvp.kvp_quantize(x, qp, keep_idx=keep_g)
    bt, nb = workloads.make_block_table(T, bs, seed=8, spare=2, device=DEV)
    before = rng.integers(0, 0x7F80, (L, nb, bs, H, D)).astype(np.uint16)
    pool = bits_to_torch(before, DEV)
    pg = kvp.PagedKV(pool, bt, T)
    kvp.kvp_dequantize_paged_scatter(qp, keep_g, pg)
    torch.cuda.synchronize()
    codes, scales = qp.codes.cpu().numpy(), qp.scales.cpu().numpy()
    mins = qp.mins.cpu().numpy() if asym else None
    want = oracle.dequantize_paged_scatter(codes, scales, mins, bits, group, keep, T, bt.cpu().numpy(), nb, bs,
                                           pool=before.copy(), per_channel=per_channel)
    assert np.array_equal(torch_bits(pg.pool), want)
    # and the plane that was restored is the oracle's own (so the whole drop -> quantize -> restore chain is checked)
    if per_channel:
        ref = oracle.quantize_channel(xb, bits, group, keep_idx=keep, Tp=qp.Tp, asym=asym)
    elif asym:
        ref = oracle.quantize_asym(xb, bits, group, keep_idx=keep, Tp=qp.Tp)
    else:
        ref = oracle.quantize(xb, bits, group, keep_idx=keep, Tp=qp.Tp) + (None,)
    _check_plane(qp, ref)


def test_scatter_restore_errors():
    kvp = _kvp()
    _say("scatter errors")
    L, T, H, D, k = 1, 64, 2, 128, 16
    qp = kvp.alloc_qplane(L, k, H, D, 4, 64, DEV)
    qp.codes.zero_()
    qp.scales.zero_()
    bt, nb = workloads.make_block_table(T, 16, seed=0, device=DEV)
    pg = kvp.alloc_paged(L, T, H, D, bt, nb, 16)
    keep = torch.arange(k, dtype=torch.int32, device=DEV).repeat(L, H, 1).contiguous()
    kvp.kvp_dequantize_paged_scatter(qp, keep, pg)
    with pytest.raises(ValueError):
        kvp.kvp_dequantize_paged_scatter(qp, keep[:, :, :8].contiguous(), pg)
    small = kvp.alloc_paged(L, 8, H, D, bt[:1].contiguous(), nb, 16)     # pool shorter than the plane
    with pytest.raises(kvp.KVPError) as e:
        kvp.kvp_dequantize_paged_scatter(qp, keep, small)
    assert e.value.code == -3
    torch.cuda.synchronize()
