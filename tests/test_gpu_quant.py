"""GPU parity: kvp_quantize / kvp_dequantize_paged against the CPU oracle, bit for bit.

Every case prints its name before touching the GPU so that a fault names its case.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import bits_to_torch, torch_bits

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
ALL_CODECS = [(8, 128), (8, 64), (8, 32), (4, 128), (4, 64), (4, 32), (2, 128), (2, 64), (2, 32)]


def _kvp():
    import paper_2512_14946_amd as kvp
    return kvp


def _say(*a):
    print("[case]", *a, flush=True)


def _special_rows(D=128):
    """Rows that exercise ties, zeros, tiny and huge magnitudes, mixed-scale groups."""
    rng = np.random.default_rng(7)
    rows = []
    rows.append(np.zeros(D))                                               # all zero
    rows.append(np.where(np.arange(D) % 2 == 0, 3.0, -3.0))                # constant magnitude
    rows.append(np.round(rng.standard_normal(D) * 4) / 4)                  # dyadic: exact .5 ties
    rows.append(np.round(rng.standard_normal(D) * 16) / 16 * 7)            # multiples of 7/16: ties vs qmax 7
    rows.append(np.round(rng.standard_normal(D) * 8) / 8 * 127)            # ties vs qmax 127
    rows.append(rng.standard_normal(D) * 2.0 ** -60)                       # tiny but inside the graded range
    rows.append(rng.standard_normal(D) * 2.0 ** 60)                        # huge
    rows.append(rng.standard_normal(D) * 2.0 ** -45)                       # well inside the fast-path range
    rows.append(rng.standard_normal(D) * 2.0 ** 45)
    rows.append(rng.standard_normal(D) * 2.0 ** -110)                      # below the fast-path range
    rows.append(rng.standard_normal(D) * 2.0 ** 110)                       # above the fast-path range
    r = rng.standard_normal(D)
    r[:32] = 0.0                                                           # one zero group among non-zero ones
    rows.append(r)
    r = rng.standard_normal(D)
    r[5] = 1000.0                                                          # one outlier per row
    rows.append(r)
    rows.append(np.full(D, 2.0 ** -120))                                   # subnormal scales
    return np.stack(rows).astype(np.float32)


@pytest.mark.parametrize("bits,group", ALL_CODECS)
def test_quantize_dequantize_bit_exact(bits, group):
    kvp = _kvp()
    L, T, H, D, bs = 3, 203, 8, 128, 16          # 203 tokens: several blocks and a ragged tail page
    _say("quant/dequant", bits, group, (L, T, H, D))
    K, _ = workloads.make_kv(L, T, H, D, seed=bits * 10 + group)
    xb = torch_bits(K).copy()
    sp = torch_bits(torch.from_numpy(_special_rows(D)).to(torch.bfloat16))
    xb[0, :sp.shape[0], 0] = sp
    xb[2, -sp.shape[0]:, 7] = sp
    x = bits_to_torch(xb, DEV)
    qp = kvp.alloc_qplane(L, T, H, D, bits, group, DEV)
    qp.codes.fill_(0xEE)
    qp.scales.fill_(float("nan"))
    kvp.kvp_quantize(x, qp)
    torch.cuda.synchronize()
    ocodes, oscales = oracle.quantize(xb, bits, group, Tp=qp.Tp)
    assert np.array_equal(qp.codes.cpu().numpy(), ocodes)
    assert np.array_equal(qp.scales.cpu().numpy().view(np.uint32), oscales.view(np.uint32))

    bt, nb = workloads.make_block_table(T, bs, seed=3, spare=3, device=DEV)
    pg = kvp.alloc_paged(L, T, H, D, bt, nb, bs, fill_nan=True)
    kvp.kvp_dequantize_paged(qp, pg)
    torch.cuda.synchronize()
    opool = oracle.dequantize_paged(ocodes, oscales, bits, group, T, bt.cpu().numpy(), nb, bs,
                                    pool=torch_bits(torch.full((L, nb, bs, H, D), float("nan"),
                                                               dtype=torch.bfloat16)).copy())
    assert np.array_equal(torch_bits(pg.pool), opool)


@pytest.mark.parametrize("bits,group", [(8, 128), (4, 32), (2, 64)])
def test_quantize_strided_gather_paged_sources(bits, group):
    kvp = _kvp()
    L, T, H, D, bs = 2, 150, 4, 128, 16
    _say("quant sources", bits, group)
    K, V = workloads.make_kv(L, T, H + 2, D, seed=11)
    xb_full = torch_bits(K)
    x_full = K.to(DEV)
    # (a) strided view: heads 1..4 of a 6-head tensor
    xv = x_full[:, :, 1:1 + H]
    qp = kvp.alloc_qplane(L, T, H, D, bits, group, DEV)
    kvp.kvp_quantize(xv, qp)
    oc, os_ = oracle.quantize(xb_full[:, :, 1:1 + H], bits, group, Tp=qp.Tp)
    torch.cuda.synchronize()
    assert np.array_equal(qp.codes.cpu().numpy(), oc)
    assert np.array_equal(qp.scales.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    # (b) gathered: per-head keep lists
    rng = np.random.default_rng(5)
    k = 37
    keep = np.stack([[np.sort(rng.choice(T, k, replace=False)) for _ in range(H)] for _ in range(L)]).astype(np.int32)
    qg = kvp.alloc_qplane(L, k, H, D, bits, group, DEV)
    kvp.kvp_quantize(xv, qg, keep_idx=torch.from_numpy(keep).to(DEV))
    og, ogs = oracle.quantize(xb_full[:, :, 1:1 + H], bits, group, keep_idx=keep, Tp=qg.Tp)
    torch.cuda.synchronize()
    assert np.array_equal(qg.codes.cpu().numpy(), og)
    assert np.array_equal(qg.scales.cpu().numpy().view(np.uint32), ogs.view(np.uint32))
    # (c) paged source, flat and gathered
    xc = np.ascontiguousarray(xb_full[:, :, 1:1 + H])
    bt, nb = workloads.make_block_table(T, bs, seed=9, spare=1)
    pool = np.zeros((L, nb, bs, H, D), dtype=np.uint16)
    btn = bt.numpy()
    for t in range(T):
        pool[:, btn[t // bs], t % bs] = xc[:, t]
    src = kvp.PagedKV(bits_to_torch(pool, DEV), bt.to(DEV), T)
    qpp = kvp.alloc_qplane(L, T, H, D, bits, group, DEV)
    kvp.kvp_quantize(src, qpp)
    qpg = kvp.alloc_qplane(L, k, H, D, bits, group, DEV)
    kvp.kvp_quantize(src, qpg, keep_idx=torch.from_numpy(keep).to(DEV))
    torch.cuda.synchronize()
    assert np.array_equal(qpp.codes.cpu().numpy(), oc) and np.array_equal(qpp.scales.cpu().numpy(), os_)
    assert np.array_equal(qpg.codes.cpu().numpy(), og) and np.array_equal(qpg.scales.cpu().numpy(), ogs)


def test_quantize_argument_errors_enqueue_nothing():
    kvp = _kvp()
    _say("argument errors")
    x = torch.zeros(1, 16, 8, 128, dtype=torch.bfloat16, device=DEV)
    qp = kvp.alloc_qplane(1, 16, 8, 128, 4, 64, DEV)
    bad = kvp.QPlane(qp.codes, qp.scales, 4, 64, 15)            # T mismatch
    with pytest.raises(kvp.KVPError) as e:
        kvp.kvp_quantize(x, bad)
    assert e.value.code == -3
    bad = kvp.QPlane(qp.codes, qp.scales.view(1, 16, 8, -1), 3, 64, 16)
    with pytest.raises((kvp.KVPError, ValueError)):
        kvp.kvp_quantize(x, bad)
    x64 = torch.zeros(1, 16, 8, 64, dtype=torch.bfloat16, device=DEV)
    q64 = kvp.alloc_qplane(1, 16, 8, 64, 4, 32, DEV)
    with pytest.raises(kvp.KVPError) as e:
        kvp.kvp_quantize(x64, q64)
    assert e.value.code == -4
    with pytest.raises(kvp.KVPError) as e:                       # misaligned view
        kvp.kvp_quantize(x.view(-1)[4:4 + 8 * 8 * 128].view(1, 8, 8, 128), kvp.alloc_qplane(1, 8, 8, 128, 4, 64, DEV))
    assert e.value.code == -2
    torch.cuda.synchronize()


@pytest.mark.parametrize("bits", [8, 4])
def test_scale_exact_for_every_bf16_amax(bits):
    # the kernel derives the scale from the group abs-max with a short fma sequence instead of a
    # division: check it against the oracle's IEEE division for every finite bf16 magnitude
    kvp = _kvp()
    _say("all bf16 amax", bits)
    mags = np.arange(0, 0x7F80, dtype=np.uint16)                    # every finite non-negative bf16
    n = len(mags)
    T = (n + 7) // 8
    xb = np.zeros((1, T, 8, 128), dtype=np.uint16)
    flat = xb.reshape(-1, 128)
    flat[:n, 3] = mags                                             # group 0 of each row
    flat[:n, 40] = mags | 0x8000                                   # group 1: the same magnitude, negative
    flat[:n, 41] = (mags >> 1)                                     # plus some smaller element
    x = bits_to_torch(xb, DEV)
    qp = kvp.alloc_qplane(1, T, 8, 128, bits, 32, DEV)
    kvp.kvp_quantize(x, qp)
    torch.cuda.synchronize()
    oc, os_ = oracle.quantize(xb, bits, 32, Tp=qp.Tp)
    assert np.array_equal(qp.scales.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    assert np.array_equal(qp.codes.cpu().numpy(), oc)


def _asym_special_rows(D=128):
    """Rows whose (x - min)/scale lands on exact .5 ties, plus degenerate ranges."""
    rng = np.random.default_rng(17)
    rows = []
    for levels in (3, 15, 255):
        # halves on [-a, levels - a]: scale is exactly 1 when both ends are present in every group
        r = rng.integers(0, 2 * levels + 1, D) / 2.0 - 4.0
        r[::32] = -4.0
        r[1::32] = levels - 4.0
        rows.append(r)
        # the same grid scaled by 3/8 (scale = 0.375, ties stay exact)
        rows.append(r * 0.375)
    rows.append(np.full(D, 1.5))                                           # constant group: range 0
    rows.append(np.where(np.arange(D) % 2 == 0, 0.0, -0.0))                # +0 / -0 only
    rows.append(np.where(np.arange(D) % 2 == 0, -0.0, 0.0))                # -0 first
    rows.append(np.full(D, -0.0))                                          # -0 only: min, range, scale all +0
    r = -np.abs(rng.standard_normal(D))
    r[3::8] = -0.0                                                         # maximum is a negative zero
    rows.append(r)
    rows.append(np.abs(rng.standard_normal(D)) + 100.0)                    # far from zero: x - min is exact, range small
    rows.append(-np.abs(rng.standard_normal(D)) * 2.0 ** 40)               # all negative, large
    r = rng.standard_normal(D) * 2.0 ** -8
    r[7] = 900.0                                                           # one-sided outlier
    rows.append(r)
    return np.stack(rows).astype(np.float32)


@pytest.mark.parametrize("bits,group", ALL_CODECS)
def test_asymmetric_quantize_dequantize_bit_exact(bits, group):
    kvp = _kvp()
    L, T, H, D, bs = 3, 203, 8, 128, 16
    _say("asym quant/dequant", bits, group, (L, T, H, D))
    _, V = workloads.make_kv(L, T, H, D, seed=bits * 10 + group + 1)
    xb = torch_bits(V).copy()
    sp = torch_bits(torch.from_numpy(np.concatenate([_special_rows(D), _asym_special_rows(D)])).to(torch.bfloat16))
    xb[0, :sp.shape[0], 0] = sp
    xb[2, -sp.shape[0]:, 7] = sp
    x = bits_to_torch(xb, DEV)
    qp = kvp.alloc_qplane(L, T, H, D, bits, group, DEV, asymmetric=True)
    qp.codes.fill_(0xEE)
    qp.scales.fill_(float("nan"))
    qp.mins.fill_(float("nan"))
    kvp.kvp_quantize(x, qp)
    torch.cuda.synchronize()
    ocodes, oscales, omins = oracle.quantize_asym(xb, bits, group, Tp=qp.Tp)
    assert np.array_equal(qp.scales.cpu().numpy().view(np.uint32), oscales.view(np.uint32))
    assert np.array_equal(qp.mins.cpu().numpy().view(np.uint32), omins.view(np.uint32))
    assert np.array_equal(qp.codes.cpu().numpy(), ocodes)

    bt, nb = workloads.make_block_table(T, bs, seed=4, spare=3, device=DEV)
    pg = kvp.alloc_paged(L, T, H, D, bt, nb, bs, fill_nan=True)
    kvp.kvp_dequantize_paged(qp, pg)
    torch.cuda.synchronize()
    opool = oracle.dequantize_paged_asym(ocodes, oscales, omins, bits, group, T, bt.cpu().numpy(), nb, bs,
                                         pool=torch_bits(torch.full((L, nb, bs, H, D), float("nan"),
                                                                    dtype=torch.bfloat16)).copy())
    assert np.array_equal(torch_bits(pg.pool), opool)


@pytest.mark.parametrize("bits,group", [(4, 64), (2, 32)])
def test_asymmetric_gather_and_paged_sources(bits, group):
    kvp = _kvp()
    L, T, H, D, bs = 2, 150, 4, 128, 16
    _say("asym sources", bits, group)
    _, V = workloads.make_kv(L, T, H + 2, D, seed=12)
    xb_full = torch_bits(V)
    xv = V.to(DEV)[:, :, 1:1 + H]
    xc = np.ascontiguousarray(xb_full[:, :, 1:1 + H])
    rng = np.random.default_rng(6)
    k = 41
    keep = np.stack([[np.sort(rng.choice(T, k, replace=False)) for _ in range(H)] for _ in range(L)]).astype(np.int32)
    og = oracle.quantize_asym(xc, bits, group, keep_idx=keep, Tp=48)
    qg = kvp.alloc_qplane(L, k, H, D, bits, group, DEV, asymmetric=True)
    assert qg.Tp == 48
    kvp.kvp_quantize(xv, qg, keep_idx=torch.from_numpy(keep).to(DEV))
    bt, nb = workloads.make_block_table(T, bs, seed=10, spare=1)
    pool = np.zeros((L, nb, bs, H, D), dtype=np.uint16)
    btn = bt.numpy()
    for t in range(T):
        pool[:, btn[t // bs], t % bs] = xc[:, t]
    src = kvp.PagedKV(bits_to_torch(pool, DEV), bt.to(DEV), T)
    qpg = kvp.alloc_qplane(L, k, H, D, bits, group, DEV, asymmetric=True)
    kvp.kvp_quantize(src, qpg, keep_idx=torch.from_numpy(keep).to(DEV))
    torch.cuda.synchronize()
    for q in (qg, qpg):
        assert np.array_equal(q.codes.cpu().numpy(), og[0])
        assert np.array_equal(q.scales.cpu().numpy().view(np.uint32), og[1].view(np.uint32))
        assert np.array_equal(q.mins.cpu().numpy().view(np.uint32), og[2].view(np.uint32))


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_asymmetric_scale_exact_for_many_ranges(bits):
    # the kernel forms range / (2^bits - 1) without a division instruction: check scale, min and codes
    # against the oracle's IEEE arithmetic for every finite bf16 maximum over a zero minimum and for
    # 2^18 random (min, max) pairs whose difference has a full-width significand
    kvp = _kvp()
    _say("asym ranges", bits)
    rng = np.random.default_rng(bits)
    mags = np.arange(0, 0x7F00, dtype=np.uint16)
    n_pairs = 1 << 18
    n = len(mags) + n_pairs
    T = (n + 7) // 8
    xb = np.zeros((1, T, 8, 128), dtype=np.uint16)
    flat = xb.reshape(-1, 128)
    flat[:len(mags), 5] = mags                                              # group 0: min 0, max = every bf16
    flat[:len(mags), 40] = mags | 0x8000                                    # group 1: max 0, min = every -bf16
    e = rng.integers(100, 150, n_pairs).astype(np.uint16)                   # exponents near each other
    hi = ((e << 7) | rng.integers(0, 128, n_pairs).astype(np.uint16))
    lo = (((e - rng.integers(0, 9, n_pairs).astype(np.uint16)) << 7) | rng.integers(0, 128, n_pairs).astype(np.uint16))
    sl = slice(len(mags), n)
    flat[sl, :] = lo[:, None]                                               # every element at the minimum ...
    flat[sl, 3::32] = hi[:, None]                                           # ... one maximum per 32 channels
    flat[sl, 9::32] = (lo + 1)[:, None]                                     # and a near-minimum element
    flat[sl, :64] |= 0x8000                                                 # first half negated: min = -hi
    x = bits_to_torch(xb, DEV)
    qp = kvp.alloc_qplane(1, T, 8, 128, bits, 32, DEV, asymmetric=True)
    kvp.kvp_quantize(x, qp)
    torch.cuda.synchronize()
    oc, os_, om = oracle.quantize_asym(xb, bits, 32, Tp=qp.Tp)
    assert np.array_equal(qp.scales.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    assert np.array_equal(qp.mins.cpu().numpy().view(np.uint32), om.view(np.uint32))
    assert np.array_equal(qp.codes.cpu().numpy(), oc)


def test_hip_graph_replays_match_eager():
    # the library neither allocates nor synchronizes, so its calls can be captured; every replay must give
    # the eager result, with eager work and synchronizations between the replays
    kvp = _kvp()
    _say("hip graph replay")
    L, T, H, D, bs = 2, 300, 8, 128, 16
    K, V = workloads.make_kv(L, T, H, D, seed=77)
    Kd, Vd = K.to(DEV), V.to(DEV)
    qp = kvp.alloc_qplane(L, T, H, D, 4, 64, DEV)
    bt, nb = workloads.make_block_table(T, bs, seed=2, device=DEV)
    pg = kvp.alloc_paged(L, T, H, D, bt, nb, bs)
    x = torch.empty_like(Kd)

    def step():
        kvp.kvp_quantize(x, qp)
        kvp.kvp_dequantize_paged(qp, pg)

    x.copy_(Kd)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    for rep, src in enumerate([Kd, Vd, Kd, Vd]):
        x.copy_(src)                             # eager work between the replays
        qp.codes.fill_(0xEE)
        pg.pool.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        got_codes, got_pool = qp.codes.clone(), pg.pool.clone()
        step()                                   # the eager result for the same input
        torch.cuda.synchronize()
        assert torch.equal(got_codes, qp.codes), rep
        assert torch.equal(got_pool.view(torch.int16), pg.pool.view(torch.int16)), rep
    oc, _ = oracle.quantize(torch_bits(V), 4, 64, Tp=qp.Tp)
    assert np.array_equal(qp.codes.cpu().numpy(), oc)


def test_corrected_hardware_reciprocal_equals_ieee_division_on_this_device():
    # the asymmetric quantizer forms fl32(1 / scale) without a division; the library re-proves on the running GPU
    # that this equals the IEEE quotient for every operand of the range it is used in (2^23 significands x 121 exponents)
    kvp = _kvp()
    _say("reciprocal self-test")
    assert kvp.kvp_selftest_reciprocal() == 0
