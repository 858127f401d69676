"""Pins for the oracle's scatter restore (dropped+quantized plane back to the original token positions).

The element arithmetic is that of the compact dequantizers, which are pinned on their own; what is new
is index movement.  So: (1) the result equals the compact restore followed by a numpy scatter, for all
four codecs; (2) dropped positions keep their previous contents; (3) a tiny brute force spells out
the destination address with a non-trivial block table.
"""
import numpy as np
import pytest

import oracle
import workloads
from helpers import torch_bits


def _keep(rng, L, H, T, k):
    return np.stack([[np.sort(rng.choice(T, k, replace=False)) for _ in range(H)] for _ in range(L)]).astype(np.int32)


@pytest.mark.parametrize("bits,group,asym,per_channel", [(4, 64, False, False), (2, 32, True, False), (8, 32, False, True),
                                                         (4, 32, True, True)])
def test_equals_compact_restore_then_scatter(bits, group, asym, per_channel):
    L, T, H, D, bs, k = 2, 100, 3, 128, 16, 37
    rng = np.random.default_rng(bits + group)
    K, _ = workloads.make_kv(L, T, H, D, seed=2)
    xb = torch_bits(K)
    keep = _keep(rng, L, H, T, k)
    Tp = 48
    if per_channel:
        codes, scales, mins = oracle.quantize_channel(xb, bits, group, keep_idx=keep, Tp=Tp, asym=asym)
        compact = oracle.dequantize_paged_channel(codes, scales, mins, bits, group, k, np.arange(3, dtype=np.int32), 3, bs)
    elif asym:
        codes, scales, mins = oracle.quantize_asym(xb, bits, group, keep_idx=keep, Tp=Tp)
        compact = oracle.dequantize_paged_asym(codes, scales, mins, bits, group, k, np.arange(3, dtype=np.int32), 3, bs)
    else:
        codes, scales = oracle.quantize(xb, bits, group, keep_idx=keep, Tp=Tp)
        mins = None
        compact = oracle.dequantize_paged(codes, scales, bits, group, k, np.arange(3, dtype=np.int32), 3, bs)
    compact = compact.reshape(L, 3 * bs, H, D)[:, :k]                          # [L][k][H][D]
    bt, nb = workloads.make_block_table(T, bs, seed=1, spare=2)
    bt = bt.numpy()
    before = np.random.default_rng(9).integers(0, 0x7F80, (L, nb, bs, H, D)).astype(np.uint16)
    got = oracle.dequantize_paged_scatter(codes, scales, mins, bits, group, keep, T, bt, nb, bs, pool=before.copy(),
                                          per_channel=per_channel)
    want = before.copy()
    for l in range(L):
        for h in range(H):
            for i in range(k):
                t = keep[l, h, i]
                want[l, bt[t // bs], t % bs, h] = compact[l, i, h]
    assert np.array_equal(got, want)
    # the kept rows are the quantization of the source rows: close to them
    x = xb.astype(np.uint32) << 16
    y = got.astype(np.uint32) << 16
    xs = x.view(np.float32)[0, keep[0, 1], 1]
    ys = y.view(np.float32)[0, bt[keep[0, 1] // bs], keep[0, 1] % bs, 1]
    assert np.mean((xs - ys) ** 2) < np.mean(xs ** 2)


def test_tiny_brute_force_addresses():
    # 1 layer, 2 heads, D = 8 (int8, one group): slot i of head h lands at pool[bt[t//bs]][t%bs][h]
    L, T, H, D, bs, k = 1, 6, 2, 8, 2, 2
    x = (np.arange(L * T * H * D, dtype=np.float32).reshape(L, T, H, D) % 13 - 6) * 0.5
    from helpers import to_bf16_bits, bits_to_f32
    xb = to_bf16_bits(x)
    keep = np.array([[[1, 4], [0, 5]]], dtype=np.int32)
    codes, scales = oracle.quantize(xb, 8, 8, keep_idx=keep)
    bt = np.array([2, 0, 3], dtype=np.int32)
    pool = oracle.dequantize_paged_scatter(codes, scales, None, 8, 8, keep, T, bt, 4, bs, fill=0x7FC0)
    y = bits_to_f32(pool)                                                       # [1][4][2][2][8]
    deq = lambda i, h: bits_to_f32(oracle.dequantize_paged(codes[:, i:i + 1, h:h + 1], scales[:, i:i + 1, h:h + 1], 8, 8, 1,
                                                           np.zeros(1, np.int32), 1, 1))[0, 0, 0, 0]
    assert np.array_equal(y[0, 2, 1, 0], deq(0, 0))       # head 0 slot 0 <- token 1: page 0 -> block 2, offset 1
    assert np.array_equal(y[0, 3, 0, 0], deq(1, 0))       # head 0 slot 1 <- token 4: page 2 -> block 3, offset 0
    assert np.array_equal(y[0, 2, 0, 1], deq(0, 1))       # head 1 slot 0 <- token 0: block 2, offset 0
    assert np.array_equal(y[0, 3, 1, 1], deq(1, 1))       # head 1 slot 1 <- token 5: block 3, offset 1
    written = np.zeros((4, 2, 2), dtype=bool)
    for (b, o, h) in [(2, 1, 0), (3, 0, 0), (2, 0, 1), (3, 1, 1)]:
        written[b, o, h] = True
    assert np.all(pool[0][~written] == 0x7FC0)            # every other row untouched
    assert np.allclose(y[0, 2, 1, 0], x[0, 1, 0], atol=0.02)
