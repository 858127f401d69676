"""Pins for the oracle's per-channel (token-axis) group quantizer.

(1) hand-worked examples (tests/golden/channel_quant_examples.txt);
(2) reduction to the per-token quantizers, which are pinned on their own: a G-token tile of one
    head, transposed, is a set of rows whose single group is the G tokens of a channel;
(3) exact rational IEEE arithmetic on random tiles with ragged tails and keep lists;
(4) invariants: error bound, padding, ragged groups ignore padding, outlier channels isolated.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads
from helpers import bits_to_f32, fl32, flbf16, frac_of_f32, rint_even, to_bf16_bits, torch_bits

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "channel_quant_examples.txt")


def _blocks():
    out, cur = [], {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":", 1)
        if key == "name" and cur:
            out.append(cur)
            cur = {}
        cur[key.strip()] = val.strip()
    out.append(cur)
    return out


def _matrix(text, conv):
    return [[conv(tok) for tok in row.split()] for row in text.split(";")]


def _unpack(codes, bits, signed):
    per = 8 // bits
    c = codes.astype(np.int32)
    f = np.stack([(c >> (bits * i)) & ((1 << bits) - 1) for i in range(per)], axis=-1).reshape(*codes.shape[:-1], -1)
    if signed:
        f = np.where(f >= (1 << (bits - 1)), f - (1 << bits), f)
    return f


@pytest.mark.parametrize("case", _blocks(), ids=lambda c: c["name"])
def test_hand_worked_examples(case):
    bits, group, asym = int(case["bits"]), int(case["group"]), bool(int(case["asym"]))
    x = np.array(_matrix(case["x"], float), dtype=np.float32)                # [T][D]
    T, D = x.shape
    xb = to_bf16_bits(x).reshape(1, T, 1, D)
    assert np.array_equal(bits_to_f32(xb).reshape(T, D), x)                   # inputs are exact bf16
    codes, scales, mins = oracle.quantize_channel(xb, bits, group, asym=asym)
    want_codes = np.array(_matrix(case["codes"], lambda s: int(s, 16)), dtype=np.uint8)
    want_scales = np.array(_matrix(case["scales"], lambda s: int(s, 16)), dtype=np.uint32)
    assert np.array_equal(codes.reshape(T, -1), want_codes)
    assert np.array_equal(scales.view(np.uint32).reshape(want_scales.shape), want_scales)
    if asym:
        want_mins = np.array(_matrix(case["mins"], lambda s: int(s, 16)), dtype=np.uint32)
        assert np.array_equal(mins.view(np.uint32).reshape(want_mins.shape), want_mins)
    bs = 2
    nb = (T + bs - 1) // bs
    pool = oracle.dequantize_paged_channel(codes, scales, mins, bits, group, T, np.arange(nb, dtype=np.int32), nb, bs)
    want = np.array(_matrix(case["dequant"], float), dtype=np.float32)
    assert np.array_equal(bits_to_f32(pool).reshape(-1, D)[:T], want)


@pytest.mark.parametrize("bits", [8, 4, 2])
@pytest.mark.parametrize("asym", [False, True])
def test_reduces_to_per_token_quantizer_on_transposed_tile(bits, asym):
    G, D = 32, 128
    K, _ = workloads.make_kv(1, 3 * G, 1, D, seed=5)
    xb = torch_bits(K)                                                       # [1][96][1][128]
    codes, scales, mins = oracle.quantize_channel(xb, bits, G, asym=asym)
    q = _unpack(codes, bits, signed=not asym)[0, :, 0]                        # [96][128]
    for g in range(3):
        tile = np.ascontiguousarray(xb[0, g * G:(g + 1) * G, 0].T).reshape(1, D, 1, G)   # rows = channels, D' = G tokens
        if asym:
            c2, s2, m2 = oracle.quantize_asym(tile, bits, G)
            assert np.array_equal(mins[0, g, 0].view(np.uint32), m2[0, :, 0, 0].view(np.uint32))
        else:
            c2, s2 = oracle.quantize(tile, bits, G)
        assert np.array_equal(scales[0, g, 0].view(np.uint32), s2[0, :, 0, 0].view(np.uint32))
        assert np.array_equal(q[g * G:(g + 1) * G].T, _unpack(c2, bits, signed=not asym)[0, :, 0])


@pytest.mark.parametrize("bits,asym", [(8, False), (4, True), (2, False), (2, True)])
def test_exact_rational_arithmetic_ragged_and_gathered(bits, asym):
    L, T, H, D, G = 2, 45, 2, 8, 16
    rng = np.random.default_rng(bits + 10 * asym)
    x = np.round(rng.standard_normal((L, T, H, D)) * 8) / 8                  # dyadic values: plenty of exact ties
    x[0, :, 0, 3] *= 16
    xb = to_bf16_bits(x.astype(np.float32))
    k = 21
    keep = np.stack([[np.sort(rng.choice(T, k, replace=False)) for _ in range(H)] for _ in range(L)]).astype(np.int32)
    for keep_idx, n_slots, Tp in ((None, T, 48), (keep, k, 32)):
        codes, scales, mins = oracle.quantize_channel(xb, bits, G, keep_idx=keep_idx, Tp=Tp, asym=asym)
        q = _unpack(codes, bits, signed=not asym)
        qmax, levels = (1 << (bits - 1)) - 1, (1 << bits) - 1
        ng = (Tp + G - 1) // G
        assert scales.shape == (L, ng, H, D)
        for l in range(L):
            for h in range(H):
                for c in range(D):
                    for g in range(ng):
                        slots = range(g * G, min((g + 1) * G, n_slots))
                        toks = [int(keep_idx[l, h, i]) if keep_idx is not None else i for i in slots]
                        vals = [frac_of_f32(bits_to_f32(xb[l, t, h, c:c + 1])[0]) for t in toks]
                        if not vals:
                            assert scales[l, g, h, c] == 0 and (mins is None or mins[l, g, h, c] == 0)
                            continue
                        if asym:
                            mn = min(vals)
                            sc = fl32(fl32(max(vals) - mn) / levels)
                            assert frac_of_f32(mins[l, g, h, c]) == mn
                        else:
                            mn = Fraction(0)
                            sc = fl32(max(abs(v) for v in vals) / qmax)
                        assert frac_of_f32(scales[l, g, h, c]) == sc
                        for i, v in zip(slots, vals):
                            if sc == 0:
                                want = 0
                            elif asym:
                                want = min(levels, max(0, rint_even(fl32(fl32(v - mn) / sc))))
                            else:
                                want = min(qmax, max(-qmax, rint_even(fl32(v / sc))))
                            assert q[l, i, h, c] == want, (l, i, h, c)
        assert not codes[:, n_slots:].any()                                   # padding slots hold zero codes
        # dequantization, exactly
        bs = 16
        nb = (n_slots + bs - 1) // bs
        pool = oracle.dequantize_paged_channel(codes, scales, mins, bits, G, n_slots, np.arange(nb, dtype=np.int32), nb, bs)
        y = bits_to_f32(pool).reshape(L, nb * bs, H, D)
        for l in range(L):
            for i in range(0, n_slots, 5):
                for h in range(H):
                    for c in range(D):
                        sc = frac_of_f32(scales[l, i // G, h, c])
                        prod = fl32(int(q[l, i, h, c]) * sc)
                        if asym:
                            prod = fl32(prod + frac_of_f32(mins[l, i // G, h, c]))
                        assert frac_of_f32(y[l, i, h, c]) == flbf16(prod)
        assert np.all(pool.reshape(L, nb * bs, H, D)[:, n_slots:] == 0x7FC0)  # slots past T untouched


@pytest.mark.parametrize("bits,G", [(4, 32), (2, 128), (8, 64)])
def test_invariants_and_outlier_channel_isolation(bits, G):
    L, T, H, D = 2, 300, 2, 128
    K, _ = workloads.make_kv(L, T, H, D, seed=3)
    xb = torch_bits(K)
    x = bits_to_f32(xb).astype(np.float64)
    bs = 16
    nb = (T + bs - 1) // bs
    err = {}
    for asym in (False, True):
        codes, scales, mins = oracle.quantize_channel(xb, bits, G, asym=asym, Tp=nb * bs)
        pool = oracle.dequantize_paged_channel(codes, scales, mins, bits, G, T, np.arange(nb, dtype=np.int32), nb, bs)
        y = bits_to_f32(pool).reshape(L, nb * bs, H, D)[:, :T].astype(np.float64)
        s = np.repeat(scales.astype(np.float64), G, axis=1)[:, :T]
        # |x - y| <= scale/2 plus the bf16 rounding of the reconstruction
        assert np.all(np.abs(x - y) <= 0.5 * s * (1 + 2.0 ** -20) + np.abs(y) * 2.0 ** -8 + 1e-30)
        err[asym] = np.mean((x - y) ** 2)
        # a ragged last group sees only its real members: quantizing the tail alone gives the same bytes
        t0 = (T // G) * G
        c2, s2, m2 = oracle.quantize_channel(np.ascontiguousarray(xb[:, t0:]), bits, G, asym=asym)
        assert np.array_equal(c2, codes[:, t0:T])
        assert np.array_equal(s2[:, 0].view(np.uint32), scales[:, T // G].view(np.uint32))
    # per-channel groups isolate the generator's outlier channels: smaller error than per-token groups of
    # the same size at the same number of bits
    ct, st = oracle.quantize(xb, bits, min(G, D))
    yt = bits_to_f32(oracle.dequantize_paged(ct, st, bits, min(G, D), T, np.arange(nb, dtype=np.int32), nb, bs)
                     ).reshape(L, nb * bs, H, D)[:, :T]
    if bits >= 4:       # (a ternary code cannot use the finer per-channel scale of N(0,1) data: no claim there)
        assert err[False] < np.mean((x - yt) ** 2)
    assert err[True] < err[False]   # the zero-point variant spends its levels on [min, max] only
