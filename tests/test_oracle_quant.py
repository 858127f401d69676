"""Pins for the oracle's group-wise quantize / dequantize_paged (CPU only).

The paper gives no formula for the quantization category (Background, "KV
cache compression"), so these pins fix the stated reading: symmetric abs-max
scaling, IEEE binary32 division, round-half-to-even, little-endian packing.
They check the oracle against things other than itself: hand-worked dyadic
examples (tests/golden/quant_examples.txt), exact rational arithmetic with
explicit IEEE rounding, invariants, special cases and a library conversion.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads
from helpers import (bits_to_f32, fl32, flbf16, frac_of_f32, rint_even, to_bf16_bits, torch_bits)

QMAX = {8: 127, 4: 7, 2: 1}
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quant_examples.txt")


def _row(vals):
    return to_bf16_bits(np.array(vals, dtype=np.float32)).reshape(1, 1, 1, -1)


def _unpack(codes: np.ndarray, bits: int) -> np.ndarray:
    """Packed bytes [..., nbytes] -> signed codes [..., nbytes*8/bits] (test-side, for the invariants)."""
    per = 8 // bits
    c = codes.astype(np.int32)
    fields = np.stack([(c >> (bits * i)) & ((1 << bits) - 1) for i in range(per)], axis=-1)
    fields = np.where(fields >= (1 << (bits - 1)), fields - (1 << bits), fields)
    return fields.reshape(*codes.shape[:-1], codes.shape[-1] * per)


def _golden_cases(asym=False):
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split("|")]
            name, bits, xs, scale_hex, bytes_hex = parts[:5]
            if name.startswith("asym_") != asym:
                continue
            case = (name, int(bits), [float(v) for v in xs.split()], int(scale_hex, 16),
                    [int(b, 16) for b in bytes_hex.split()])
            cases.append(case + ((int(parts[5], 16),) if asym else ()))
    return cases


@pytest.mark.parametrize("name,bits,xs,scale_bits,expect_bytes", _golden_cases(), ids=lambda c: str(c)[:24])
def test_hand_worked_examples(name, bits, xs, scale_bits, expect_bytes):
    x = _row(xs)
    codes, scales = oracle.quantize(x, bits, len(xs))
    assert scales.view(np.uint32).ravel().tolist() == [scale_bits], name
    assert codes.ravel().tolist() == expect_bytes, name


def test_division_not_reciprocal():
    # -0.5 / fl(1/7) rounds to -3.4999998 -> -3; multiplying by 7 would give -3.5 -> -4.
    x = _row([1.0, -0.5, 0.25, 0.0])
    codes, scales = oracle.quantize(x, 4, 4)
    assert _unpack(codes, 4).ravel().tolist() == [7, -3, 2, 0]
    assert Fraction(float(scales.ravel()[0])) == fl32(Fraction(1, 7))


def _expected_row(xbits: np.ndarray, bits: int, group: int):
    """Codes and scales of one row from exact rationals + explicit IEEE rounding."""
    qmax = QMAX[bits]
    xs = [frac_of_f32(v) for v in bits_to_f32(xbits)]
    codes, scales = [], []
    for g0 in range(0, len(xs), group):
        grp = xs[g0:g0 + group]
        amax = max(abs(v) for v in grp)
        scale = fl32(amax / qmax)
        scales.append(scale)
        for v in grp:
            if scale == 0:
                codes.append(0)
            else:
                q = rint_even(fl32(v / scale))
                codes.append(max(-qmax, min(qmax, q)))
    return codes, scales


@pytest.mark.parametrize("bits", [8, 4, 2])
@pytest.mark.parametrize("group", [8, 32])
def test_exact_rational_arithmetic(bits, group):
    rng = np.random.default_rng(bits * 100 + group)
    D = 64
    # mix of magnitudes, exact ties (dyadic values) and tiny values
    vals = rng.standard_normal((6, D)).astype(np.float32)
    vals[1] *= 2.0 ** -20
    vals[2] = np.round(vals[2] * 4) / 4          # dyadic: many exact .5 ties
    vals[3, :group] = 0.0                        # an all-zero group
    vals[4] = np.ldexp(np.round(vals[4] * 8), -3 - 60)
    vals[5] *= 1e4
    x = to_bf16_bits(vals).reshape(1, 6, 1, D)
    codes, scales = oracle.quantize(x, bits, group)
    for t in range(6):
        ecodes, escales = _expected_row(x[0, t, 0], bits, group)
        assert [Fraction(float(s)) for s in scales[0, t, 0]] == escales
        assert _unpack(codes[0, t, 0], bits).tolist() == ecodes


@pytest.mark.parametrize("bits,group", [(8, 128), (8, 32), (4, 64), (4, 32), (2, 32), (2, 128)])
def test_invariants_on_generator_data(bits, group):
    K, V = workloads.make_kv(2, 96, 2, 128, seed=3)
    for plane in (K, V):
        x = torch_bits(plane)
        codes, scales = oracle.quantize(x, bits, group)
        q = _unpack(codes, bits).astype(np.float64)
        xf = bits_to_f32(x).astype(np.float64)
        s = np.repeat(scales.astype(np.float64), group, axis=-1)
        qmax = QMAX[bits]
        assert np.all(np.abs(q) <= qmax)
        # |q*scale - x| <= scale/2; the binary32 rounding of the quotient (|x/scale| <= qmax, relative
        # error 2^-24) can move a value across a rounding boundary by at most qmax * 2^-24 code units
        slack = 0.5 + qmax * 2.0 ** -24
        assert np.all(np.abs(q * s - xf) <= s * slack)
        # every non-zero group reaches +-qmax, and scale*qmax reproduces amax to one ulp
        qg = np.abs(q).reshape(*q.shape[:-1], -1, group).max(-1)
        amax = np.abs(xf).reshape(*xf.shape[:-1], -1, group).max(-1)
        assert np.all(qg[amax > 0] == qmax)
        assert np.all(np.abs(scales * qmax - amax) <= amax * 2.0 ** -23)
        # dequantized bf16 stays within scale/2 plus one bf16 rounding
        bt, nb = workloads.make_block_table(x.shape[1], 16, seed=1)
        pool = oracle.dequantize_paged(codes, scales, bits, group, x.shape[1], bt.numpy(), nb, 16)
        y = np.empty_like(x)
        for t in range(x.shape[1]):
            y[:, t] = pool[:, bt[t // 16], t % 16]
        yf = bits_to_f32(y).astype(np.float64)
        assert np.all(np.abs(yf - xf) <= s * slack + np.abs(q * s) * 2.0 ** -8)


def test_special_cases():
    # all-zero group: zero scale, zero codes, dequantizes to +0
    x = _row([0.0] * 32)
    for bits in (8, 4, 2):
        codes, scales = oracle.quantize(x, bits, 32)
        assert not codes.any() and scales.ravel().tolist() == [0.0]
        pool = oracle.dequantize_paged(codes, scales, bits, 32, 1, np.array([0], np.int32), 1, 16)
        assert pool[0, 0, 0, 0].tolist() == [0] * 32
    # constant magnitude: all codes +-qmax, reconstruction exact
    vals = [3.0, -3.0] * 16
    for bits in (8, 4, 2):
        codes, scales = oracle.quantize(_row(vals), bits, 32)
        assert _unpack(codes, bits).ravel().tolist() == [QMAX[bits], -QMAX[bits]] * 16
        pool = oracle.dequantize_paged(codes, scales, bits, 32, 1, np.array([0], np.int32), 1, 16)
        rec = bits_to_f32(pool[0, 0, 0, 0])
        assert np.all(np.abs(rec - np.array(vals)) <= 3.0 * 2.0 ** -8)
    # values already on the grid come back as the same codes (idempotence)
    grid = np.arange(-7, 8, dtype=np.float32)[:8] * 0.5
    grid[0] = -3.5
    codes, scales = oracle.quantize(_row(list(grid) + [3.5] + [0.0] * 7), 4, 16)
    assert scales.ravel()[0] == 0.5
    assert _unpack(codes, 4).ravel()[:9].tolist() == [-7, -6, -5, -4, -3, -2, -1, 0, 7]


def test_size_closed_form():
    # compressed bytes / bf16 bytes = (bits/8 + 4/group) / 2
    x = np.zeros((1, 16, 8, 128), dtype=np.uint16)
    for bits, group, ratio in [(8, 128, 0.515625), (4, 64, 0.28125), (4, 32, 0.3125), (2, 32, 0.1875)]:
        codes, scales = oracle.quantize(x, bits, group)
        assert (codes.nbytes + scales.nbytes) / x.nbytes == ratio


def test_bf16_conversion_matches_library():
    rng = np.random.default_rng(0)
    f = rng.standard_normal(20000).astype(np.float32) * np.float32(2.0) ** rng.integers(-30, 30, 20000)
    # exact ties and near-ties of the bf16 rounding, subnormals, signed zeros
    u = rng.integers(0, 2 ** 32, 5000, dtype=np.uint64).astype(np.uint32)
    u = (u & 0xFFFF0000) | rng.choice(np.array([0x8000, 0x7FFF, 0x8001, 0x0000], dtype=np.uint32), 5000)
    ties = u.view(np.float32)
    ties = ties[np.isfinite(ties)]
    extra = np.array([0.0, -0.0, 1e-40, -1e-40, 3.3895e38, 1.0, -1.0], dtype=np.float32)
    allv = np.concatenate([f, ties, extra])
    want = to_bf16_bits(allv)
    got = np.array([oracle.f32_to_bf16(v) for v in allv], dtype=np.uint16)
    assert np.array_equal(got, want)
    back = np.array([oracle.bf16_to_f32(h) for h in want[:2000]], dtype=np.float32)
    assert np.array_equal(back, bits_to_f32(want[:2000]))


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_dequantize_exact_rational(bits):
    rng = np.random.default_rng(bits)
    D, group = 32, 8
    qmax = QMAX[bits]
    q = rng.integers(-qmax, qmax + 1, (4, D))
    per = 8 // bits
    packed = np.zeros((4, D // per), dtype=np.uint8)
    for i in range(per):
        packed |= ((q[:, i::per] & ((1 << bits) - 1)) << (bits * i)).astype(np.uint8)
    scales = (rng.standard_normal((4, D // group)).astype(np.float32) ** 2 + np.float32(1e-3))
    scales[1] *= np.float32(2.0 ** -100)
    codes4 = packed.reshape(1, 4, 1, -1)
    scales4 = scales.reshape(1, 4, 1, -1)
    bt = np.array([1], np.int32)
    pool = oracle.dequantize_paged(codes4, scales4, bits, group, 4, bt, 2, 16)
    assert np.all(pool[0, 0] == 0x7FC0)                      # the page the table does not name
    assert np.all(pool[0, 1, 4:] == 0x7FC0)                  # page slots beyond T
    for t in range(4):
        for c in range(D):
            want = flbf16(fl32(Fraction(int(q[t, c])) * frac_of_f32(scales[t, c // group])))
            got = Fraction(float(bits_to_f32(pool[0, 1, t, 0, c:c + 1])[0]))
            assert got == want


def test_layouts_gather_padding_paged_source():
    L, T, H, D, bs = 2, 40, 3, 64, 16
    K, _ = workloads.make_kv(L, T, H, D, seed=5)
    x = torch_bits(K)
    codes, scales = oracle.quantize(x, 4, 32, Tp=48)
    assert codes.shape == (L, 48, H, 32) and scales.shape == (L, 48, H, 2)
    assert not codes[:, T:].any() and not scales[:, T:].any()
    # each row is quantized independently: row (l,t,h) equals quantizing that row alone
    one, one_s = oracle.quantize(x[1:2, 7:8, 2:3], 4, 32)
    assert np.array_equal(one[0, 0, 0], codes[1, 7, 2]) and np.array_equal(one_s[0, 0, 0], scales[1, 7, 2])
    # strided view: a head-sliced, token-strided view gives the same rows
    sub = x[:, ::2, 1:3]
    c2, s2 = oracle.quantize(sub, 4, 32)
    assert np.array_equal(c2, codes[:, 0:T:2, 1:3]) and np.array_equal(s2, scales[:, 0:T:2, 1:3])
    # gather: slot i of head h holds token keep_idx[l][h][i]
    rng = np.random.default_rng(1)
    keep = np.stack([[np.sort(rng.choice(T, 10, replace=False)) for _ in range(H)] for _ in range(L)]).astype(np.int32)
    cg, sg = oracle.quantize(x, 4, 32, keep_idx=keep, Tp=16)
    for l in range(L):
        for h in range(H):
            assert np.array_equal(cg[l, :10, h], codes[l, keep[l, h], h])
            assert np.array_equal(sg[l, :10, h], scales[l, keep[l, h], h])
    assert not cg[:, 10:].any() and not sg[:, 10:].any()
    # paged source: scatter the flat plane into pages, read it back through the table
    bt, nb = workloads.make_block_table(T, bs, seed=2, spare=2)
    bt = bt.numpy()
    pool = np.full((L, nb, bs, H, D), 0x7FC0, dtype=np.uint16)
    for t in range(T):
        pool[:, bt[t // bs], t % bs] = x[:, t]
    cp, sp = oracle.quantize_paged_src(pool, bt, T, 4, 32, Tp=48)
    assert np.array_equal(cp, codes) and np.array_equal(sp, scales)
    cpg, spg = oracle.quantize_paged_src(pool, bt, T, 4, 32, keep_idx=keep, Tp=16)
    assert np.array_equal(cpg, cg) and np.array_equal(spg, sg)
    # round trip through the paged destination lands every token where the table says
    out = oracle.dequantize_paged(codes, scales, 4, 32, T, bt, nb, bs)
    flat, flat_s = oracle.quantize(x, 4, 32)
    ref_rows = oracle.dequantize_paged(flat, flat_s, 4, 32, T, np.arange((T + bs - 1) // bs, dtype=np.int32),
                                       (T + bs - 1) // bs, bs).reshape(L, -1, H, D)[:, :T]
    for t in range(T):
        assert np.array_equal(out[:, bt[t // bs], t % bs], ref_rows[:, t])


def test_keep_count():
    assert oracle.keep_count(0.5, 4096) == 2048
    assert oracle.keep_count(0.3, 16384) == 4916
    assert oracle.keep_count(0.1, 131072) == 13108
    assert [oracle.keep_count(r, 8192) for r in (0.25, 0.5, 0.75)] == [2048, 4096, 6144]
    assert oracle.keep_count(0.0, 10) == 1 and oracle.keep_count(1.5, 10) == 10
    assert oracle.keep_count(0.34, 3) == 2          # ceil(1.02)


# ---------------------------------------------------------------- asymmetric variant

@pytest.mark.parametrize("name,bits,xs,scale_bits,expect_bytes,min_bits", _golden_cases(asym=True),
                         ids=lambda c: str(c)[:24])
def test_asym_hand_worked_examples(name, bits, xs, scale_bits, expect_bytes, min_bits):
    codes, scales, mins = oracle.quantize_asym(_row(xs), bits, len(xs))
    assert scales.view(np.uint32).ravel().tolist() == [scale_bits], name
    assert mins.view(np.uint32).ravel().tolist() == [min_bits], name
    assert codes.ravel().tolist() == expect_bytes, name


def _unpack_unsigned(codes, bits):
    per = 8 // bits
    c = codes.astype(np.int32)
    f = np.stack([(c >> (bits * i)) & ((1 << bits) - 1) for i in range(per)], axis=-1)
    return f.reshape(*codes.shape[:-1], codes.shape[-1] * per)


@pytest.mark.parametrize("bits", [8, 4, 2])
def test_asym_exact_rational_arithmetic(bits):
    rng = np.random.default_rng(bits + 50)
    D, group, levels = 64, 16, (1 << bits) - 1
    vals = rng.standard_normal((5, D)).astype(np.float32)
    vals[1] = np.round(vals[1] * 4) / 4
    vals[2, :group] = 1.5                                  # constant group: scale 0
    vals[3] *= 1e3
    vals[4] = np.abs(vals[4]) * 2.0 ** -30
    x = to_bf16_bits(vals).reshape(1, 5, 1, D)
    codes, scales, mins = oracle.quantize_asym(x, bits, group)
    pool = oracle.dequantize_paged_asym(codes, scales, mins, bits, group, 5, np.array([0], np.int32), 1, 16)
    for t in range(5):
        xs = [frac_of_f32(v) for v in bits_to_f32(x[0, t, 0])]
        q = _unpack_unsigned(codes[0, t, 0], bits)
        for g in range(D // group):
            grp = xs[g * group:(g + 1) * group]
            mn, mx = min(grp), max(grp)
            scale = fl32(fl32(mx - mn) / levels)
            assert Fraction(float(scales[0, t, 0, g])) == scale and Fraction(float(mins[0, t, 0, g])) == mn
            for c, v in enumerate(grp):
                want = 0 if scale == 0 else max(0, min(levels, rint_even(fl32(fl32(v - mn) / scale))))
                assert q[g * group + c] == want
                back = flbf16(fl32(fl32(Fraction(int(want)) * scale) + mn))
                assert Fraction(float(bits_to_f32(pool[0, 0, t, 0, g * group + c:g * group + c + 1])[0])) == back


@pytest.mark.parametrize("bits,group", [(8, 128), (4, 32), (2, 32), (2, 128)])
def test_asym_invariants_and_gain_over_symmetric(bits, group):
    _, V = workloads.make_kv(2, 64, 2, 128, seed=9)       # V: no outlier channels (a one-sided outlier can
    x = torch_bits(V)                                     # make the 4-level asymmetric grid coarser near 0)
    xf = bits_to_f32(x).astype(np.float64)
    codes, scales, mins = oracle.quantize_asym(x, bits, group)
    levels = (1 << bits) - 1
    q = _unpack_unsigned(codes, bits).astype(np.float64)
    s = np.repeat(scales.astype(np.float64), group, -1)
    m = np.repeat(mins.astype(np.float64), group, -1)
    assert q.min() >= 0 and q.max() <= levels
    # |q*scale + min - x| <= scale/2 plus the binary32 roundings of the difference and the quotient
    assert np.all(np.abs(q * s + m - xf) <= s * (0.5 + levels * 2.0 ** -23) + np.abs(xf - m) * 2.0 ** -23)
    # the group minimum maps to code 0 and the maximum to the top level
    qg = q.reshape(*q.shape[:-1], -1, group)
    assert np.all(qg.min(-1) == 0) and np.all(qg.max(-1)[scales > 0] == levels)
    # using every level, the reconstruction error is smaller than the symmetric quantizer's
    bt = np.arange(4, dtype=np.int32)
    ya = bits_to_f32(oracle.dequantize_paged_asym(codes, scales, mins, bits, group, 64, bt, 4, 16).reshape(2, 64, 2, 128))
    cs, ss = oracle.quantize(x, bits, group)
    ys = bits_to_f32(oracle.dequantize_paged(cs, ss, bits, group, 64, bt, 4, 16).reshape(2, 64, 2, 128))
    assert np.square(ya - xf).sum() < np.square(ys - xf).sum()


@pytest.mark.parametrize("bits,group", [(8, 128), (4, 64), (4, 32), (2, 32)])
def test_numpy_float32_cross_check(bits, group):
    # the same arithmetic with a library's IEEE binary32 division and round-half-even, symmetric and asymmetric
    K, _ = workloads.make_kv(2, 64, 2, 128, seed=bits + group)
    xb = torch_bits(K)
    x = bits_to_f32(xb).reshape(-1, 128 // group, group)
    qmax = np.float32((1 << (bits - 1)) - 1)
    amax = np.abs(x).max(-1, keepdims=True)
    scale = (amax / qmax).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.where(scale > 0, np.rint((x / scale).astype(np.float32)), 0).astype(np.int32)
    codes, scales = oracle.quantize(xb, bits, group)
    assert np.array_equal(scales.reshape(-1, 128 // group), scale[..., 0])
    assert np.array_equal(_unpack(codes, bits).reshape(x.shape), q)
    levels = np.float32((1 << bits) - 1)
    mn, mx = x.min(-1, keepdims=True), x.max(-1, keepdims=True)
    sc = ((mx - mn).astype(np.float32) / levels).astype(np.float32)
    with np.errstate(divide="ignore", invalid="ignore"):
        qa = np.where(sc > 0, np.rint(((x - mn).astype(np.float32) / sc).astype(np.float32)), 0).astype(np.int32)
    ca, sa, ma = oracle.quantize_asym(xb, bits, group)
    assert np.array_equal(sa.reshape(-1, 128 // group), sc[..., 0])
    assert np.array_equal(ma.reshape(-1, 128 // group), mn[..., 0])
    assert np.array_equal(_unpack_unsigned(ca, bits).reshape(x.shape), qa)
