"""ctypes front end of the CPU oracle (oracle/kvp_oracle.cpp).

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's
cpu_baseline leg may import this; the product package never does.  It imports
nothing from the HIP package.  Arrays are numpy; bf16 tensors travel as uint16
arrays holding the raw bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvp_oracle.cpp")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_i64 = ctypes.c_int64
_i32 = ctypes.c_int32
_p = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the oracle with the host compiler; returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["g++", "-O2", "-std=c++17", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
               "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_keep_count.restype = _i64
        _lib.oracle_keep_count.argtypes = [ctypes.c_double, _i64]
        _lib.oracle_f32_to_bf16.restype = ctypes.c_uint16
        _lib.oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        _lib.oracle_bf16_to_f32.restype = ctypes.c_float
        _lib.oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        _lib.oracle_quantize.restype = ctypes.c_int
        _lib.oracle_quantize.argtypes = [_p, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _p, _i64,
                                         ctypes.c_int, ctypes.c_int, _i64, _p, _p]
        _lib.oracle_quantize_paged_src.restype = ctypes.c_int
        _lib.oracle_quantize_paged_src.argtypes = [_p, _p, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _p, _i64,
                                                   ctypes.c_int, ctypes.c_int, _i64, _p, _p]
        _lib.oracle_dequantize_paged.restype = ctypes.c_int
        _lib.oracle_dequantize_paged.argtypes = [_p, _p, ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _i64,
                                                 _i64, _p, _i64, _i64, _p, _i64]
        _lib.oracle_quantize_asym.restype = ctypes.c_int
        _lib.oracle_quantize_asym.argtypes = [_p, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _p, _i64,
                                              ctypes.c_int, ctypes.c_int, _i64, _p, _p, _p]
        _lib.oracle_dequantize_paged_asym.restype = ctypes.c_int
        _lib.oracle_dequantize_paged_asym.argtypes = [_p, _p, _p, ctypes.c_int, ctypes.c_int, _i64, _i64, _i64, _i64,
                                                      _i64, _p, _i64, _i64, _p, _i64]
        _lib.oracle_quantize_channel.restype = ctypes.c_int
        _lib.oracle_quantize_channel.argtypes = [_p, _i64, _i64, _i64, _i64, _i64, _i64, _i64, _p, _i64,
                                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, _i64, _p, _p, _p]
        _lib.oracle_dequantize_paged_channel.restype = ctypes.c_int
        _lib.oracle_dequantize_paged_channel.argtypes = [_p, _p, _p, ctypes.c_int, ctypes.c_int, ctypes.c_int, _i64, _i64,
                                                         _i64, _i64, _i64, _p, _i64, _i64, _p, _i64]
        _lib.oracle_dequantize_paged_scatter.restype = ctypes.c_int
        _lib.oracle_dequantize_paged_scatter.argtypes = [_p, _p, _p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                         _i64, _i64, _i64, _i64, _i64, _p, _i64, _p, _i64, _i64, _p, _i64]
        _lib.oracle_smooth_scores.restype = ctypes.c_int
        _lib.oracle_smooth_scores.argtypes = [_p, _i64, _i64, _i64, _i64, ctypes.c_int, ctypes.c_int, _p, _i64]
        _lib.oracle_score_tokens.restype = ctypes.c_int
        _lib.oracle_score_tokens.argtypes = [_p, _i64, _i64, _i64, _i64, _i64, _p, _i64, _i64, _i64, _i64,
                                             _i64, _i64, _i64, ctypes.c_int, ctypes.c_int, _p]
        _lib.oracle_score_keys.restype = ctypes.c_int
        _lib.oracle_score_keys.argtypes = [_p, _i64, _i64, _i64, _i64, _i64, _i64, _i64, ctypes.c_int, _p, _i64, _p]
        _lib.oracle_select_topk.restype = ctypes.c_int
        _lib.oracle_select_topk.argtypes = [_p, _i64, _i64, _i64, _i64, _p]
        _lib.oracle_eval_configs.restype = ctypes.c_int
        _lib.oracle_eval_configs.argtypes = [_p, _i64, _i64, _i64, _i64, _i64,
                                             _p, _i64, _i64, _i64,
                                             _p, _i64, _i64, _i64,
                                             _i64, _i64, _i64, _i64,
                                             _p, _p, _p, _i32, _p, _p]
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(_p)


def _view4(a: np.ndarray):
    """(array, stride_l, stride_t, stride_h) in elements of a [L][T][H][D] uint16 array."""
    assert a.dtype == np.uint16 and a.ndim == 4
    isz = a.itemsize
    assert a.strides[3] == isz, "innermost dimension must be contiguous"
    assert all(s % isz == 0 and s >= 0 for s in a.strides)
    return a, a.strides[0] // isz, a.strides[1] // isz, a.strides[2] // isz


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: bad argument (rc={rc})")


def keep_count(ratio: float, T: int) -> int:
    return int(lib().oracle_keep_count(float(ratio), int(T)))


def f32_to_bf16(x: float) -> int:
    return int(lib().oracle_f32_to_bf16(float(x)))


def bf16_to_f32(h: int) -> float:
    return float(lib().oracle_bf16_to_f32(int(h)))


def round_up(n: int, m: int) -> int:
    return (n + m - 1) // m * m


def quantize(x: np.ndarray, bits: int, group: int, keep_idx: np.ndarray | None = None, Tp: int | None = None):
    """x: uint16 [L][T][H][D] -> (codes u8 [L][Tp][H][D*bits/8], scales f32 [L][Tp][H][D/group])."""
    x, sl, st, sh = _view4(x)
    L, T, H, D = x.shape
    k = 0
    if keep_idx is not None:
        keep_idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
        assert keep_idx.shape[:2] == (L, H)
        k = keep_idx.shape[2]
    n_slots = k if keep_idx is not None else T
    if Tp is None:
        Tp = n_slots
    codes = np.full((L, Tp, H, D * bits // 8), 0xAB, dtype=np.uint8)
    scales = np.full((L, Tp, H, D // group), np.nan, dtype=np.float32)
    _check(lib().oracle_quantize(_ptr(x), L, T, H, D, sl, st, sh, _ptr(keep_idx), k, bits, group, Tp,
                                 _ptr(codes), _ptr(scales)), "quantize")
    return codes, scales


def quantize_paged_src(pool: np.ndarray, block_table: np.ndarray, T: int, bits: int, group: int,
                       keep_idx: np.ndarray | None = None, Tp: int | None = None):
    """pool: uint16 [L][num_blocks][bs][H][D] (C-contiguous per layer)."""
    assert pool.dtype == np.uint16 and pool.ndim == 5
    L, NB, bs, H, D = pool.shape
    assert pool[0].flags["C_CONTIGUOUS"]
    stride_l = pool.strides[0] // 2
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    k = 0
    if keep_idx is not None:
        keep_idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
        k = keep_idx.shape[2]
    n_slots = k if keep_idx is not None else T
    if Tp is None:
        Tp = n_slots
    codes = np.full((L, Tp, H, D * bits // 8), 0xAB, dtype=np.uint8)
    scales = np.full((L, Tp, H, D // group), np.nan, dtype=np.float32)
    _check(lib().oracle_quantize_paged_src(_ptr(pool), _ptr(block_table), L, NB, bs, H, D, T, stride_l,
                                           _ptr(keep_idx), k, bits, group, Tp, _ptr(codes), _ptr(scales)),
           "quantize_paged_src")
    return codes, scales


def dequantize_paged(codes: np.ndarray, scales: np.ndarray, bits: int, group: int, T: int,
                     block_table: np.ndarray, num_blocks: int, bs: int, pool: np.ndarray | None = None,
                     fill: int = 0x7FC0):
    """Returns the paged pool uint16 [L][num_blocks][bs][H][D]; untouched slots keep `fill` (a bf16 NaN)."""
    codes = np.ascontiguousarray(codes)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    L, Tp, H, cb = codes.shape
    D = cb * 8 // bits
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    if pool is None:
        pool = np.full((L, num_blocks, bs, H, D), fill, dtype=np.uint16)
    assert pool.flags["C_CONTIGUOUS"] and pool.shape == (L, num_blocks, bs, H, D)
    _check(lib().oracle_dequantize_paged(_ptr(codes), _ptr(scales), bits, group, L, T, Tp, H, D,
                                         _ptr(block_table), num_blocks, bs, _ptr(pool), num_blocks * bs * H * D),
           "dequantize_paged")
    return pool


def quantize_asym(x: np.ndarray, bits: int, group: int, keep_idx: np.ndarray | None = None, Tp: int | None = None):
    """Asymmetric variant -> (codes u8, scales f32, mins f32), layouts as quantize()."""
    x, sl, st, sh = _view4(x)
    L, T, H, D = x.shape
    k = 0
    if keep_idx is not None:
        keep_idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
        k = keep_idx.shape[2]
    n_slots = k if keep_idx is not None else T
    if Tp is None:
        Tp = n_slots
    codes = np.full((L, Tp, H, D * bits // 8), 0xAB, dtype=np.uint8)
    scales = np.full((L, Tp, H, D // group), np.nan, dtype=np.float32)
    mins = np.full((L, Tp, H, D // group), np.nan, dtype=np.float32)
    _check(lib().oracle_quantize_asym(_ptr(x), L, T, H, D, sl, st, sh, _ptr(keep_idx), k, bits, group, Tp,
                                      _ptr(codes), _ptr(scales), _ptr(mins)), "quantize_asym")
    return codes, scales, mins


def dequantize_paged_asym(codes, scales, mins, bits: int, group: int, T: int, block_table, num_blocks: int, bs: int,
                          pool: np.ndarray | None = None, fill: int = 0x7FC0):
    codes = np.ascontiguousarray(codes)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    mins = np.ascontiguousarray(mins, dtype=np.float32)
    L, Tp, H, cb = codes.shape
    D = cb * 8 // bits
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    if pool is None:
        pool = np.full((L, num_blocks, bs, H, D), fill, dtype=np.uint16)
    _check(lib().oracle_dequantize_paged_asym(_ptr(codes), _ptr(scales), _ptr(mins), bits, group, L, T, Tp, H, D,
                                              _ptr(block_table), num_blocks, bs, _ptr(pool), num_blocks * bs * H * D),
           "dequantize_paged_asym")
    return pool


def quantize_channel(x: np.ndarray, bits: int, group: int, keep_idx: np.ndarray | None = None, Tp: int | None = None,
                     asym: bool = False):
    """Per-channel grouping (groups of `group` token slots per channel) -> (codes u8 [L][Tp][H][D*bits/8],
    scales f32 [L][ceil(Tp/group)][H][D], mins likewise or None)."""
    x, sl, st, sh = _view4(x)
    L, T, H, D = x.shape
    k = 0
    if keep_idx is not None:
        keep_idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
        k = keep_idx.shape[2]
    n_slots = k if keep_idx is not None else T
    if Tp is None:
        Tp = n_slots
    ng = (Tp + group - 1) // group
    codes = np.full((L, Tp, H, D * bits // 8), 0xAB, dtype=np.uint8)
    scales = np.full((L, ng, H, D), np.nan, dtype=np.float32)
    mins = np.full((L, ng, H, D), np.nan, dtype=np.float32) if asym else None
    _check(lib().oracle_quantize_channel(_ptr(x), L, T, H, D, sl, st, sh, _ptr(keep_idx), k, bits, group, int(asym), Tp,
                                         _ptr(codes), _ptr(scales), _ptr(mins)), "quantize_channel")
    return codes, scales, mins


def dequantize_paged_channel(codes, scales, mins, bits: int, group: int, T: int, block_table, num_blocks: int, bs: int,
                             pool: np.ndarray | None = None, fill: int = 0x7FC0):
    codes = np.ascontiguousarray(codes)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    if mins is not None:
        mins = np.ascontiguousarray(mins, dtype=np.float32)
    L, Tp, H, cb = codes.shape
    D = cb * 8 // bits
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    if pool is None:
        pool = np.full((L, num_blocks, bs, H, D), fill, dtype=np.uint16)
    _check(lib().oracle_dequantize_paged_channel(_ptr(codes), _ptr(scales), _ptr(mins), bits, group, int(mins is not None),
                                                 L, T, Tp, H, D, _ptr(block_table), num_blocks, bs, _ptr(pool),
                                                 num_blocks * bs * H * D), "dequantize_paged_channel")
    return pool


def score_tokens(q: np.ndarray, k: np.ndarray, causal: bool = True, force_window: bool = True) -> np.ndarray:
    """q: uint16 [L][W][Hq][D], k: uint16 [L][T][Hkv][D] -> scores f32 [L][Hkv][T]."""
    q, qsl, qst, qsh = _view4(q)
    k, ksl, kst, ksh = _view4(k)
    L, W, Hq, D = q.shape
    L2, T, Hkv, D2 = k.shape
    assert L == L2 and D == D2
    scores = np.empty((L, Hkv, T), dtype=np.float32)
    _check(lib().oracle_score_tokens(_ptr(q), W, Hq, qsl, qst, qsh, _ptr(k), L, T, Hkv, D, ksl, kst, ksh,
                                     int(causal), int(force_window), _ptr(scores)), "score_tokens")
    return scores


KNORM, KEYDIFF = 0, 1


def score_keys(k: np.ndarray, method: int, tokens: np.ndarray | None = None) -> np.ndarray:
    """k: uint16 [L][T][H][D] -> key-only importance f32 [L][H][T] (or [L][H][n] for the listed tokens)."""
    k, ksl, kst, ksh = _view4(k)
    L, T, H, D = k.shape
    n = 0
    if tokens is not None:
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        n = len(tokens)
    out = np.empty((L, H, n if tokens is not None else T), dtype=np.float32)
    _check(lib().oracle_score_keys(_ptr(k), L, T, H, D, ksl, kst, ksh, int(method), _ptr(tokens), n, _ptr(out)),
           "score_keys")
    return out


def dequantize_paged_scatter(codes, scales, mins, bits: int, group: int, keep_idx, T: int, block_table,
                             num_blocks: int, bs: int, pool: np.ndarray | None = None, fill: int = 0x7FC0,
                             per_channel: bool = False):
    """Restore the k slots of a dropped+quantized plane at their original token positions of a T-token pool."""
    codes = np.ascontiguousarray(codes)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    if mins is not None:
        mins = np.ascontiguousarray(mins, dtype=np.float32)
    keep_idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
    L, Tp, H, cb = codes.shape
    D = cb * 8 // bits
    k = keep_idx.shape[2]
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    if pool is None:
        pool = np.full((L, num_blocks, bs, H, D), fill, dtype=np.uint16)
    _check(lib().oracle_dequantize_paged_scatter(_ptr(codes), _ptr(scales), _ptr(mins), bits, group, int(mins is not None),
                                                 int(per_channel), L, k, Tp, H, D, _ptr(keep_idx), T, _ptr(block_table),
                                                 num_blocks, bs, _ptr(pool), num_blocks * bs * H * D),
           "dequantize_paged_scatter")
    return pool


def smooth_scores(scores: np.ndarray, window: int, kernel: int, mode: str = "avg") -> np.ndarray:
    """1-D pooling of the prefix scores along tokens (window positions copied): f32 [n_rows][T] -> same."""
    assert scores.dtype == np.float32 and scores.ndim == 2 and scores.strides[1] == 4
    n_rows, T = scores.shape
    row_stride = scores.strides[0] // 4 if n_rows > 1 else T
    out = np.full((n_rows, T), np.nan, dtype=np.float32)
    _check(lib().oracle_smooth_scores(_ptr(scores), n_rows, T, row_stride, window, kernel,
                                      {"avg": 0, "max": 1}[mode], _ptr(out), T), "smooth_scores")
    return out


def select_topk(scores: np.ndarray, k: int) -> np.ndarray:
    """scores: f32 [n_rows][T] (rows may be strided) -> int32 [n_rows][k], ascending."""
    assert scores.dtype == np.float32 and scores.ndim == 2 and scores.strides[1] == 4
    n_rows, T = scores.shape
    row_stride = scores.strides[0] // 4 if n_rows > 1 else T
    out = np.full((n_rows, k), -1, dtype=np.int32)
    _check(lib().oracle_select_topk(_ptr(scores), n_rows, T, row_stride, k, _ptr(out)), "select_topk")
    return out


def eval_configs(q: np.ndarray, k: np.ndarray, v: np.ndarray, cfgs):
    """cfgs: iterable of (bits, group, keep_k).  Returns (loss f32 [n], partial f64 [L][n][2])."""
    q, qsl, qst, qsh = _view4(q)
    k, ksl, kst, ksh = _view4(k)
    v, vsl, vst, vsh = _view4(v)
    L, W, Hq, D = q.shape
    _, T, Hkv, _ = k.shape
    assert v.shape == k.shape
    cfgs = list(cfgs)
    n = len(cfgs)
    bits = np.array([c[0] for c in cfgs], dtype=np.int32)
    group = np.array([c[1] for c in cfgs], dtype=np.int32)
    keep = np.array([c[2] for c in cfgs], dtype=np.int64)
    loss = np.empty(n, dtype=np.float32)
    partial = np.empty((L, n, 2), dtype=np.float64)
    _check(lib().oracle_eval_configs(_ptr(q), W, Hq, qsl, qst, qsh, _ptr(k), ksl, kst, ksh,
                                     _ptr(v), vsl, vst, vsh, L, T, Hkv, D,
                                     _ptr(bits), _ptr(group), _ptr(keep), n, _ptr(loss), _ptr(partial)),
           "eval_configs")
    return loss, partial
