"""ctypes binding of libkvp.so: the same entry points as include/kvp.h, taking torch tensors.

Argument marshalling only.  torch supplies device memory and the current HIP stream; every
kernel launch happens inside the C library.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Iterable, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libkvp.so")

_i32, _i64, _vp, _sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t


class KVPError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {kvp_strerror(code)} ({code})")


class _View(ctypes.Structure):
    _fields_ = [("ptr", _vp), ("L", _i64), ("T", _i64), ("H", _i64), ("D", _i64),
                ("stride_l", _i64), ("stride_t", _i64), ("stride_h", _i64)]


class _Paged(ctypes.Structure):
    _fields_ = [("pool", _vp), ("block_table", _vp), ("L", _i64), ("num_blocks", _i64), ("bs", _i64),
                ("H", _i64), ("D", _i64), ("T", _i64), ("stride_l", _i64)]


class _QPlane(ctypes.Structure):
    _fields_ = [("codes", _vp), ("scales", _vp), ("mins", _vp), ("bits", _i32), ("group", _i32),
                ("L", _i64), ("T", _i64), ("Tp", _i64), ("H", _i64), ("D", _i64), ("group_axis", _i32)]


class _Tier(ctypes.Structure):
    _fields_ = [("capacity_bytes", ctypes.c_double), ("bandwidth_bytes_per_s", ctypes.c_double)]


class _PolicyOp(ctypes.Structure):
    _fields_ = [("ctx", _i32), ("cfg", _i32), ("tier", _i32), ("op", _i32)]


class _Dims(ctypes.Structure):
    _fields_ = [("L", _i64), ("Hkv", _i64), ("Hq", _i64), ("W", _i64), ("T", _i64), ("n_rows", _i64), ("k", _i64),
                ("n_cfgs", _i32), ("method", _i32)]


class _Config(ctypes.Structure):
    _fields_ = [("bits", _i32), ("group", _i32), ("keep_k", _i64)]


def library_path() -> str:
    return _LIB_PATH


def _load(path: str = _LIB_PATH):
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is not built; run `python -m paper_2512_14946_amd.build` "
            "(there is no CPU fallback for the kvp_* operations)")
    lib = ctypes.CDLL(path)
    P = ctypes.POINTER
    lib.kvp_quantize.restype = _i32
    lib.kvp_quantize.argtypes = [P(_View), P(_Paged), _vp, _i64, P(_QPlane), _vp]
    lib.kvp_dequantize_paged.restype = _i32
    lib.kvp_dequantize_paged.argtypes = [P(_QPlane), P(_Paged), _vp]
    lib.kvp_dequantize_paged_scatter.restype = _i32
    lib.kvp_dequantize_paged_scatter.argtypes = [P(_QPlane), _vp, P(_Paged), _vp]
    lib.kvp_score_tokens.restype = _i32
    lib.kvp_score_tokens.argtypes = [P(_View), P(_View), _i32, _i32, _vp, _vp, _sz, _vp]
    lib.kvp_score_tokens_static.restype = _i32
    lib.kvp_score_tokens_static.argtypes = [P(_View), P(_View), _i32, _i32, _vp, _vp]
    lib.kvp_score_workspace_bytes.restype = _sz
    lib.kvp_score_workspace_bytes.argtypes = [_i64] * 5
    lib.kvp_score_keys.restype = _i32
    lib.kvp_score_keys.argtypes = [P(_View), _i32, _vp, _vp, _sz, _vp]
    lib.kvp_score_keys_workspace_bytes.restype = _sz
    lib.kvp_score_keys_workspace_bytes.argtypes = [_i64, _i64, _i64, _i32]
    lib.kvp_smooth_scores.restype = _i32
    lib.kvp_smooth_scores.argtypes = [_vp, _i64, _i64, _i64, _i64, _i32, _i32, _vp, _i64, _vp]
    lib.kvp_select_topk.restype = _i32
    lib.kvp_select_topk.argtypes = [_vp, _i64, _i64, _i64, _i64, _vp, _vp, _sz, _vp]
    lib.kvp_select_workspace_bytes.restype = _sz
    lib.kvp_select_workspace_bytes.argtypes = [_i64] * 3
    lib.kvp_eval_configs.restype = _i32
    lib.kvp_eval_configs.argtypes = [P(_View), P(_View), P(_View), P(_Config), _i32, _vp, _vp, _vp, _sz, _vp]
    lib.kvp_eval_configs_ex.restype = _i32
    lib.kvp_eval_configs_ex.argtypes = [P(_View), P(_View), P(_View), P(_Config), _i32, _vp, _vp, _vp, _sz,
                                        ctypes.c_uint32, _vp]
    lib.kvp_eval_workspace_bytes.restype = _sz
    lib.kvp_eval_workspace_bytes.argtypes = [_i64] * 5 + [_i32]
    lib.kvp_utility_table.restype = _i32
    lib.kvp_utility_table.argtypes = [_vp, _vp, _i32, P(_Tier), _i32, ctypes.c_double, ctypes.c_double, _vp]
    lib.kvp_policy_insert.restype = _i32
    lib.kvp_policy_insert.argtypes = [_i32, _i32, _vp, _vp, _vp, P(_Tier), _i32, ctypes.c_double, _vp, _vp, _i32,
                                      P(_PolicyOp), _i32, P(_i32)]
    lib.kvp_workspace_bytes.restype = _sz
    lib.kvp_workspace_bytes.argtypes = [_i32, P(_Dims)]
    lib.kvp_keep_count.restype = _i64
    lib.kvp_keep_count.argtypes = [ctypes.c_double, _i64]
    lib.kvp_copy_bytes.restype = _i32
    lib.kvp_copy_bytes.argtypes = [_vp, _vp, _sz, _vp]
    lib.kvp_strerror.restype = ctypes.c_char_p
    lib.kvp_strerror.argtypes = [_i32]
    lib.kvp_selftest_reciprocal.restype = _i32
    lib.kvp_selftest_reciprocal.argtypes = [_vp, _vp]
    lib.kvp_version.restype = ctypes.c_uint32
    lib.kvp_version.argtypes = []
    return lib


_lib = _load()


# ------------------------------------------------------------------ containers

@dataclass
class QPlane:
    """Compressed plane: codes u8 [L][Tp][H][D*bits/8], scales f32 [L][Tp][H][D/group]
    (group_axis 0: groups of channels) or [L][ceil(Tp/group)][H][D] (group_axis 1: groups of token slots)."""
    codes: torch.Tensor
    scales: torch.Tensor
    bits: int
    group: int
    T: int
    mins: torch.Tensor | None = None   # set: asymmetric codec (unsigned codes, per-group minimum)
    group_axis: int = 0                # KVP_GROUP_CHANNELS = 0, KVP_GROUP_TOKENS = 1

    @property
    def Tp(self) -> int:
        return self.codes.shape[1]

    def nbytes(self) -> int:
        return self.codes.numel() + 4 * self.scales.numel() + (4 * self.mins.numel() if self.mins is not None else 0)


@dataclass
class PagedKV:
    """Paged bf16 plane: pool [L][num_blocks][bs][H][D], block_table int32 [ceil(T/bs)]."""
    pool: torch.Tensor
    block_table: torch.Tensor
    T: int


def alloc_qplane(L: int, T: int, H: int, D: int, bits: int, group: int, device, page: int = 16,
                 asymmetric: bool = False, per_channel: bool = False) -> QPlane:
    Tp = (T + page - 1) // page * page
    codes = torch.empty(L, Tp, H, D * bits // 8, dtype=torch.uint8, device=device)
    sshape = (L, (Tp + group - 1) // group, H, D) if per_channel else (L, Tp, H, D // group)
    scales = torch.empty(sshape, dtype=torch.float32, device=device)
    mins = torch.empty(sshape, dtype=torch.float32, device=device) if asymmetric else None
    return QPlane(codes, scales, bits, group, T, mins, int(per_channel))


def alloc_paged(L: int, T: int, H: int, D: int, block_table: torch.Tensor, num_blocks: int, bs: int = 16,
                fill_nan: bool = False) -> PagedKV:
    dev = block_table.device
    if fill_nan:
        pool = torch.full((L, num_blocks, bs, H, D), float("nan"), dtype=torch.bfloat16, device=dev)
    else:
        pool = torch.empty(L, num_blocks, bs, H, D, dtype=torch.bfloat16, device=dev)
    return PagedKV(pool, block_table, T)


# ------------------------------------------------------------------ marshalling

# Marshalled structs are cached: a tensor keeps the struct built from it (keyed by its data pointer and element
# count), a QPlane / PagedKV keeps its struct as long as it refers to the same tensor objects and sizes.  A call on
# operands seen before then costs a few attribute reads instead of a dozen shape / stride / dtype queries, which is
# most of the host time of a small, launch-bound call.

_raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream(stream, like: torch.Tensor | None = None) -> int:
    if stream is None:
        if _raw_stream is not None and like is not None:
            return _raw_stream(like.get_device())
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _need_cuda(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("kvp_* operations run on the GPU only: tensors must live on a cuda device")


def _view(t: torch.Tensor) -> _View:
    # the marshalled struct is cached on the tensor, keyed by everything it is made of (an in-place
    # transpose_ / as_strided_ / set_ changes shape or strides under the same storage pointer)
    c = getattr(t, "_kvp_view", None)
    if c is not None and c[0] == t.data_ptr() and c[1] == t.shape and c[2] == t.stride():
        return c[3]
    if t.dtype != torch.bfloat16 or t.dim() != 4:
        raise ValueError("expected a bf16 tensor [L][T][H][D]")
    if t.stride(3) != 1:
        raise ValueError("innermost dimension must be contiguous")
    L, T, H, D = t.shape
    v = _View(t.data_ptr(), L, T, H, D, t.stride(0), t.stride(1), t.stride(2))
    try:
        t._kvp_view = (t.data_ptr(), t.shape, t.stride(), v)
    except Exception:   # a tensor type that takes no attributes
        pass
    return v


def _paged(p: PagedKV) -> _Paged:
    c = p.__dict__.get("_c")
    if (c is not None and c[0] is p.pool and c[1] is p.block_table and c[2] == p.T and c[3] == p.pool.data_ptr()
            and c[4] == p.pool.shape and c[5] == p.pool.stride() and c[6] == p.block_table.data_ptr()
            and c[7] == p.block_table.shape):
        return c[8]
    pool = p.pool
    if pool.dtype != torch.bfloat16 or pool.dim() != 5 or not pool[0].is_contiguous():
        raise ValueError("pool must be bf16 [L][num_blocks][bs][H][D], contiguous per layer")
    if p.block_table.dtype != torch.int32 or not p.block_table.is_contiguous():
        raise ValueError("block_table must be contiguous int32")
    L, NB, bs, H, D = pool.shape
    if p.block_table.numel() < (p.T + bs - 1) // bs:
        raise ValueError("block_table is shorter than ceil(T / bs)")
    _need_cuda(pool, p.block_table)
    v = _Paged(pool.data_ptr(), p.block_table.data_ptr(), L, NB, bs, H, D, p.T, pool.stride(0))
    p.__dict__["_c"] = (p.pool, p.block_table, p.T, pool.data_ptr(), pool.shape, pool.stride(), p.block_table.data_ptr(),
                        p.block_table.shape, v)
    return v


def _qplane(q: QPlane) -> _QPlane:
    c = q.__dict__.get("_c")
    if (c is not None and c[0] is q.codes and c[1] is q.scales and c[2] is q.mins and c[3] == q.T and c[4] == q.bits
            and c[5] == q.group and c[6] == q.group_axis and c[7] == q.codes.data_ptr() and c[8] == q.codes.shape
            and c[9] == q.scales.data_ptr() and c[10] == q.scales.shape
            and (q.mins is None or (c[11] == q.mins.data_ptr() and c[12] == q.mins.shape))):
        return c[13]
    if q.codes.dtype != torch.uint8 or q.scales.dtype != torch.float32:
        raise ValueError("codes must be uint8 and scales float32")
    if not (q.codes.is_contiguous() and q.scales.is_contiguous()):
        raise ValueError("codes and scales must be contiguous")
    L, Tp, H, cb = q.codes.shape
    D = cb * 8 // q.bits
    want = (L, (Tp + q.group - 1) // q.group, H, D) if q.group_axis == 1 else (L, Tp, H, D // q.group)
    if tuple(q.scales.shape) != want:
        raise ValueError("scales shape does not match codes")
    mins = None
    if q.mins is not None:
        if q.mins.dtype != torch.float32 or not q.mins.is_contiguous() or tuple(q.mins.shape) != tuple(q.scales.shape):
            raise ValueError("mins must be contiguous float32 with the shape of scales")
        mins = q.mins.data_ptr()
    _need_cuda(q.codes, q.scales, q.mins)
    v = _QPlane(q.codes.data_ptr(), q.scales.data_ptr(), mins, q.bits, q.group, L, q.T, Tp, H, D, q.group_axis)
    q.__dict__["_c"] = (q.codes, q.scales, q.mins, q.T, q.bits, q.group, q.group_axis, q.codes.data_ptr(), q.codes.shape,
                        q.scales.data_ptr(), q.scales.shape, mins, None if q.mins is None else q.mins.shape, v)
    return v


def _check(rc: int, what: str):
    if rc != 0:
        raise KVPError(rc, what)


def _workspace(ws, nbytes: int, device, stream=None):
    """(tensor kept alive by the caller, pointer, bytes).  A workspace allocated here is a temporary: when the
    call runs on a stream other than torch's current one, the allocator is told so that it does not hand the
    memory out again while the kernels still use it."""
    if ws is None:
        if nbytes == 0:
            return None, None, 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
        if stream is not None:
            s = stream if isinstance(stream, torch.cuda.Stream) else torch.cuda.ExternalStream(int(stream))
            if s != torch.cuda.current_stream(device):
                ws.record_stream(s)
    return ws, ws.data_ptr(), ws.numel() * ws.element_size()


# ------------------------------------------------------------------ entry points

def kvp_strerror(code: int) -> str:
    return _lib.kvp_strerror(int(code)).decode()


def kvp_selftest_reciprocal(stream=None) -> int:
    """Operands (of 2^23 x 121) for which the corrected hardware reciprocal differs from the IEEE quotient."""
    out = torch.zeros(1, dtype=torch.int64, device="cuda")
    _check(_lib.kvp_selftest_reciprocal(out.data_ptr(), _stream(stream)), "kvp_selftest_reciprocal")
    return int(out.item())


def kvp_version() -> int:
    return int(_lib.kvp_version())


KVP_WS_SCORE_TOKENS, KVP_WS_SCORE_KEYS, KVP_WS_SELECT_TOPK, KVP_WS_EVAL_CONFIGS = 0, 1, 2, 3


def kvp_workspace_bytes(op: int, L: int = 0, Hkv: int = 0, Hq: int = 0, W: int = 0, T: int = 0, n_rows: int = 0,
                        k: int = 0, n_cfgs: int = 0, method: int = 0) -> int:
    """Scratch bytes of one call of entry point `op` (KVP_WS_*) for these sizes."""
    d = _Dims(L, Hkv, Hq, W, T, n_rows, k, n_cfgs, method)
    return int(_lib.kvp_workspace_bytes(int(op), ctypes.byref(d)))


def kvp_keep_count(ratio: float, T: int) -> int:
    return int(_lib.kvp_keep_count(float(ratio), int(T)))


def kvp_quantize(src, dst: QPlane, keep_idx: torch.Tensor | None = None, stream=None) -> QPlane:
    """src: bf16 tensor [L][T][H][D] (strided view allowed) or PagedKV.  Fills dst.codes / dst.scales."""
    k = 0
    kp = None
    if keep_idx is not None:
        if keep_idx.dtype != torch.int32 or not keep_idx.is_contiguous() or keep_idx.dim() != 3 or not keep_idx.is_cuda:
            raise ValueError("keep_idx must be a contiguous int32 cuda tensor [L][H][k]")
        k = keep_idx.shape[2]
        kp = keep_idx.data_ptr()
    qp = _qplane(dst)
    if isinstance(src, PagedKV):
        pg = _paged(src)
        rc = _lib.kvp_quantize(None, ctypes.byref(pg), kp, k, ctypes.byref(qp), _stream(stream, dst.codes))
    else:
        if not src.is_cuda:
            raise ValueError("kvp_* operations run on the GPU only: tensors must live on a cuda device")
        vw = _view(src)
        rc = _lib.kvp_quantize(ctypes.byref(vw), None, kp, k, ctypes.byref(qp), _stream(stream, dst.codes))
    if rc != 0:
        raise KVPError(rc, "kvp_quantize")
    return dst


def kvp_dequantize_paged(src: QPlane, dst: PagedKV, stream=None) -> PagedKV:
    qp, pg = _qplane(src), _paged(dst)
    rc = _lib.kvp_dequantize_paged(ctypes.byref(qp), ctypes.byref(pg), _stream(stream, src.codes))
    if rc != 0:
        raise KVPError(rc, "kvp_dequantize_paged")
    return dst


def kvp_dequantize_paged_scatter(src: QPlane, keep_idx: torch.Tensor, dst: PagedKV, stream=None) -> PagedKV:
    """Restore the k slots of a dropped+quantized plane at tokens keep_idx int32 [L][H][k] of a T-token pool."""
    _need_cuda(keep_idx)
    qp, pg = _qplane(src), _paged(dst)
    if keep_idx.dtype != torch.int32 or not keep_idx.is_contiguous() or tuple(keep_idx.shape) != (qp.L, qp.H, src.T):
        raise ValueError("keep_idx must be contiguous int32 [L][H][k] with k = src.T")
    _check(_lib.kvp_dequantize_paged_scatter(ctypes.byref(qp), keep_idx.data_ptr(), ctypes.byref(pg), _stream(stream)),
           "kvp_dequantize_paged_scatter")
    return dst


def kvp_score_workspace_bytes(L: int, Hkv: int, Hq: int, W: int, T: int) -> int:
    return int(_lib.kvp_score_workspace_bytes(L, Hkv, Hq, W, T))


def kvp_score_tokens(q_win: torch.Tensor, k: torch.Tensor, scores: torch.Tensor | None = None, causal: bool = True,
                     force_window: bool = True, ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """q_win bf16 [L][W][Hq][D], k bf16 [L][T][Hkv][D] -> scores f32 [L][Hkv][T]."""
    _need_cuda(q_win, k, scores, ws)
    L, T, Hkv, _ = k.shape
    _, W, Hq, _ = q_win.shape
    if scores is None:
        scores = torch.empty(L, Hkv, T, dtype=torch.float32, device=k.device)
    if scores.dtype != torch.float32 or not scores.is_contiguous() or tuple(scores.shape) != (L, Hkv, T):
        raise ValueError("scores must be contiguous float32 [L][Hkv][T]")
    ws, wp, wb = _workspace(ws, kvp_score_workspace_bytes(L, Hkv, Hq, W, T), k.device, stream)
    qv, kv = _view(q_win), _view(k)
    _check(_lib.kvp_score_tokens(ctypes.byref(qv), ctypes.byref(kv), int(causal), int(force_window),
                                 scores.data_ptr(), wp, wb, _stream(stream)), "kvp_score_tokens")
    return scores


KVP_SCORE_STATIC_SCRATCH_BYTES = 4 << 20


def kvp_score_tokens_static(q_win: torch.Tensor, k: torch.Tensor, scores: torch.Tensor, causal: bool = True,
                            force_window: bool = True, stream=None) -> torch.Tensor:
    """kvp_score_tokens with the scratch in the library's own fixed device array: nothing is allocated,
    here or in the library, so `scores` must be supplied (contiguous f32 [L][Hkv][T])."""
    _need_cuda(q_win, k, scores)
    L, T, Hkv, _ = k.shape
    if scores.dtype != torch.float32 or not scores.is_contiguous() or tuple(scores.shape) != (L, Hkv, T):
        raise ValueError("scores must be contiguous float32 [L][Hkv][T]")
    qv, kv = _view(q_win), _view(k)
    _check(_lib.kvp_score_tokens_static(ctypes.byref(qv), ctypes.byref(kv), int(causal), int(force_window),
                                        scores.data_ptr(), _stream(stream)), "kvp_score_tokens_static")
    return scores


KVP_SCORE_KNORM, KVP_SCORE_KEYDIFF = 0, 1


def kvp_score_keys_workspace_bytes(L: int, H: int, T: int, method: int) -> int:
    return int(_lib.kvp_score_keys_workspace_bytes(L, H, T, method))


def kvp_score_keys(k: torch.Tensor, method: int, scores: torch.Tensor | None = None,
                   ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """k bf16 [L][T][H][D] -> key-only importance f32 [L][H][T] (knorm or keydiff), keep the largest."""
    _need_cuda(k, scores, ws)
    L, T, H, _ = k.shape
    if scores is None:
        scores = torch.empty(L, H, T, dtype=torch.float32, device=k.device)
    if scores.dtype != torch.float32 or not scores.is_contiguous() or tuple(scores.shape) != (L, H, T):
        raise ValueError("scores must be contiguous float32 [L][H][T]")
    ws, wp, wb = _workspace(ws, kvp_score_keys_workspace_bytes(L, H, T, method), k.device, stream)
    kv = _view(k)
    _check(_lib.kvp_score_keys(ctypes.byref(kv), int(method), scores.data_ptr(), wp, wb, _stream(stream)),
           "kvp_score_keys")
    return scores


def kvp_select_workspace_bytes(n_rows: int, T: int, k: int) -> int:
    return int(_lib.kvp_select_workspace_bytes(n_rows, T, k))


def kvp_select_topk(scores: torch.Tensor, k: int, idx_out: torch.Tensor | None = None,
                    ws: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """scores f32 [n_rows][T] (row stride >= T) -> idx int32 [n_rows][k], ascending."""
    _need_cuda(scores, idx_out, ws)
    if scores.dtype != torch.float32 or scores.dim() != 2 or (scores.shape[1] > 1 and scores.stride(1) != 1):
        raise ValueError("scores must be float32 [n_rows][T] with contiguous rows")
    n_rows, T = scores.shape
    row_stride = scores.stride(0) if n_rows > 1 else T
    if idx_out is None:
        idx_out = torch.empty(n_rows, k, dtype=torch.int32, device=scores.device)
    if idx_out.dtype != torch.int32 or not idx_out.is_contiguous() or tuple(idx_out.shape) != (n_rows, k):
        raise ValueError("idx_out must be contiguous int32 [n_rows][k]")
    ws, wp, wb = _workspace(ws, kvp_select_workspace_bytes(n_rows, T, k), scores.device, stream)
    _check(_lib.kvp_select_topk(scores.data_ptr(), n_rows, T, row_stride, k, idx_out.data_ptr(), wp, wb,
                                _stream(stream)), "kvp_select_topk")
    return idx_out


def kvp_smooth_scores(scores: torch.Tensor, window: int, kernel: int, mode: str = "avg",
                      out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """1-D pooling ("avg" or "max", odd kernel) of the prefix scores of f32 [n_rows][T]; window entries copied."""
    _need_cuda(scores, out)
    if scores.dtype != torch.float32 or scores.dim() != 2 or (scores.shape[1] > 1 and scores.stride(1) != 1):
        raise ValueError("scores must be float32 [n_rows][T] with contiguous rows")
    n_rows, T = scores.shape
    if out is None:
        out = torch.empty(n_rows, T, dtype=torch.float32, device=scores.device)
    if out.dtype != torch.float32 or tuple(out.shape) != (n_rows, T) or (T > 1 and out.stride(1) != 1):
        raise ValueError("out must be float32 [n_rows][T] with contiguous rows")
    _check(_lib.kvp_smooth_scores(scores.data_ptr(), n_rows, T, scores.stride(0) if n_rows > 1 else T, window, kernel,
                                  {"avg": 0, "max": 1}[mode], out.data_ptr(), out.stride(0) if n_rows > 1 else T,
                                  _stream(stream)), "kvp_smooth_scores")
    return out


def kvp_eval_workspace_bytes(L: int, Hkv: int, Hq: int, W: int, T: int, n_cfgs: int) -> int:
    return int(_lib.kvp_eval_workspace_bytes(L, Hkv, Hq, W, T, n_cfgs))


def kvp_eval_configs(q_win: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cfgs: Iterable[Sequence[int]],
                     loss: torch.Tensor | None = None, partial: torch.Tensor | None = None,
                     ws: torch.Tensor | None = None, stream=None, want_partial: bool = False,
                     pv_matrix_cores: bool = False, pv_fp32: bool = False):
    """cfgs: (bits, group, keep_k) triples.  Returns loss f32 [n] (and partial f32 [L][n][2] if asked).
    pv_matrix_cores / pv_fp32 select kvp_eval_configs_ex with KVP_EVAL_PV_MATRIX_CORES / KVP_EVAL_PV_FP32."""
    _need_cuda(q_win, k, v, loss, partial, ws)
    cfgs = list(cfgs)
    n = len(cfgs)
    L, T, Hkv, _ = k.shape
    _, W, Hq, _ = q_win.shape
    arr = (_Config * max(n, 1))(*[_Config(int(b), int(g), int(kk)) for b, g, kk in cfgs])
    if loss is None:
        loss = torch.empty(n, dtype=torch.float32, device=k.device)
    if want_partial and partial is None:
        partial = torch.empty(L, n, 2, dtype=torch.float32, device=k.device)
    ws, wp, wb = _workspace(ws, kvp_eval_workspace_bytes(L, Hkv, Hq, W, T, n), k.device, stream)
    qv, kv, vv = _view(q_win), _view(k), _view(v)
    pp = partial.data_ptr() if partial is not None else None
    flags = (KVP_EVAL_PV_MATRIX_CORES if pv_matrix_cores else 0) | (KVP_EVAL_PV_FP32 if pv_fp32 else 0)
    if flags:
        _check(_lib.kvp_eval_configs_ex(ctypes.byref(qv), ctypes.byref(kv), ctypes.byref(vv), arr, n, loss.data_ptr(),
                                        pp, wp, wb, flags, _stream(stream)), "kvp_eval_configs_ex")
    else:
        _check(_lib.kvp_eval_configs(ctypes.byref(qv), ctypes.byref(kv), ctypes.byref(vv), arr, n, loss.data_ptr(),
                                     pp, wp, wb, _stream(stream)), "kvp_eval_configs")
    return (loss, partial) if partial is not None else loss


KVP_OP_INSERT, KVP_OP_COMPRESS, KVP_OP_EVICT = 0, 1, 2
KVP_EVAL_PV_MATRIX_CORES = 1
KVP_EVAL_PV_FP32 = 2


def _tiers(tiers):
    return (_Tier * len(tiers))(*[_Tier(float(c), float(b)) for c, b in tiers])


def kvp_utility_table(quality, nbytes, tiers, alpha: float, frequency: float = 1.0):
    """Host call.  quality, nbytes: sequences [n_cfg]; tiers: [(capacity_bytes, bandwidth)] -> util [n_tiers][n_cfg]."""
    import numpy as np
    q = np.ascontiguousarray(quality, dtype=np.float64)
    b = np.ascontiguousarray(nbytes, dtype=np.float64)
    out = np.empty((len(tiers), len(q)), dtype=np.float64)
    _check(_lib.kvp_utility_table(q.ctypes.data, b.ctypes.data, len(q), _tiers(tiers), len(tiers), float(alpha),
                                  float(frequency), out.ctypes.data), "kvp_utility_table")
    return out


def kvp_policy_insert(nbytes, quality, frequency, tiers, alpha: float, ctx_tier, ctx_cfg, incoming: int,
                      max_ops: int | None = None):
    """Host call.  nbytes, quality: [n_ctx][n_cfg]; ctx_tier / ctx_cfg: int32 numpy arrays updated in place.
    Returns the list of (ctx, cfg, tier, op)."""
    import numpy as np
    b = np.ascontiguousarray(nbytes, dtype=np.float64)
    q = np.ascontiguousarray(quality, dtype=np.float64)
    f = np.ascontiguousarray(frequency, dtype=np.float64)
    n_ctx, n_cfg = b.shape
    if ctx_tier.dtype != np.int32 or ctx_cfg.dtype != np.int32:
        raise ValueError("ctx_tier and ctx_cfg must be int32 numpy arrays")
    if max_ops is None:
        max_ops = 1 + n_ctx * (n_cfg + len(tiers))
    ops = (_PolicyOp * max_ops)()
    n = _i32(0)
    rc = _lib.kvp_policy_insert(n_ctx, n_cfg, b.ctypes.data, q.ctypes.data, f.ctypes.data, _tiers(tiers), len(tiers),
                                float(alpha), ctx_tier.ctypes.data, ctx_cfg.ctypes.data, int(incoming), ops, max_ops,
                                ctypes.byref(n))
    _check(rc, "kvp_policy_insert")
    return [(o.ctx, o.cfg, o.tier, o.op) for o in ops[: n.value]]


def kvp_copy_bytes(dst: torch.Tensor, src: torch.Tensor, stream=None):
    _need_cuda(dst, src)
    n = src.numel() * src.element_size()
    _check(_lib.kvp_copy_bytes(dst.data_ptr(), src.data_ptr(), n, _stream(stream)), "kvp_copy_bytes")
