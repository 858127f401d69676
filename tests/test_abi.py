"""CPU-only checks of the C-ABI boundary: the library loads, exports every symbol the header
declares, and its host-side helpers and argument validation work without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "kvp.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2512_14946_amd import build
    if not os.path.exists(build.LIB):
        build.build_library()
    return ctypes.CDLL(build.LIB)


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert {"kvp_quantize", "kvp_dequantize_paged", "kvp_score_tokens", "kvp_select_topk",
            "kvp_eval_configs"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in kvp.h but not exported"


def test_host_helpers(lib):
    lib.kvp_keep_count.restype = ctypes.c_int64
    lib.kvp_keep_count.argtypes = [ctypes.c_double, ctypes.c_int64]
    assert lib.kvp_keep_count(0.5, 4096) == 2048
    assert lib.kvp_keep_count(0.3, 16384) == 4916
    assert lib.kvp_keep_count(0.1, 131072) == 13108
    assert [lib.kvp_keep_count(r, 8192) for r in (0.25, 0.5, 0.75)] == [2048, 4096, 6144]
    assert lib.kvp_keep_count(0.0, 5) == 1 and lib.kvp_keep_count(2.0, 5) == 5
    lib.kvp_strerror.restype = ctypes.c_char_p
    assert lib.kvp_strerror(0) == b"ok"
    assert all(len(lib.kvp_strerror(c)) >= 2 for c in range(-7, 1))
    lib.kvp_version.restype = ctypes.c_uint32
    assert lib.kvp_version() >= 0x00010000


def test_validation_rejects_before_any_launch(lib):
    # NULL structs / pointers are refused on the host: no GPU is needed (and none is touched)
    lib.kvp_quantize.restype = ctypes.c_int32
    lib.kvp_quantize.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_int64] + [ctypes.c_void_p] * 2
    assert lib.kvp_quantize(None, None, None, 0, None, None) == -1
    lib.kvp_dequantize_paged.restype = ctypes.c_int32
    lib.kvp_dequantize_paged.argtypes = [ctypes.c_void_p] * 3
    assert lib.kvp_dequantize_paged(None, None, None) == -1
    lib.kvp_select_topk.restype = ctypes.c_int32
    lib.kvp_select_topk.argtypes = [ctypes.c_void_p] + [ctypes.c_int64] * 4 + [ctypes.c_void_p] * 2 + \
        [ctypes.c_size_t, ctypes.c_void_p]
    assert lib.kvp_select_topk(None, 1, 8, 8, 4, None, None, 0, None) == -1
    lib.kvp_score_tokens.restype = ctypes.c_int32
    lib.kvp_score_tokens.argtypes = [ctypes.c_void_p] * 2 + [ctypes.c_int32] * 2 + [ctypes.c_void_p] * 2 + \
        [ctypes.c_size_t, ctypes.c_void_p]
    assert lib.kvp_score_tokens(None, None, 1, 1, None, None, 0, None) == -1
    lib.kvp_copy_bytes.restype = ctypes.c_int32
    lib.kvp_copy_bytes.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert lib.kvp_copy_bytes(None, None, 16, None) == -1
    assert lib.kvp_copy_bytes(16, 32, 8, None) == -2
    lib.kvp_dequantize_paged_scatter.restype = ctypes.c_int32
    lib.kvp_dequantize_paged_scatter.argtypes = [ctypes.c_void_p] * 4
    assert lib.kvp_dequantize_paged_scatter(None, None, None, None) == -1
    lib.kvp_smooth_scores.restype = ctypes.c_int32
    lib.kvp_smooth_scores.argtypes = [ctypes.c_void_p] + [ctypes.c_int64] * 4 + [ctypes.c_int32] * 2 + \
        [ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
    assert lib.kvp_smooth_scores(None, 1, 8, 8, 0, 3, 0, None, 8, None) == -1
    assert lib.kvp_smooth_scores(256, 1, 8, 8, 0, 4, 0, 4096, 8, None) == -4      # even kernel
    assert lib.kvp_smooth_scores(256, 1, 8, 8, 0, 3, 7, 4096, 8, None) == -4      # unknown mode
    assert lib.kvp_smooth_scores(256, 1, 8, 8, 9, 3, 0, 4096, 8, None) == -3      # window longer than the row
    assert lib.kvp_smooth_scores(256, 2, 8, 8, 0, 3, 0, 256 + 32, 8, None) == -3  # overlapping rows
    assert lib.kvp_smooth_scores(256, 0, 8, 8, 0, 3, 0, 4096, 8, None) == 0       # nothing to do
    lib.kvp_eval_configs_ex.restype = ctypes.c_int32
    lib.kvp_eval_configs_ex.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int32] + [ctypes.c_void_p] * 3 + \
        [ctypes.c_size_t, ctypes.c_uint32, ctypes.c_void_p]
    assert lib.kvp_eval_configs_ex(None, None, None, None, 1, None, None, None, 0, 4, None) == -4   # unknown flag
    assert lib.kvp_eval_configs_ex(None, None, None, None, 1, None, None, None, 0, 3, None) == -4   # exclusive flags
    assert lib.kvp_eval_configs_ex(None, None, None, None, 1, None, None, None, 0, 1, None) == -1
    lib.kvp_score_keys.restype = ctypes.c_int32
    lib.kvp_score_keys.argtypes = [ctypes.c_void_p, ctypes.c_int32] + [ctypes.c_void_p] * 2 + [ctypes.c_size_t, ctypes.c_void_p]
    assert lib.kvp_score_keys(None, 0, None, None, 0, None) == -1


def test_static_scratch_entry_point_rejects_oversized_shapes_on_the_host(lib):
    # the size check is host arithmetic on the structs and comes before any GPU call: fake, aligned, never
    # dereferenced pointers are enough
    class View(ctypes.Structure):
        _fields_ = [("ptr", ctypes.c_void_p)] + [(n, ctypes.c_int64) for n in ("L", "T", "H", "D", "sl", "st", "sh")]
    lib.kvp_score_tokens_static.restype = ctypes.c_int32
    lib.kvp_score_tokens_static.argtypes = [ctypes.POINTER(View)] * 2 + [ctypes.c_int32] * 2 + [ctypes.c_void_p] * 2
    lib.kvp_score_workspace_bytes.restype = ctypes.c_size_t
    lib.kvp_score_workspace_bytes.argtypes = [ctypes.c_int64] * 5
    L, T, H, G, W = 80, 16384, 8, 8, 64
    assert lib.kvp_score_workspace_bytes(L, H, G * H, W, T) > (4 << 20)
    k = View(4096, L, T, H, 128, T * H * 128, H * 128, 128)
    q = View(8192, L, W, G * H, 128, W * G * H * 128, G * H * 128, 128)
    assert lib.kvp_score_tokens_static(ctypes.byref(q), ctypes.byref(k), 1, 1, 4096, None) == -5
    assert lib.kvp_score_tokens_static(None, None, 1, 1, None, None) == -1
    # one layer of the same shape fits
    assert lib.kvp_score_workspace_bytes(1, H, G * H, W, T) <= (4 << 20)
    assert lib.kvp_score_workspace_bytes(1, 8, 64, 64, 131072) <= (4 << 20)


def test_one_sizing_call_agrees_with_the_per_operation_helpers(lib):
    class Dims(ctypes.Structure):
        _fields_ = [(n, ctypes.c_int64) for n in ("L", "Hkv", "Hq", "W", "T", "n_rows", "k")] + \
                   [("n_cfgs", ctypes.c_int32), ("method", ctypes.c_int32)]
    lib.kvp_workspace_bytes.restype = ctypes.c_size_t
    lib.kvp_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.POINTER(Dims)]
    for f, n in (("kvp_score_workspace_bytes", 5), ("kvp_select_workspace_bytes", 3)):
        getattr(lib, f).restype = ctypes.c_size_t
        getattr(lib, f).argtypes = [ctypes.c_int64] * n
    lib.kvp_score_keys_workspace_bytes.restype = ctypes.c_size_t
    lib.kvp_score_keys_workspace_bytes.argtypes = [ctypes.c_int64] * 3 + [ctypes.c_int32]
    lib.kvp_eval_workspace_bytes.restype = ctypes.c_size_t
    lib.kvp_eval_workspace_bytes.argtypes = [ctypes.c_int64] * 5 + [ctypes.c_int32]
    d = Dims(32, 8, 32, 32, 8192, 112, 13108, 40, 1)
    assert lib.kvp_workspace_bytes(0, ctypes.byref(d)) == lib.kvp_score_workspace_bytes(32, 8, 32, 32, 8192) > 0
    assert lib.kvp_workspace_bytes(1, ctypes.byref(d)) == lib.kvp_score_keys_workspace_bytes(32, 8, 8192, 1) > 0
    assert lib.kvp_workspace_bytes(3, ctypes.byref(d)) == lib.kvp_eval_workspace_bytes(32, 8, 32, 32, 8192, 40) > 0
    assert lib.kvp_workspace_bytes(2, ctypes.byref(d)) == lib.kvp_select_workspace_bytes(112, 8192, 13108) == 0
    d.T = 131072
    long_rows = lib.kvp_select_workspace_bytes(112, 131072, 13108)
    assert lib.kvp_workspace_bytes(2, ctypes.byref(d)) == long_rows
    assert 112 * 16384 * 4 < long_rows < 112 * 16384 * 4 + (1 << 16)      # 64 KiB of candidate slots per row + counts
    assert lib.kvp_select_workspace_bytes(112, (1 << 18) + 1, 5) == 0          # beyond the split path: one block per row
    assert lib.kvp_workspace_bytes(9, ctypes.byref(d)) == 0 and lib.kvp_workspace_bytes(0, None) == 0
    # a long row without its workspace is refused on the host
    lib.kvp_select_topk.restype = ctypes.c_int32
    lib.kvp_select_topk.argtypes = [ctypes.c_void_p] + [ctypes.c_int64] * 4 + [ctypes.c_void_p] * 2 + \
        [ctypes.c_size_t, ctypes.c_void_p]
    assert lib.kvp_select_topk(4096, 2, 40000, 40000, 100, 8192, None, 0, None) == -5
    assert lib.kvp_select_topk(4096, 2, 40000, 40000, 100, 8192, 1 << 20, 64, None) == -5


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2512_14946_amd as kvp
    x = torch.zeros(1, 16, 8, 128, dtype=torch.bfloat16)
    qp = kvp.alloc_qplane(1, 16, 8, 128, 4, 64, "cpu")
    with pytest.raises(ValueError):
        kvp.kvp_quantize(x, qp)
    with pytest.raises(ValueError):
        kvp.kvp_select_topk(torch.zeros(2, 8), 4)
