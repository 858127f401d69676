"""Host logic of the Python binding: the marshalled structs are cached per tensor and must follow every change of
what they are made of (no GPU needed: only pointers, shapes and strides are read)."""
import torch

from paper_2512_14946_amd import kvp as binding


def test_view_cache_follows_in_place_metadata_changes():
    t = torch.zeros(2, 6, 4, 128, dtype=torch.bfloat16)
    v = binding._view(t)
    assert (v.L, v.T, v.H, v.D, v.stride_l, v.stride_t, v.stride_h) == (2, 6, 4, 128, 6 * 4 * 128, 4 * 128, 128)
    assert binding._view(t) is v                                   # served from the cache
    t.transpose_(0, 1)                                             # same storage pointer, same element count
    w = binding._view(t)
    assert (w.L, w.T, w.stride_l, w.stride_t) == (6, 2, 4 * 128, 6 * 4 * 128)
    t.as_strided_((1, 3, 4, 128), (6 * 4 * 128, 2 * 4 * 128, 128, 1))
    x = binding._view(t)
    assert (x.L, x.T, x.stride_t) == (1, 3, 2 * 4 * 128)


def test_qplane_and_paged_caches_follow_replaced_tensors(monkeypatch):
    monkeypatch.setattr(binding, "_need_cuda", lambda *ts: None)   # only the descriptors are built here, nothing runs
    q = binding.alloc_qplane(1, 32, 2, 128, 4, 32, "cpu")
    a = binding._qplane(q)
    assert binding._qplane(q) is a
    q.scales = torch.zeros_like(q.scales)                          # another scales buffer under the same descriptor
    b = binding._qplane(q)
    assert b is not a and b.scales == q.scales.data_ptr()
    pool = torch.zeros(1, 4, 16, 2, 128, dtype=torch.bfloat16)
    p = binding.PagedKV(pool, torch.arange(2, dtype=torch.int32), 32)
    c = binding._paged(p)
    assert binding._paged(p) is c
    p.block_table = torch.tensor([3, 1], dtype=torch.int32)
    d = binding._paged(p)
    assert d is not c and d.block_table == p.block_table.data_ptr()
