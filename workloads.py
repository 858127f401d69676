"""Seeded synthetic inputs shaped like the KV caches of the paper's serving workloads.

This module holds NO arithmetic of the method: it only draws random tensors and
page tables.  Both the HIP path and the CPU oracle are fed from here (the bytes
generated on one side are copied to the other, so the two never depend on the
generator reproducing bit-identical numbers across devices).

Recipe (every config, seed stated per call):
  K ~ N(0,1) in fp32; for each (layer, kv head) `n_outliers` channel indices,
  fixed for all tokens and drawn once without replacement, are multiplied by
  `outlier_scale`; cast to bf16.  V ~ N(0,1) -> bf16.  Window queries
  Q ~ N(0,1) -> bf16, shape [L][W][G*Hkv][D].  Block tables are a seeded random
  permutation of the physical blocks (pages scattered as in a live server).
These stand in for real KV caches of long-context datasets (mean lengths
12K-108K tokens in the paper's dataset table), which are not available here.
"""
from __future__ import annotations

import torch

# name -> shape and op parameters of the five benchmark configurations
CONFIGS = {
    "single_layer_int8": dict(L=1, H=8, D=128, T=4096, G=4, W=32, bits=8, group=128, keep_ratio=0.5,
                              outlier_scale=8.0, bs=16),
    "llama3_8b_int4_paged": dict(L=32, H=8, D=128, T=32768, G=4, W=32, bits=4, group=64, keep_ratio=None,
                                 outlier_scale=8.0, bs=16),
    "utility_sweep": dict(L=32, H=8, D=128, T=8192, G=4, W=32, n_ctx=64, bits_set=(8, 4, 2),
                          group_set=(32, 64, 128), keep_ratios=(0.25, 0.5, 0.75), outlier_scale=8.0, bs=16),
    "llama3_70b_drop_int4": dict(L=80, H=8, D=128, T=16384, G=8, W=64, bits=4, group=32, keep_ratio=0.3,
                                 outlier_scale=8.0, bs=16),
    "long_context_int2": dict(L=28, H=4, D=128, T=131072, G=7, W=32, bits=2, group=32, keep_ratio=0.1,
                              outlier_scale=16.0, bs=16),
}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_kv(L: int, T: int, H: int, D: int, seed: int = 0, outlier_scale: float = 8.0, n_outliers: int = 4,
            device="cpu"):
    """K, V as bf16 tensors [L][T][H][D]."""
    g = _gen(seed, device)
    # outlier channels: fixed per (layer, head), drawn once without replacement
    ch = torch.rand(L, H, D, generator=g, device=device).argsort(dim=-1)[..., :n_outliers]
    mult = torch.ones(L, H, D, device=device)
    mult.scatter_(-1, ch, float(outlier_scale))
    K = torch.empty(L, T, H, D, dtype=torch.bfloat16, device=device)
    V = torch.empty(L, T, H, D, dtype=torch.bfloat16, device=device)
    for l in range(L):  # layer by layer keeps the fp32 staging small
        K[l] = (torch.randn(T, H, D, generator=g, device=device) * mult[l]).to(torch.bfloat16)
        V[l] = torch.randn(T, H, D, generator=g, device=device).to(torch.bfloat16)
    return K, V


def make_q(L: int, W: int, Hq: int, D: int, seed: int = 0, device="cpu"):
    """Window queries (the last W positions of the context), bf16 [L][W][Hq][D]."""
    g = _gen(seed + 1_000_003, device)
    return torch.randn(L, W, Hq, D, generator=g, device=device).to(torch.bfloat16)


def make_block_table(T: int, bs: int = 16, seed: int = 0, spare: int = 0, device="cpu"):
    """int32 [ceil(T/bs)] physical block ids: a random permutation of num_blocks = ceil(T/bs) + spare."""
    nb = (T + bs - 1) // bs + spare
    g = _gen(seed + 2_000_003, "cpu")
    perm = torch.randperm(nb, generator=g)[: (T + bs - 1) // bs].to(torch.int32)
    return perm.to(device), nb


def make_scores(n_rows: int, T: int, seed: int = 0, device="cpu", levels: int | None = None):
    """Stand-in score rows, fp32 [n_rows][T]: squared normals, or a few discrete levels (many ties)."""
    g = _gen(seed + 3_000_003, device)
    if levels is None:
        return torch.randn(n_rows, T, generator=g, device=device).square_()
    return torch.randint(0, levels, (n_rows, T), generator=g, device=device).to(torch.float32)
