"""GPU parity of kvp_select_topk on seeded random row lengths of every class (rows resident in registers, rows split
over workgroups, rows streamed by one workgroup) with adversarial value distributions (heavy ties, ascending rows,
forty decades of magnitude, +inf and -0 entries), rows farther apart than their length.  Indices bit-exact."""
import numpy as np
import pytest
import torch

import oracle

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _kvp():
    import paper_2512_14946_amd as kvp
    return kvp


def _select_cases():
    rng = np.random.default_rng(1234)
    cases = []
    for i in range(36):
        kind = i % 6
        if kind == 0:
            T = int(rng.integers(1, 300))
        elif kind == 1:
            T = int(rng.integers(300, 16385))
        elif kind == 2:
            T = int(rng.integers(16385, 40000))
        elif kind == 3:
            T = int(rng.integers(40000, 262145))
        elif kind == 4:
            T = int(rng.choice([16384, 16385, 32768, 32769, 65536, 131072, 262144, 262145]))
        else:
            T = int(rng.integers(262145, 300000))
        n_rows = int(rng.integers(1, 4)) if T > 60000 else int(rng.integers(1, 12))
        k = [1, T, max(1, T // 2), int(rng.integers(1, T + 1)), max(1, T // 10)][int(rng.integers(0, 5))]
        cases.append((i, T, n_rows, k, i % 5))
    return cases


@pytest.mark.parametrize("seed,T,n_rows,k,dist", _select_cases())
def test_select_topk_random_shapes(seed, T, n_rows, k, dist):
    kvp = _kvp()
    print("[case] select", dict(seed=seed, T=T, n_rows=n_rows, k=k, dist=dist), flush=True)
    rng = np.random.default_rng(10_000 + seed)
    if dist == 0:
        s = rng.standard_normal((n_rows, T)).astype(np.float32) ** 2
    elif dist == 1:
        s = rng.integers(0, 4, (n_rows, T)).astype(np.float32)                              # heavy ties
    elif dist == 2:
        s = np.sort(rng.standard_normal((n_rows, T)).astype(np.float32), axis=1)            # ascending rows
    elif dist == 3:
        s = (rng.standard_normal((n_rows, T)) * 10.0 ** rng.uniform(-20, 20, (n_rows, 1))).astype(np.float32)
    else:
        s = rng.standard_normal((n_rows, T)).astype(np.float32)
        s[:, rng.integers(0, T, max(1, T // 50))] = np.inf                                   # forced-window style +inf
        s[rng.integers(0, n_rows), rng.integers(0, T)] = -0.0
    pad = int(rng.integers(0, 3)) * 4                                                        # rows farther apart than T
    buf = torch.zeros(n_rows, T + pad, dtype=torch.float32, device=DEV)
    buf[:, :T] = torch.from_numpy(s).to(DEV)
    got = kvp.kvp_select_topk(buf[:, :T], k)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), oracle.select_topk(s, k))
