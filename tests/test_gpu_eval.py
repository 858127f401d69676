"""GPU parity: kvp_eval_configs against the CPU oracle (1e-2 relative + 1e-5 absolute)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from helpers import torch_bits

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _kvp():
    import paper_2512_14946_amd as kvp
    return kvp


PV_MODES = {"pv_dot2_fp16": {}, "pv_fp32": {"pv_fp32": True}, "pv_matrix_cores": {"pv_matrix_cores": True}}


def _case(L, W, G, H, T, cfgs, seed, outlier=8.0, pv="pv_dot2_fp16"):
    kvp = _kvp()
    D = 128
    print("[case] eval", dict(L=L, W=W, G=G, H=H, T=T, n=len(cfgs), pv=pv), flush=True)
    K, V = workloads.make_kv(L, T, H, D, seed=seed, outlier_scale=outlier)
    Q = workloads.make_q(L, W, G * H, D, seed=seed)
    loss, partial = kvp.kvp_eval_configs(Q.to(DEV), K.to(DEV), V.to(DEV), cfgs, want_partial=True,
                                         **PV_MODES[pv])
    torch.cuda.synchronize()
    loss, partial = loss.cpu().numpy(), partial.cpu().numpy()
    ref, ref_partial = oracle.eval_configs(torch_bits(Q), torch_bits(K), torch_bits(V), cfgs)
    assert np.all(np.abs(loss - ref) <= 1e-2 * np.abs(ref) + 1e-5), (loss, ref)
    assert np.allclose(partial[..., 1], ref_partial[..., 1], rtol=1e-3)
    # the numerator is the square of the loss's numerator: twice the relative tolerance of the loss
    assert np.all(np.abs(partial[..., 0] - ref_partial[..., 0]) <= 2e-2 * ref_partial[..., 0] + 1e-7)
    return loss, ref


def _sweep(T):
    ks = [oracle.keep_count(r, T) for r in (0.25, 0.5, 0.75)] + [T]
    variants = [(16, 0)] + [(b, g) for b in (8, 4, 2) for g in (32, 64, 128)]
    return [(b, g, k) for (b, g) in variants for k in ks]


BOTH_PV = pytest.mark.parametrize("pv", list(PV_MODES))


@BOTH_PV
def test_full_candidate_sweep_small(pv):
    T = 300                                            # ragged: 300 = 9 tiles of 32 + 12
    cfgs = _sweep(T)
    assert len(cfgs) == 40
    loss, ref = _case(2, 32, 4, 2, T, cfgs, seed=0, pv=pv)
    assert loss[3] == 0.0                              # (16 bits, keep all) is the identity, exactly
    order = {c: i for i, c in enumerate(cfgs)}
    for g in (32, 64, 128):                            # fewer bits, larger loss
        assert loss[order[(8, g, T)]] < loss[order[(4, g, T)]] < loss[order[(2, g, T)]]


@BOTH_PV
def test_padded_row_blocks_and_tiny_keep(pv):
    T = 200
    cfgs = [(16, 0, T), (8, 128, T), (4, 32, 77), (2, 64, 33), (16, 0, 5), (4, 64, 1)]
    # M = 224: two row blocks, the second partly filled
    _case(1, 32, 7, 2, T, cfgs, seed=1, outlier=16.0, pv=pv)


@BOTH_PV
def test_many_rows_and_duplicates(pv):
    T = 130
    cfgs = [(8, 32, 64), (8, 32, 64), (16, 0, 64), (2, 32, T)]
    loss, _ = _case(1, 64, 8, 1, T, cfgs, seed=2, pv=pv)      # M = 512: four row blocks
    assert loss[0] == loss[1]


@BOTH_PV
def test_no_16_bit_config_and_no_keep_all(pv):
    """No configuration asks for 16 bits and none keeps every token: the reference comes from a hidden stream that
    walks the tokens no keep level holds as well."""
    T = 150
    cfgs = [(4, 64, 50), (8, 128, 100), (2, 32, 100)]
    _case(2, 32, 4, 2, T, cfgs, seed=3, pv=pv)
    _case(1, 16, 2, 1, 97, [(8, 32, 40)], seed=4, pv=pv)      # a single configuration
    # the 16-bit codec is listed last and never with all tokens
    _case(1, 32, 4, 1, T, [(2, 128, 75), (4, 32, 20), (16, 0, 75)], seed=5, pv=pv)


def test_pv_modes_agree():
    """The three forms of the P.V product against each other on one input: the matrix-core form (two-term bf16
    split of P) follows the fp32 form to 1e-4, the default form (P rounded to fp16) to 2e-3."""
    kvp = _kvp()
    L, W, G, H, T, D = 2, 32, 4, 2, 1000, 128
    print("[case] eval modes", dict(L=L, W=W, G=G, H=H, T=T), flush=True)
    K, V = workloads.make_kv(L, T, H, D, seed=9, outlier_scale=8.0)
    Q = workloads.make_q(L, W, G * H, D, seed=9)
    cfgs = _sweep(T)
    out = {m: kvp.kvp_eval_configs(Q.to(DEV), K.to(DEV), V.to(DEV), cfgs, **kw).cpu().numpy() for m, kw in PV_MODES.items()}
    ref = out["pv_fp32"]
    assert np.all(np.abs(out["pv_matrix_cores"] - ref) <= 1e-4 * ref + 1e-7)
    assert np.all(np.abs(out["pv_dot2_fp16"] - ref) <= 2e-3 * ref + 1e-6)
    assert out["pv_dot2_fp16"][3] == 0.0 and ref[3] == 0.0


def test_value_range_of_the_fp16_pair_form():
    """V beyond the fp16 range: the default P.V form (fp16 pairs) must answer with a non-finite loss, never a
    plausible number; the fp32 form stays within tolerance of the oracle.  Small magnitudes (fp16 subnormals)
    stay within tolerance in both."""
    kvp = _kvp()
    L, W, G, H, T, D = 1, 32, 2, 1, 160, 128
    print("[case] eval value range", dict(L=L, W=W, G=G, H=H, T=T), flush=True)
    K, V = workloads.make_kv(L, T, H, D, seed=11, outlier_scale=8.0)
    Q = workloads.make_q(L, W, G * H, D, seed=11)
    cfgs = [(16, 0, T), (8, 32, T), (4, 64, 80)]
    big = V.clone()
    big[0, 3, 0, 5] = 1.0e5
    got = kvp.kvp_eval_configs(Q.to(DEV), K.to(DEV), big.to(DEV), cfgs).cpu().numpy()
    assert not np.all(np.isfinite(got))
    ref, _ = oracle.eval_configs(torch_bits(Q), torch_bits(K), torch_bits(big), cfgs)
    got32 = kvp.kvp_eval_configs(Q.to(DEV), K.to(DEV), big.to(DEV), cfgs, pv_fp32=True).cpu().numpy()
    assert np.all(np.abs(got32 - ref) <= 1e-2 * np.abs(ref) + 1e-5), (got32, ref)
    small = (V.float() * 2.0 ** -12).to(torch.bfloat16)          # |v| around 2^-12: many values below 2^-14
    ref, _ = oracle.eval_configs(torch_bits(Q), torch_bits(K), torch_bits(small), cfgs)
    for kw in ({}, {"pv_fp32": True}):
        got = kvp.kvp_eval_configs(Q.to(DEV), K.to(DEV), small.to(DEV), cfgs, **kw).cpu().numpy()
        assert np.all(np.abs(got - ref) <= 1e-2 * np.abs(ref) + 1e-5), (kw, got, ref)


def test_errors():
    kvp = _kvp()
    q = torch.zeros(1, 8, 4, 128, dtype=torch.bfloat16, device=DEV)
    k = torch.zeros(1, 64, 2, 128, dtype=torch.bfloat16, device=DEV)
    with pytest.raises(kvp.KVPError):
        kvp.kvp_eval_configs(q, k, k, [(3, 32, 64)])
    with pytest.raises(kvp.KVPError):
        kvp.kvp_eval_configs(q, k, k, [(4, 32, 65)])
    with pytest.raises(kvp.KVPError):
        kvp.kvp_eval_configs(q, k, k, [(4, 32, 8)], ws=torch.empty(16, dtype=torch.uint8, device=DEV))
    with pytest.raises(kvp.KVPError):                  # the two P.V flags exclude each other
        kvp.kvp_eval_configs(q, k, k, [(4, 32, 8)], pv_matrix_cores=True, pv_fp32=True)
