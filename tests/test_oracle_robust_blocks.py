"""Pins for the oracle's deployed hierarchy (Section 5.2, setups 2 and 3; Appendix B.1):
A0 = Multi-Krum / Bulyan inside every vote group, A1 = mean."""
import numpy as np
import pytest

import oracle
import workloads
from test_oracle_krum import _krum_by_subsets


def test_uneven_groups_of_appendix_b1_by_brute_force():
    # 15 votes in two groups of 7 and 8; each group's Multi-Krum checked by subset enumeration
    rng = np.random.default_rng(4)
    base = rng.integers(-6, 7, size=(15, 4)).astype(np.float32)
    G = np.repeat(base, 3, axis=0)
    out, winner, block_out, sels = oracle.detox_step_robust_blocks(G, 3, 2, "multikrum", f=2, m=3)
    assert [len(s) for s in sels] == [3, 3]
    for b, (lo, hi) in enumerate(((0, 7), (7, 15))):
        X = base[lo:hi]
        D = ((X[:, None, :].astype(np.int64) - X[None, :, :].astype(np.int64)) ** 2).sum(-1)
        _, sel = _krum_by_subsets(D.tolist(), 2, 3)
        assert sels[b].tolist() == sel
        np.testing.assert_allclose(block_out[b], X[sel].astype(np.float64).mean(axis=0), rtol=1e-7)
    np.testing.assert_allclose(out, block_out.astype(np.float64).mean(axis=0), rtol=1e-7)


@pytest.mark.parametrize("a0,B,f", [("multikrum", 3, 0), ("bulyan", 3, 0), ("multikrum", 1, 0), ("bulyan", 5, 0)])
def test_no_attack_and_f0_is_the_plain_mean(a0, B, f):
    w = workloads.config(3, d=900)
    w.byz.clear()
    out, _, _, _ = oracle.detox_step_robust_blocks(w.matrix(), 3, B, a0, f)
    ref = w.honest_mean()
    assert np.linalg.norm(out - ref) / np.linalg.norm(ref) < 1e-6


@pytest.mark.parametrize("a0,B,f", [("multikrum", 2, 2), ("bulyan", 1, 2), ("bulyan", 1, 3)])
def test_independent_of_byzantine_content_and_single_group_is_the_aggregator(a0, B, f):
    w = workloads.config(3, d=1200)
    out, winner, block_out, sels = oracle.detox_step_robust_blocks(w.matrix(), 3, B, a0, f)
    if B == 1:
        votes = w.base          # every vote is honest here
        direct = oracle.bulyan(votes, f)[0]
        assert out.tobytes() == direct.tobytes()
    for i in list(w.byz):
        w.byz[i] = np.full(w.d, 1e9, dtype=np.float32)
    out2 = oracle.detox_step_robust_blocks(w.matrix(), 3, B, a0, f)[0]
    assert out.tobytes() == out2.tobytes()


def test_requirements_per_group():
    w = workloads.config(3, d=50)
    with pytest.raises(oracle.OracleError):
        oracle.detox_step_robust_blocks(w.matrix(), 3, 2, "bulyan", 2)      # groups of 7 and 8 < 4*2+3
