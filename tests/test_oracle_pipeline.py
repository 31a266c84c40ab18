"""End-to-end pins for the oracle's DETOX step (Algorithms 1 and 2)."""
import numpy as np
import pytest

import oracle
import workloads


def test_config1_by_hand():
    # three honest votes, vote groups of one: the output is the per-coordinate median of the
    # three honest gradients, whatever the Byzantine node sent
    w = workloads.config(1)
    out, winner, Zh = oracle.detox_step(w.matrix(), 3, 3, "coord_median")
    assert out.tobytes() == np.median(w.base, axis=0).astype(np.float32).tobytes()


@pytest.mark.parametrize("idx,B,agg,kw", [
    (2, 5, "multikrum", dict(f=1, m=3)), (3, 5, "multikrum", dict(f=1, m=3)),
    (4, 15, "bulyan", dict(f=1)), (4, 5, "coord_median", {}), (5, 7, "geomedian", {})])
def test_output_does_not_depend_on_what_the_byzantine_rows_hold(idx, B, agg, kw):
    # Section 3.1: with fewer than r/2 Byzantine members per group every vote is honest
    w = workloads.config(idx, d=2003)
    out, winner, _ = oracle.detox_step(w.matrix(), w.r, B, agg, **kw)
    rng = np.random.default_rng(idx)
    for i in list(w.byz):
        w.byz[i] = rng.standard_normal(w.d).astype(np.float32) * 1e6
    out2, winner2, _ = oracle.detox_step(w.matrix(), w.r, B, agg, **kw)
    assert out.tobytes() == out2.tobytes() and winner.tolist() == winner2.tolist()


@pytest.mark.parametrize("agg,kw", [("multikrum", dict(f=0, m=5)), ("bulyan", dict(f=0))])
def test_no_attack_reduces_to_the_plain_mean(agg, kw):
    w = workloads.config(3, d=1500)
    w.byz.clear()
    out, _, _ = oracle.detox_step(w.matrix(), 3, 5, agg, **kw)
    ref = w.honest_mean()
    assert np.linalg.norm(out - ref) / np.linalg.norm(ref) < 1e-6


def test_group_and_vote_permutations_cancel():
    w = workloads.config(3, d=700)
    G = w.matrix()
    out, _, _ = oracle.detox_step(G, 3, 5, "coord_median")
    rng = np.random.default_rng(9)
    order = rng.permutation(15)
    group_rows = np.concatenate([3 * g + rng.permutation(3) for g in order]).astype(np.int32)
    vote_perm = np.argsort(order).astype(np.int32)           # put the votes back in their old order
    out2, _, _ = oracle.detox_step(G, 3, 5, "coord_median", group_rows=group_rows, vote_perm=vote_perm)
    assert out.tobytes() == out2.tobytes()
