"""Pins for the oracle in the synthetic mean-estimation setting of Section 5.3 (220000 nodes in
groups of 11, q = floor(e^11 / 3) Byzantine nodes): long key lists in the median, the expected
number of Byzantine votes of Appendix A.1, and the qualitative claim of the experiment."""
import math

import numpy as np
import pytest
from scipy.stats import hypergeom

import oracle
import workloads


@pytest.mark.parametrize("count", [257, 1000, 4001, 220000, 219999])
def test_median_of_long_columns_against_numpy_partition(count):
    rng = np.random.default_rng(count)
    X = rng.standard_normal((count, 3)).astype(np.float32)
    X[:, 1] = rng.integers(-3, 4, size=count)            # long runs of equal values
    got = oracle.coord_median(X)
    k = count // 2
    part = np.partition(X, [k - 1, k] if count > 1 else [k], axis=0)
    want = part[k] if count % 2 else (part[k - 1] + part[k]) * np.float32(0.5)
    assert got.tobytes() == want.astype(np.float32).tobytes()


def test_q_is_floor_e_to_the_r_over_three():
    w = workloads.mean_estimation(2)
    assert (w.n, w.r, w.q, w.groups) == (220000, 11, 19958, 20000)
    assert w.q == math.floor(math.exp(11) / 3)
    v = next(iter(w.byz.values()))
    assert abs(np.linalg.norm(v.astype(np.float64)) - 100.0) < 1e-3 and np.all(v == v[0])


def test_byzantine_votes_match_the_closed_form_of_appendix_a1():
    """E[q_hat] = (p/r) * P[a uniformly drawn group of r holds at least (r+1)/2 Byzantine nodes]:
    3.44 for this setting.  The filter must hand exactly those groups to the Byzantine vector and
    every other group to its honest value."""
    p, r = 220000, 11
    q = math.floor(math.exp(r) / 3)
    expected = (p / r) * hypergeom.sf((r + 1) // 2 - 1, p, q, r)
    assert 3.3 < expected < 3.6
    seen = []
    for seed in range(40):
        w = workloads.mean_estimation(2, seed=seed)
        G = w.matrix()
        winner = oracle.majority_filter(G, r)
        assert (winner >= 0).all()                        # Byzantine nodes collude: never a split
        is_byz = np.zeros(p, dtype=bool)
        is_byz[list(w.byz)] = True
        per_group = is_byz.reshape(-1, r).sum(axis=1)
        assert np.array_equal(is_byz[winner], per_group >= (r + 1) // 2)
        seen.append(int(is_byz[winner].sum()))
    # mean of 40 draws of a (nearly) Poisson(3.44) count: standard error 0.29
    assert abs(np.mean(seen) - expected) < 1.0
    assert max(seen) <= 12


def test_detox_lowers_the_error_and_its_growth_with_d():
    """Section 5.3: the l2 norm of the estimate (true mean 0) is smaller after DETOX, and grows
    less from d = 20 to d = 60."""
    err = {}
    for d in (20, 60):
        w = workloads.mean_estimation(d)
        G = w.matrix()
        B = w.detox[0]["B"]
        err[d, "D-median"] = np.linalg.norm(oracle.detox_step(G, w.r, B, "coord_median")[0])
        err[d, "median"] = np.linalg.norm(oracle.coord_median(G))
        assert err[d, "D-median"] < 0.3 * err[d, "median"]
    assert err[60, "D-median"] - err[20, "D-median"] < err[60, "median"] - err[20, "median"]


def test_detox_lowers_the_error_of_the_geometric_median():
    w = workloads.mean_estimation(30, n=44000, q=3991)        # the same Byzantine fraction
    G = w.matrix()
    detox = np.linalg.norm(oracle.detox_step(G, w.r, 25, "geomedian")[0])
    plain = np.linalg.norm(oracle.geomedian(G, 50, 1e-8))
    assert detox < 0.5 * plain
