"""Pins for the oracle's coordinate-wise trimmed mean (Section 4, third aggregator; alpha = 1/4)."""
import itertools

import numpy as np
import pytest
from scipy.stats import trim_mean

import oracle
import workloads


@pytest.mark.parametrize("count,g", [(5, 1), (8, 2), (9, 2), (15, 3), (45, 11), (105, 26), (7, 0)])
def test_against_scipy_trim_mean(count, g):
    X = workloads.distinct_rows(count + g, count, 400)
    got = oracle.trimmed_mean(X, g)
    ref = trim_mean(X.astype(np.float64), g / count + 1e-12, axis=0)     # cuts floor(p*n) per end
    np.testing.assert_allclose(got, ref, rtol=2e-7, atol=1e-12)


def test_special_cases():
    X = workloads.distinct_rows(3, 9, 300)
    np.testing.assert_allclose(oracle.trimmed_mean(X, 0), X.astype(np.float64).mean(axis=0), rtol=2e-7, atol=1e-12)
    assert oracle.trimmed_mean(X, 4).tobytes() == oracle.coord_median(X).tobytes()      # one value left
    Y = workloads.distinct_rows(4, 8, 300)
    np.testing.assert_allclose(oracle.trimmed_mean(Y, 3), oracle.coord_median(Y), rtol=2e-7)   # two left
    with pytest.raises(oracle.OracleError):
        oracle.trimmed_mean(Y, 4)


def test_brute_force_and_permutations():
    vals = np.array([3.0, -1.0, 10.0, 2.0, 2.0, -7.0, 0.5], dtype=np.float32)
    ref = None
    for perm in itertools.permutations(range(7)):
        got = oracle.trimmed_mean(vals[list(perm)].reshape(7, 1), 2)[0]
        ref = got if ref is None else ref
        assert got == ref
    assert ref == np.float32((0.5 + 2.0 + 2.0) / 3)


def test_bounded_by_honest_values_under_attack():
    # with g >= number of outliers the result stays inside the range of the honest values
    X = workloads.distinct_rows(9, 9, 500, sigma=0.03)
    X[2] = 1e6; X[5] = -1e6
    out = oracle.trimmed_mean(X, 2)
    honest = np.delete(X, [2, 5], axis=0)
    assert (out <= honest.max(axis=0)).all() and (out >= honest.min(axis=0)).all()


def test_step_with_alpha_one_quarter():
    w = workloads.config(5, d=999)          # 21 votes, all honest
    out, _, Zh = oracle.detox_step(w.matrix(), 5, 7, "trimmed_mean", f=-1)      # floor(7/4) = 1 per end
    S = np.sort(Zh.astype(np.float64), axis=0)
    np.testing.assert_allclose(out, S[1:6].mean(axis=0), rtol=2e-7, atol=1e-12)
