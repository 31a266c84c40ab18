"""Pins for the oracle's Bulyan (cited rule; Appendix B.1 states count >= 4f+3 and the
per-coordinate-median second stage)."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads
from conftest import read_golden


def _select_by_subsets(D, f):
    count = len(D)
    pool = list(range(count))
    sel = []
    for _ in range(count - 2 * f):
        k = max(len(pool) - f - 2, 1)
        def score(a):
            others = [b for b in pool if b != a]
            if not others:
                return Fraction(0)
            return min(sum(Fraction(D[a][b]) for b in S) for S in itertools.combinations(others, min(k, len(others))))
        best = min(pool, key=lambda a: (score(a), a))
        sel.append(best); pool.remove(best)
    return sel


@pytest.mark.parametrize("count,f", [(7, 1), (8, 1), (11, 2), (5, 0)])
def test_selection_brute_force(count, f):
    for seed in range(5):
        X = workloads.integer_rows(7 * count + seed, count, 5, -5, 5)
        D = oracle.pairwise_sqdist(X)
        assert oracle.bulyan_select(D, f).tolist() == _select_by_subsets(D.tolist(), f)


def _trim_by_subsets(vals, beta):
    """The beta values closest to the median = the beta-subset with the least summed |v - med|."""
    vals = [Fraction(float(v)) for v in vals]
    s = sorted(vals)
    med = s[len(s) // 2] if len(s) % 2 else (s[len(s) // 2 - 1] + s[len(s) // 2]) / 2
    best = min(itertools.combinations(range(len(vals)), beta),
               key=lambda S: sum(abs(vals[i] - med) for i in S))
    return float(sum(vals[i] for i in best) / beta)


@pytest.mark.parametrize("theta,beta", [(5, 3), (7, 3), (9, 5), (6, 2), (13, 11)])
def test_trimmed_mean_brute_force(theta, beta):
    X = workloads.distinct_rows(theta * 31 + beta, theta, 40)
    got = oracle.bulyan_trim(X, np.arange(theta), beta)
    ref = np.array([_trim_by_subsets(X[:, c], beta) for c in range(X.shape[1])])
    np.testing.assert_allclose(got, ref.astype(np.float32), rtol=3e-7, atol=1e-12)


def test_tie_in_closeness_takes_the_lower_value():
    X = np.array([[1], [2], [3], [4], [5]], dtype=np.float32)
    assert oracle.bulyan_trim(X, np.arange(5), 2)[0] == np.float32(2.5)
    assert oracle.bulyan_trim(X, np.arange(5), 1)[0] == np.float32(3.0)
    assert oracle.bulyan_trim(X, np.arange(5), 4)[0] == np.float32(2.5)       # {3,2,4,1}


def test_the_kept_values_are_a_window_around_the_median():
    theta, beta = 13, 11
    X = workloads.distinct_rows(77, theta, 300)
    got = oracle.bulyan_trim(X, np.arange(theta), beta)
    S = np.sort(X.astype(np.float64), axis=0)
    windows = np.stack([S[lo:lo + beta].mean(axis=0) for lo in range(theta - beta + 1)])
    assert (np.abs(windows - got).min(axis=0) < 1e-6 * np.abs(got) + 1e-9).all()


def test_special_cases():
    X = workloads.distinct_rows(9, 9, 200)
    out, sel = oracle.bulyan(X, 0)                       # f = 0: theta = beta = count -> mean
    assert sorted(sel.tolist()) == list(range(9))
    np.testing.assert_allclose(out, X.astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-9)
    row = workloads.distinct_rows(3, 1, 100)
    out, sel = oracle.bulyan(np.repeat(row, 11, axis=0), 2)
    assert out.tobytes() == row[0].tobytes() and sel.tolist() == list(range(7))
    # beta = 1: the coordinate-wise median of the selected rows
    Y = workloads.distinct_rows(10, 7, 150)
    rows = np.array([4, 0, 6, 2, 5], dtype=np.int32)
    assert oracle.bulyan_trim(Y, rows, 1).tobytes() == oracle.coord_median(Y[rows]).tobytes()


def test_requirement_and_permutation():
    mins = {r[0]: int(r[2]) for r in read_golden("appendix_b1_examples.txt") if r[0].endswith("min_count")}
    assert mins["bulyan_min_count"] == 4 * 2 + 3
    with pytest.raises(oracle.OracleError) as e:
        oracle.bulyan(workloads.distinct_rows(1, 10, 8), 2)
    assert e.value.code == oracle.EPRECOND
    X = workloads.distinct_rows(2, 11, 500)
    out, sel = oracle.bulyan(X, 2)
    perm = np.random.default_rng(3).permutation(11)
    out_p, sel_p = oracle.bulyan(X[perm], 2)
    assert [int(perm[i]) for i in sel_p] == sel.tolist()
    assert out_p.tobytes() == out.tobytes()


def test_byzantine_rows_are_trimmed():
    w = workloads.config(4, d=3000)
    G = w.matrix()
    out, sel = oracle.bulyan(G, 5)
    assert np.abs(out).max() < 0.05                     # uniform[-1,1] rows would show up as ~0.5
