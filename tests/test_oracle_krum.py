"""Pins for the oracle's pairwise distances and Multi-Krum (Section 4, "Improved speed";
Appendix B.1 for the requirement count >= 2f+3)."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
from scipy.spatial.distance import cdist

import oracle
import workloads
from conftest import read_golden


def test_distances_against_scipy_and_exact_integers():
    X = workloads.distinct_rows(4, 9, 70001, sigma=0.03)     # spans two 65536-coordinate chunks
    D = oracle.pairwise_sqdist(X)
    ref = cdist(X.astype(np.float64), X.astype(np.float64), "sqeuclidean")
    np.testing.assert_allclose(D, ref, rtol=1e-12, atol=0)
    assert (np.diag(D) == 0).all() and (D == D.T).all()
    Xi = workloads.integer_rows(8, 6, 1000)
    Di = oracle.pairwise_sqdist(Xi)
    exact = ((Xi[:, None, :].astype(np.int64) - Xi[None, :, :].astype(np.int64)) ** 2).sum(-1)
    assert (Di == exact).all()


def test_identical_rows_have_zero_distance():
    w = workloads.config(2, d=5000)
    D = oracle.pairwise_sqdist(w.matrix())
    for i in range(w.n):
        for j in range(w.n):
            same = i // 3 == j // 3 and i not in w.byz and j not in w.byz
            assert (D[i, j] == 0) == (same or i == j)


def _krum_by_subsets(D, f, m):
    """Definition by enumeration: score(a) = min over (count-f-2)-subsets of the others of the
    summed distance; then pick the m best one at a time, lower index on ties."""
    count = len(D)
    k = count - f - 2
    scores = []
    for a in range(count):
        others = [b for b in range(count) if b != a]
        scores.append(min(sum(Fraction(D[a][b]) for b in S) for S in itertools.combinations(others, k)))
    left = list(range(count))
    sel = []
    for _ in range(m):
        best = min(left, key=lambda a: (scores[a], a))
        sel.append(best); left.remove(best)
    return scores, sel


@pytest.mark.parametrize("count,f", [(5, 1), (6, 1), (7, 2), (7, 0), (8, 2), (9, 3)])
def test_multikrum_brute_force(count, f):
    for seed in range(6):
        X = workloads.integer_rows(100 * count + seed, count, 4, -6, 6)
        D = oracle.pairwise_sqdist(X)
        for m in (1, 2, count - f):
            scores, sel = _krum_by_subsets(D.tolist(), f, m)
            out, got_sel, got_scores = oracle.multikrum(X, f, m)
            assert got_scores.tolist() == [float(s) for s in scores]
            assert got_sel.tolist() == sel
            mean = X[sel].astype(np.float64).sum(axis=0) / m
            np.testing.assert_allclose(out, mean.astype(np.float32), rtol=0, atol=0)


def test_hand_example_on_a_line():
    g = {r[0]: r[1:] for r in read_golden("krum_hand_example.txt")}
    X = np.array([[float(v)] for v in g["points"]], dtype=np.float32)
    out1, sel1, scores = oracle.multikrum(X, 1, 1)
    assert scores.tolist() == [float(v) for v in g["scores"]]
    assert sel1.tolist() == [int(v) for v in g["selected_m1"]] and out1[0] == X[sel1[0], 0]
    out3, sel3, _ = oracle.multikrum(X, 1, 3)
    assert sel3.tolist() == [int(v) for v in g["selected_m3"]]
    assert out3[0] == np.float32(float(g["mean_m3"][0]))


def test_requirements():
    mins = {r[0]: int(r[2]) for r in read_golden("appendix_b1_examples.txt") if r[0].endswith("min_count")}
    assert mins["multikrum_min_count"] == 2 * 2 + 3
    X = workloads.distinct_rows(1, 6, 10)
    with pytest.raises(oracle.OracleError) as e:
        oracle.multikrum(X, 2, 1)                       # 6 < 2*2+3
    assert e.value.code == oracle.EPRECOND
    oracle.multikrum(workloads.distinct_rows(1, 7, 10), 2, 1)
    with pytest.raises(oracle.OracleError):
        oracle.multikrum(X, 1, 6)                       # m > count - f


def test_all_rows_identical_and_plain_mean():
    row = workloads.distinct_rows(3, 1, 300)
    X = np.repeat(row, 7, axis=0)
    out, sel, scores = oracle.multikrum(X, 2, 3)
    assert out.tobytes() == row[0].tobytes() and sel.tolist() == [0, 1, 2] and (scores == 0).all()
    Y = workloads.distinct_rows(5, 9, 300)
    out, sel, _ = oracle.multikrum(Y, 0, 9)             # f = 0, m = count: the average
    assert sorted(sel.tolist()) == list(range(9))
    np.testing.assert_allclose(out, Y.astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-9)


def test_translation_and_permutation():
    X = workloads.integer_rows(21, 9, 50)
    _, sel, scores = oracle.multikrum(X, 2, 4)
    shift = np.arange(50, dtype=np.float32) * 4 - 64
    _, sel_t, scores_t = oracle.multikrum(X + shift, 2, 4)
    assert sel_t.tolist() == sel.tolist() and scores_t.tolist() == scores.tolist()
    Y = workloads.distinct_rows(22, 9, 400)             # no ties: selection is a set property
    _, sel, _ = oracle.multikrum(Y, 2, 4)
    perm = np.random.default_rng(0).permutation(9)
    _, sel_p, _ = oracle.multikrum(Y[perm], 2, 4)
    assert [int(perm[i]) for i in sel_p] == sel.tolist()


def test_outliers_are_never_selected():
    w = workloads.config(2, d=20000)
    G = w.matrix()
    _, sel, _ = oracle.multikrum(G, 2, 13)
    assert not (set(sel.tolist()) & set(w.byz))


def test_nan_scores_rank_last():
    D = np.array([[0, 1, 2, 3, 4], [1, 0, 1, 2, 3], [2, 1, 0, 1, 2], [3, 2, 1, 0, 1], [4, 3, 2, 1, 0]], dtype=np.float64)
    D[1, :] = np.nan; D[:, 1] = np.nan; D[1, 1] = 0
    sel, scores = oracle.multikrum_from_dist(D, 1, 4)
    assert np.isnan(scores[1]) and sel.tolist()[-1] != 1 and 1 not in sel.tolist()
