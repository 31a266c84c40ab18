"""Pins for the oracle's geometric median, argmin_x sum_j ||x - x_j|| (appendix, proof of the
robustness theorem), computed by Weiszfeld's iteration."""
import numpy as np
import pytest
from scipy.optimize import minimize

import oracle
import workloads


def _objective(x, X):
    return np.sqrt(((X.astype(np.float64) - x) ** 2).sum(axis=1)).sum()


def test_fermat_point_of_an_isosceles_triangle():
    # all angles below 120 degrees: the minimiser sees every side under 120 degrees, which for
    # the base (0,0)-(1,0) and apex (0.5, 2) puts it at height tan(30 deg)/2 on the axis
    X = np.array([[0, 0], [1, 0], [0.5, 2.0]], dtype=np.float32)
    out = oracle.geomedian(X, iters=200, eps=1e-12)
    np.testing.assert_allclose(out, [0.5, np.tan(np.pi / 6) / 2], atol=1e-6)


def test_obtuse_triangle_picks_the_vertex():
    # an angle of 120 degrees or more: the minimiser is that vertex
    X = np.array([[0, 0], [10, 1], [-10, 1]], dtype=np.float32)
    out = oracle.geomedian(X, iters=2000, eps=1e-12)
    np.testing.assert_allclose(out, [0, 0], atol=2e-3)


def test_one_dimension_converges_to_the_median():
    X = np.array([[1.0], [2.0], [7.0], [50.0], [3.0]], dtype=np.float32)
    out = oracle.geomedian(X, iters=500, eps=1e-12)
    assert abs(out[0] - 3.0) < 1e-3


def test_one_and_two_points():
    X = workloads.distinct_rows(1, 1, 64)
    assert oracle.geomedian(X, iters=10).tobytes() == X[0].tobytes()
    Y = workloads.distinct_rows(2, 2, 64)
    out = oracle.geomedian(Y, iters=10)
    np.testing.assert_allclose(out, Y.astype(np.float64).mean(axis=0), rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("count,d", [(5, 3), (7, 10), (12, 2)])
def test_against_a_general_minimiser_and_stationarity(count, d):
    X = workloads.distinct_rows(count * d, count, d)
    out, obj = oracle.geomedian(X, iters=300, eps=1e-12, with_objective=True)
    assert (np.diff(obj) <= 1e-12 * obj[0]).all()             # never increases
    res = minimize(_objective, X.astype(np.float64).mean(axis=0), args=(X,), method="BFGS",
                   options=dict(gtol=1e-10))
    assert obj[-1] <= res.fun * (1 + 1e-9)
    np.testing.assert_allclose(out, res.x, atol=2e-4)
    diff = out.astype(np.float64) - X.astype(np.float64)
    grad = (diff / np.linalg.norm(diff, axis=1, keepdims=True)).sum(axis=0)
    assert np.linalg.norm(grad) / count < 1e-4


def test_zero_iterations_is_the_mean_and_first_step_is_weighted():
    X = workloads.distinct_rows(5, 6, 40)
    X64 = X.astype(np.float64)
    mean = X64.mean(axis=0)
    np.testing.assert_allclose(oracle.geomedian(X, iters=0), mean.astype(np.float32), rtol=0, atol=0)
    w = 1.0 / np.linalg.norm(X64 - mean, axis=1)
    step1 = (w[:, None] * X64).sum(axis=0) / w.sum()
    np.testing.assert_allclose(oracle.geomedian(X, iters=1), step1.astype(np.float32), rtol=1e-7)


def test_eps_floors_the_distance():
    # start exactly on a data point (mean of 3 collinear symmetric points is the middle one):
    # its weight is 1/eps, so the iterate stays there
    X = np.array([[-1.0, 0], [0, 0], [1.0, 0]], dtype=np.float32)
    out = oracle.geomedian(X, iters=5, eps=1e-8)
    np.testing.assert_allclose(out, [0, 0], atol=1e-12)


def test_robust_to_a_far_outlier():
    X = workloads.distinct_rows(8, 7, 500, sigma=0.03)
    X[3] = 100.0
    out = oracle.geomedian(X, iters=50)
    assert np.abs(out).max() < 0.2 and np.abs(X.mean(axis=0)).min() > 10
