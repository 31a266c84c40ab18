"""Pins for the oracle's coordinate-wise median (Section 4; the l1 geometric median)."""
import itertools

import numpy as np
import pytest

import oracle
import workloads


@pytest.mark.parametrize("count", [1, 2, 3, 4, 5, 6, 7, 8, 13, 35, 105])
def test_against_numpy_median(count):
    X = workloads.distinct_rows(11, count, 501)
    got = oracle.coord_median(X)
    ref = np.median(X.astype(np.float64), axis=0)
    if count % 2:
        assert got.tobytes() == ref.astype(np.float32).tobytes()
    else:
        np.testing.assert_allclose(got, ref, rtol=2e-7, atol=1e-30)


@pytest.mark.parametrize("count", [3, 5, 7])
def test_every_permutation_gives_the_same_median(count):
    vals = np.array([3.5, -1.0, 0.0, 7.25, -1.0, 2.0, 9.0][:count], dtype=np.float32)
    ref = None
    for perm in itertools.permutations(range(count)):
        got = oracle.coord_median(vals[list(perm)].reshape(count, 1))[0]
        ref = got if ref is None else ref
        assert got == ref
    below = (vals < ref).sum(); above = (vals > ref).sum()
    assert below <= count // 2 and above <= count // 2 and ref in vals


def test_l1_optimality_and_membership():
    # the median minimises sum_j |x - x_j| per coordinate: at most half the values lie strictly
    # on either side, and for an odd count it is one of the inputs, bit for bit
    X = workloads.integer_rows(3, 9, 2000, -3, 3)        # many ties
    med = oracle.coord_median(X)
    assert ((X < med).sum(axis=0) <= 4).all() and ((X > med).sum(axis=0) <= 4).all()
    assert (X == med).any(axis=0).all()


def test_even_count_is_fp32_midpoint():
    X = np.array([[1.0], [4.0], [2.0], [8.0]], dtype=np.float32)
    assert oracle.coord_median(X)[0] == np.float32(3.0)
    a, b = np.float32(1.0000001), np.float32(1.0000004)
    X = np.array([[a], [b]], dtype=np.float32)
    assert oracle.coord_median(X)[0] == (a + b) * np.float32(0.5)


def test_signed_zero_and_nan_order():
    nz, pz = np.float32(-0.0), np.float32(0.0)
    X = np.array([[pz], [nz], [nz]], dtype=np.float32)
    assert np.signbit(oracle.coord_median(X)[0])
    X = np.array([[pz], [nz], [pz]], dtype=np.float32)
    assert not np.signbit(oracle.coord_median(X)[0])
    nan = np.float32(np.nan)
    # positive NaNs order above +inf: two of five still leave a finite median
    X = np.array([[nan], [1.0], [2.0], [3.0], [nan]], dtype=np.float32)
    assert oracle.coord_median(X)[0] == np.float32(3.0)
    X = np.array([[nan], [1.0], [nan], [3.0], [nan]], dtype=np.float32)
    assert np.isnan(oracle.coord_median(X)[0])


def test_strided_input():
    X = workloads.distinct_rows(2, 5, 96)
    buf = np.zeros((5, 128), dtype=np.float32); buf[:, :96] = X
    assert oracle.coord_median(buf[:, :96]).tobytes() == oracle.coord_median(X).tobytes()
