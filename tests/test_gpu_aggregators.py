"""GPU parity: robust aggregators against the CPU oracle.  Selections, medians: bit-exact.
Means and geometric median: relative L2 error at most 1e-5."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import dev_matrix, host, rel_l2

pytestmark = pytest.mark.gpu
TOL = 1e-5


@pytest.fixture(scope="module")
def dx():
    import torch
    assert torch.cuda.is_available()
    import paper_1907_12205_amd as dx
    return dx


MEDIAN_COUNTS = [1, 2, 3, 4, 5, 6, 7, 8, 9, 13, 15, 16, 17, 21, 24, 25, 32, 35, 45, 56, 57, 64, 100, 105, 128]


@pytest.mark.parametrize("count", MEDIAN_COUNTS)
def test_coord_median(dx, count):
    d = 3001 if count > 32 else 10007
    X = workloads.distinct_rows(count, count, d)
    X[:, 5] = 0.0; X[: count // 2, 5] = -0.0           # signed zeros
    X[0, 9] = np.nan; X[-1, 11] = np.inf
    X[:, 17] = X[0, 17]                                # all equal
    ref = oracle.coord_median(X)
    for ld, off in ((None, 0), ((d + 63) // 64 * 64, 0), (None, 1)):
        got = host(dx.robust_coord_median(dev_matrix(X, ld, off)))
        assert got.tobytes() == ref.tobytes(), (count, ld, off)


def test_coord_median_integer_ties(dx):
    X = workloads.integer_rows(5, 9, 5000, -2, 2)
    assert host(dx.robust_coord_median(dev_matrix(X))).tobytes() == oracle.coord_median(X).tobytes()


SQDIST_COUNTS = [1, 2, 5, 7, 8, 9, 15, 16, 17, 32, 33, 45, 48, 64, 70, 83, 96, 105, 112, 113, 128]


@pytest.mark.parametrize("count", SQDIST_COUNTS)
def test_pairwise_sqdist(dx, count):
    d = 20011
    X = workloads.distinct_rows(1000 + count, count, d, sigma=0.03)
    ref = oracle.pairwise_sqdist(X)
    tol = 1e-12 if count <= 8 else 2e-6
    for ld, off in ((None, 0), ((d + 63) // 64 * 64, 0), (None, 1)):
        D = host(dx.robust_pairwise_sqdist(dev_matrix(X, ld, off)))
        assert (D == D.T).all() and (np.diag(D) == 0).all()
        assert np.abs(D - ref).max() <= tol * ref.max() + 1e-300, (count, ld, off)


@pytest.mark.parametrize("count", [9, 33, 105, 128])
@pytest.mark.parametrize("d", [1, 3, 31, 32, 33, 63, 64, 65, 97, 1000, 1024])
def test_pairwise_sqdist_on_very_short_rows(dx, count, d):
    """Up to 1024 columns the Gram matrix of more than 8 rows is formed in fp64."""
    X = workloads.distinct_rows(count + d, count, d, sigma=0.03, mean=0.5)
    ref = oracle.pairwise_sqdist(X)
    for ld in (None, (d + 63) // 64 * 64, d + 1):
        D = host(dx.robust_pairwise_sqdist(dev_matrix(X, ld, 0)))
        assert (D == D.T).all() and (np.diag(D) == 0).all()
        assert np.abs(D - ref).max() <= 1e-11 * ref.max() + 1e-300, (count, d, ld)


@pytest.mark.parametrize("count", [9, 33, 105, 128])
@pytest.mark.parametrize("d", [1025, 1031, 1055, 1056, 1057, 1087, 1088, 1089, 1121])
def test_pairwise_sqdist_on_the_shortest_rows_of_the_matrix_core_kernels(dx, count, d):
    """Just above 1024 columns: few tiles per wavefront, ragged last tiles of every length class."""
    X = workloads.distinct_rows(count + d, count, d, sigma=0.03, mean=0.5)
    ref = oracle.pairwise_sqdist(X)
    for ld in (None, (d + 63) // 64 * 64):
        D = host(dx.robust_pairwise_sqdist(dev_matrix(X, ld, 0)))
        assert np.abs(D - ref).max() <= 2e-6 * ref.max() + 1e-300, (count, d, ld)


def test_geomedian_in_one_dimension_when_an_iterate_nearly_hits_a_row(dx):
    """Nine values on a line for which the second Weiszfeld iterate lands 2e-6 from one of them
    (the values' spread is 0.06): the weight of that value is the reciprocal of a distance that
    is the small difference of Gram entries, which the fp64 Gram matrix of short rows resolves."""
    z = np.array([0.0186256, -0.00200855, -0.04061466, -0.01330629, 0.0087603, 0.00847142,
                  0.00571794, 0.00715502, 0.01970924], dtype=np.float32).reshape(9, 1)
    for iters in (2, 3, 7, 50):
        ref = oracle.geomedian(z, iters=iters, eps=1e-8)
        got = host(dx.robust_geomedian(dev_matrix(z), iters=iters, eps=1e-8))
        assert abs(float(got[0]) - float(ref[0])) <= 1e-6 * abs(float(ref[0])), (iters, got, ref)


@pytest.mark.parametrize("count", [6, 15, 45, 105])
def test_identical_rows_give_exact_zero_and_equal_distances(dx, count):
    r = 3
    base = workloads.distinct_rows(7, count // r, 9001, sigma=0.03)
    X = np.repeat(base, r, axis=0)
    D = host(dx.robust_pairwise_sqdist(dev_matrix(X)))
    for a in range(X.shape[0]):
        for b in range(X.shape[0]):
            if a // r == b // r:
                assert D[a, b] == 0.0
                assert (D[a] == D[b]).all()
            else:
                assert D[a, b] > 0


def test_integer_rows_distances_are_exact(dx):
    for count in (5, 12, 45):
        X = workloads.integer_rows(count, count, 4000)
        D = host(dx.robust_pairwise_sqdist(dev_matrix(X)))
        assert (D == oracle.pairwise_sqdist(X)).all()


def _multikrum_case(dx, X, f, m):
    ref_out, ref_sel, ref_scores = oracle.multikrum(X, f, m)
    out, sel, scores = dx.robust_multikrum(dev_matrix(X), f, m)
    assert host(sel).tolist() == ref_sel.tolist()
    np.testing.assert_allclose(host(scores), ref_scores, rtol=3e-6, atol=1e-300)
    assert rel_l2(host(out), ref_out) <= TOL
    return ref_sel


@pytest.mark.parametrize("count,f,m", [(5, 1, 3), (5, 1, 1), (7, 2, 5), (8, 0, 8), (15, 2, 13),
                                        (16, 6, 1), (45, 5, 40), (45, 21, 3), (105, 10, 95), (128, 40, 7)])
def test_multikrum_distinct_rows(dx, count, f, m):
    X = workloads.distinct_rows(count * 7 + f, count, 30011, sigma=0.03)
    X[count // 2] += 0.01                                # one row clearly farther than the rest
    _multikrum_case(dx, X, f, m)


@pytest.mark.parametrize("idx,d", [(2, 70001), (3, 50003), (5, 20002)])
def test_multikrum_vanilla_on_replicated_matrix(dx, idx, d):
    # replicas have exactly tied scores: the tie rule (lower row first) must hold on the GPU too
    w = workloads.config(idx, d=d)
    G = w.matrix()
    for spec in w.vanilla:
        if spec["aggregator"] != "multikrum":
            continue
        sel = _multikrum_case(dx, G, spec["f"], spec["m"])
        assert not (set(sel.tolist()) & set(w.byz))


def test_multikrum_integer_rows_with_ties(dx):
    for seed in range(5):
        X = workloads.integer_rows(seed, 9, 64, -2, 2)
        _multikrum_case(dx, X, 2, 4)


@pytest.mark.parametrize("count,f", [(7, 1), (15, 1), (15, 3), (11, 2), (45, 5), (45, 10), (16, 0), (105, 10), (128, 31)])
def test_bulyan(dx, count, f):
    X = workloads.distinct_rows(count * 3 + f, count, 20011, sigma=0.03)
    ref_out, ref_sel = oracle.bulyan(X, f)
    out, sel = dx.robust_bulyan(dev_matrix(X), f)
    assert host(sel).tolist() == ref_sel.tolist()
    assert rel_l2(host(out), ref_out) <= TOL


def test_bulyan_on_replicated_matrix_and_heavy_tails(dx):
    w = workloads.config(4, d=30011)
    G = w.matrix()
    ref_out, ref_sel = oracle.bulyan(G, 5)
    out, sel = dx.robust_bulyan(dev_matrix(G), 5)
    assert host(sel).tolist() == ref_sel.tolist()
    assert rel_l2(host(out), ref_out) <= TOL


@pytest.mark.parametrize("d", [1_600_003, 2_000_003, 3_145_727, 4_000_037, 6_291_456, 6_300_001])
def test_averages_of_many_rows_at_middle_sizes(dx, d):
    """Mean of 20 selected rows and weighted sum of 24 rows where the averaging kernel holds 2, 4
    or 8 chunks of 1024 columns per workgroup back before it stores them (d from 1.6M on, on a
    256-CU chip), with a ragged last chunk and without one."""
    X = workloads.distinct_rows(77, 24, d, sigma=0.03)
    X[3] += 0.05
    ref_out, ref_sel, _ = oracle.multikrum(X, 2, 20)
    Xd = dev_matrix(X)
    out, sel, _ = dx.robust_multikrum(Xd, 2, 20)
    assert host(sel).tolist() == ref_sel.tolist()
    assert rel_l2(host(out), ref_out) <= TOL
    edges = np.r_[0:2048, d - 2048:d]
    np.testing.assert_allclose(host(out)[edges], ref_out[edges], rtol=1e-5, atol=1e-9)
    ref = oracle.geomedian(X, iters=3, eps=1e-8)
    got = host(dx.robust_geomedian(Xd, iters=3, eps=1e-8))
    assert rel_l2(got, ref) <= TOL
    np.testing.assert_allclose(got[edges], ref[edges], rtol=1e-4, atol=1e-8)


@pytest.mark.parametrize("count", [1, 2, 3, 7, 8, 9, 21, 45])
def test_geomedian(dx, count):
    X = workloads.distinct_rows(50 + count, count, 20011, sigma=0.03)
    if count >= 7:
        X[1] = 100.0                                     # a far outlier
    for iters in (0, 1, 50):
        ref = oracle.geomedian(X, iters=iters, eps=1e-8)
        got = host(dx.robust_geomedian(dev_matrix(X), iters=iters, eps=1e-8))
        assert rel_l2(got, ref) <= TOL, (count, iters)


def test_aggregators_accept_unaligned_rows(dx):
    X = workloads.distinct_rows(3, 15, 5003, sigma=0.03)
    ref_out, ref_sel, _ = oracle.multikrum(X, 2, 13)
    ref_b, ref_bsel = oracle.bulyan(X, 1)
    ref_g = oracle.geomedian(X)
    for ld, off in ((5003, 1), (5004, 2), (5003, 0)):
        Xd = dev_matrix(X, ld, off)
        out, sel, _ = dx.robust_multikrum(Xd, 2, 13)
        assert host(sel).tolist() == ref_sel.tolist() and rel_l2(host(out), ref_out) <= TOL
        out, sel = dx.robust_bulyan(Xd, 1)
        assert host(sel).tolist() == ref_bsel.tolist() and rel_l2(host(out), ref_b) <= TOL
        assert rel_l2(host(dx.robust_geomedian(Xd)), ref_g) <= TOL


@pytest.mark.parametrize("count,g", [(1, 0), (3, 1), (5, 1), (5, 0), (8, 2), (8, 3), (15, 3), (16, 4), (25, 6),
                                     (45, 11), (57, 14), (105, 26), (128, 32), (128, 63)])
def test_trimmed_mean(dx, count, g):
    d = 3001 if count > 32 else 10007
    X = workloads.distinct_rows(count + 77, count, d)
    X[:, 5] = 0.0; X[: count // 2, 5] = -0.0
    X[:, 17] = X[0, 17]
    ref = oracle.trimmed_mean(X, g)
    for ld, off in ((None, 0), ((d + 63) // 64 * 64, 0), (None, 1)):
        got = host(dx.robust_trimmed_mean(dev_matrix(X, ld, off), g))
        assert rel_l2(got, ref) <= TOL
        if 2 * g == count - 1:          # a single value survives: the median, bit for bit
            assert got.tobytes() == oracle.coord_median(X).tobytes()


# ---- rows that share a component much larger than their spread ------------------------------------
# Honest gradients are a common gradient plus noise (the case Krum is defined for); distances do not
# depend on the common part, and neither may the fp32 Gram path (more than 8 rows).
OFFSET_COUNTS = [9, 16, 45, 105]
OFFSETS = [10, 100, 1000]       # common component, in units of the spread


@pytest.mark.parametrize("k", OFFSETS)
@pytest.mark.parametrize("count", OFFSET_COUNTS)
def test_pairwise_sqdist_with_a_common_offset(dx, count, k):
    d, sigma = 20011, 0.03
    X = workloads.distinct_rows(2000 + count, count, d, sigma=sigma, mean=k * sigma)
    ref = oracle.pairwise_sqdist(X)
    for ld, off in ((None, 0), ((d + 63) // 64 * 64, 0), (None, 1)):
        D = host(dx.robust_pairwise_sqdist(dev_matrix(X, ld, off)))
        assert (D == D.T).all() and (np.diag(D) == 0).all()
        assert np.abs(D - ref).max() <= 2e-6 * ref.max(), (count, k, ld, off)


@pytest.mark.parametrize("k", OFFSETS)
@pytest.mark.parametrize("count", OFFSET_COUNTS)
def test_selections_and_geomedian_with_a_common_offset(dx, count, k):
    d, sigma = 30011, 0.03
    X = workloads.distinct_rows(3000 + count, count, d, sigma=sigma, mean=k * sigma)
    X[count // 2] += np.float32(0.01)
    f = (count - 3) // 4
    _multikrum_case(dx, X, f, count - f)
    ref_out, ref_sel = oracle.bulyan(X, f)
    out, sel = dx.robust_bulyan(dev_matrix(X), f)
    assert host(sel).tolist() == ref_sel.tolist()
    assert rel_l2(host(out), ref_out) <= TOL
    X[1] = np.float32(-5.0)                              # a far outlier as well
    ref = oracle.geomedian(X, iters=30, eps=1e-8)
    got = host(dx.robust_geomedian(dev_matrix(X), iters=30, eps=1e-8))
    assert rel_l2(got, ref) <= TOL


@pytest.mark.parametrize("count", OFFSET_COUNTS)
def test_selection_does_not_change_under_translation(dx, count):
    """GPU twin of the oracle's translation pin: adding one vector to every row (exactly, here:
    small integers plus multiples of 1/8) leaves Multi-Krum's and Bulyan's selections unchanged."""
    d = 8192
    X = workloads.integer_rows(count, count, d, -8, 8) / np.float32(8.0)
    f = (count - 3) // 4
    sel0 = host(dx.robust_multikrum(dev_matrix(X), f, count - f)[1]).tolist()
    bul0 = host(dx.robust_bulyan(dev_matrix(X), f)[1]).tolist()
    assert sel0 == oracle.multikrum(X, f, count - f)[1].tolist()
    assert bul0 == oracle.bulyan(X, f)[1].tolist()
    shift = (workloads.integer_rows(99, 1, d, -4096, 4096) / np.float32(8.0))[0]
    Y = X + shift                                         # exact in fp32
    assert ((Y - shift) == X).all()
    assert host(dx.robust_multikrum(dev_matrix(Y), f, count - f)[1]).tolist() == sel0
    assert host(dx.robust_bulyan(dev_matrix(Y), f)[1]).tolist() == bul0


@pytest.mark.parametrize("bad", ["far", "nan", "inf"])
@pytest.mark.parametrize("count", [15, 45])
def test_reference_row_is_not_taken_from_the_outliers(dx, count, bad):
    """Row 0 (and a few more) far away, NaN or infinite while the others share a large common
    component: the distances among the clean rows must keep their accuracy."""
    d, sigma = 20011, 0.03
    X = workloads.distinct_rows(4000 + count, count, d, sigma=sigma, mean=1000 * sigma)
    nbad = max(1, count // 5)
    for i in range(nbad):
        X[2 * i] = {"far": np.float32(-100.0 * (i + 1)), "nan": np.float32(np.nan), "inf": np.float32(np.inf)}[bad]
    clean = [i for i in range(count) if not (i % 2 == 0 and i // 2 < nbad)]
    ref = oracle.pairwise_sqdist(X)
    D = host(dx.robust_pairwise_sqdist(dev_matrix(X)))
    sub, rsub = D[np.ix_(clean, clean)], ref[np.ix_(clean, clean)]
    assert np.abs(sub - rsub).max() <= 2e-6 * rsub.max()
    if bad == "far":
        assert np.abs(D - ref).max() <= 2e-6 * ref.max()
        _multikrum_case(dx, X, nbad, count - nbad - 2)
