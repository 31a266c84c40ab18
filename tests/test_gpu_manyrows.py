"""GPU parity for the mean-estimation regime of Section 5.3 (very many short rows): the
row-parallel filter and block means, and the coordinate-wise / geometric median over any number
of rows, element by element against the CPU oracle."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import dev_matrix, host, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dx():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import paper_1907_12205_amd as dx
    dx.lib()
    return dx


def _attacked(rng, groups, r, d):
    """Replicated honest rows with three kinds of damaged groups: one odd member, a colluding
    majority, and members that all differ (no majority)."""
    base = rng.standard_normal((groups, d)).astype(np.float32)
    G = np.repeat(base, r, axis=0)
    hit = rng.choice(groups, size=groups // 6, replace=False)
    for g in hit:
        kind = int(g) % 3
        if kind == 0:
            G[g * r + int(rng.integers(r))] = rng.standard_normal(d).astype(np.float32)
        elif kind == 1 and r >= 3:
            bad = np.full(d, 7.0, dtype=np.float32)
            for k in rng.permutation(r)[: r // 2 + 1]:
                G[g * r + int(k)] = bad
        else:
            for k in range(r):
                G[g * r + k, int(rng.integers(d))] += np.float32(1 + k)   # one coordinate differs
    return G


@pytest.mark.parametrize("r,d,ld", [(11, 100, 100), (11, 20, 24), (3, 37, 37), (5, 130, 131),
                                    (2, 64, 64), (1, 9, 9), (7, 300, 304)])
def test_row_parallel_filter_and_block_means(dx, r, d, ld):
    import torch
    rng = np.random.default_rng(1000 * r + d)
    groups = 1100 + 7 * r
    G = _attacked(rng, groups, r, d)
    ref_w = oracle.majority_filter(G, r)
    assert (ref_w < 0).sum() > 0 or r == 1
    Gd = dev_matrix(G, ld=ld)
    w = dx.detox_majority_filter(Gd, r)
    assert host(w).tolist() == ref_w.tolist()
    perm = rng.permutation(groups).astype(np.int32)
    for B, vp in ((65, None), (groups, None), (1, None), (33, perm)):
        ref = oracle.block_mean(G, ref_w, B, vp)
        vpd = None if vp is None else torch.from_numpy(vp).cuda()
        w2, Zhat = dx.detox_filter_block_mean(Gd, r, B, vote_perm=vpd)
        assert host(w2).tolist() == ref_w.tolist()
        assert host(Zhat).tobytes() == ref.tobytes()
        alone = dx.detox_block_mean(Gd, w2, B, vote_perm=vpd)
        assert host(alone).tobytes() == ref.tobytes()


def test_row_parallel_filter_with_a_group_table(dx):
    import torch
    rng = np.random.default_rng(5)
    groups, r, d = 1300, 5, 48
    G = _attacked(rng, groups, r, d)
    table = rng.permutation(groups * r).astype(np.int32)      # groups of scattered rows
    ref_w = oracle.majority_filter(G, r, table)
    w = dx.detox_majority_filter(dev_matrix(G), r, group_rows=torch.from_numpy(table).cuda())
    assert host(w).tolist() == ref_w.tolist()
    # the winner is the LOWEST row index of the majority value, whatever the order in the table
    same = np.repeat(rng.standard_normal((groups, d)).astype(np.float32), r, axis=0)
    ref_w = oracle.majority_filter(same, r, table[::-1].copy())
    w = dx.detox_majority_filter(dev_matrix(same), r, group_rows=torch.from_numpy(table[::-1].copy()).cuda())
    assert host(w).tolist() == ref_w.tolist()


SPECIAL = np.array([0.0, -0.0, np.inf, -np.inf, np.nan, -np.nan, 1e-45, -1e-45, 3.0, -3.0], dtype=np.float32)


@pytest.mark.parametrize("count,d,ld", [(129, 5, 5), (1000, 20, 20), (1001, 100, 104), (4097, 130, 131),
                                        (64, 3, 3), (2, 70, 70), (1, 4, 4), (50000, 1, 1)])
def test_coord_median_many(dx, count, d, ld):
    rng = np.random.default_rng(count + d)
    X = rng.standard_normal((count, d)).astype(np.float32)
    got = host(dx.robust_coord_median_many(dev_matrix(X, ld=ld)))
    assert got.tobytes() == oracle.coord_median(X).tobytes()
    # heavy ties: few distinct values, so the middle sits inside a run of equal keys
    T = rng.integers(-2, 3, size=(count, d)).astype(np.float32)
    got = host(dx.robust_coord_median_many(dev_matrix(T, ld=ld)))
    assert got.tobytes() == oracle.coord_median(T).tobytes()
    # signed zeros, infinities, NaNs of both signs, denormals: the total order on bit patterns
    S = SPECIAL[rng.integers(0, len(SPECIAL), size=(count, d))]
    got = host(dx.robust_coord_median_many(dev_matrix(S, ld=ld)))
    assert got.tobytes() == oracle.coord_median(S).tobytes()


def test_coord_median_many_agrees_with_the_sorting_network(dx):
    X = workloads.distinct_rows(3, 105, 1000)
    Xd = dev_matrix(X)
    assert host(dx.robust_coord_median_many(Xd)).tobytes() == host(dx.robust_coord_median(Xd)).tobytes()


@pytest.mark.parametrize("count,d,ld,iters", [(500, 20, 20, 50), (5000, 100, 100, 50), (777, 128, 132, 20),
                                              (300, 1, 1, 50), (64, 17, 17, 0), (1, 5, 5, 3),
                                              (20000, 33, 36, 10)])
def test_geomedian_many(dx, count, d, ld, iters):
    rng = np.random.default_rng(7 * count + d)
    X = rng.standard_normal((count, d)).astype(np.float32)
    X[: count // 10] = 50.0 / np.sqrt(d)                      # a cluster of outliers
    ref = oracle.geomedian(X, iters, 1e-8)
    got = host(dx.robust_geomedian_many(dev_matrix(X, ld=ld), iters, 1e-8))
    assert rel_l2(got, ref) <= 1e-5


def test_geomedian_many_floor_on_the_distance(dx):
    """All rows equal: every distance is 0, the weights are 1/eps and the iterate stays put."""
    X = np.tile(np.arange(40, dtype=np.float32), (300, 1))
    got = host(dx.robust_geomedian_many(dev_matrix(X), 5, 1e-8))
    assert rel_l2(got, oracle.geomedian(X, 5, 1e-8)) <= 1e-6
    assert np.array_equal(got, X[0])


def test_many_argument_errors(dx):
    import torch
    X = torch.zeros((300, 129), device="cuda:0")
    with pytest.raises(dx.DetoxError) as e:
        dx.robust_geomedian_many(X)
    assert e.value.code == 1
    small = torch.empty(256, dtype=torch.uint8, device="cuda:0")
    with pytest.raises(dx.DetoxError) as e:
        dx.robust_coord_median_many(X, ws=small)
    assert e.value.code == 3
    with pytest.raises(dx.DetoxError) as e:
        dx.robust_geomedian_many(X[:, :100], ws=small)
    assert e.value.code == 3


@pytest.mark.parametrize("d", [20, 100])
def test_mean_estimation_at_full_size(dx, d):
    """n = 220000, r = 11, q = floor(e^11 / 3) = 19958 (Section 5.3), every output compared."""
    import torch
    w = workloads.mean_estimation(d)
    G = w.matrix()
    Gd = torch.from_numpy(G).cuda()
    ref_w = oracle.majority_filter(G, w.r)
    B = w.detox[0]["B"]
    ref_med, _, ref_Z = oracle.detox_step(G, w.r, B, "coord_median")
    b = dx.detox_step(Gd, w.r, w.q, B, "coord_median")
    assert host(b.winner).tolist() == ref_w.tolist()
    assert host(b.Zhat).tobytes() == ref_Z.tobytes()
    assert host(b.out).tobytes() == ref_med.tobytes()
    ref_gm, _, _ = oracle.detox_step(G, w.r, B, "geomedian")
    b = dx.detox_step(Gd, w.r, w.q, B, "geomedian")
    assert rel_l2(host(b.out), ref_gm) <= 1e-5
    # the same aggregators over all 220000 rows
    got = host(dx.robust_coord_median_many(Gd))
    assert got.tobytes() == oracle.coord_median(G).tobytes()
    ref = oracle.geomedian(G, 50, 1e-8)
    got_gm = host(dx.robust_geomedian_many(Gd, 50, 1e-8))
    assert rel_l2(got_gm, ref) <= 1e-5
    # the claim of Section 5.3: the estimate after DETOX is much closer to the true mean (0)
    assert np.linalg.norm(host(b.out)) < 0.3 * np.linalg.norm(got_gm)
    assert np.linalg.norm(ref_med) < 0.3 * np.linalg.norm(got)


def test_largest_number_of_node_groups(dx):
    """n/r = 65535 is the limit of this build; one more is refused before anything is launched."""
    import torch
    rng = np.random.default_rng(65535)
    groups, r, d = 65535, 2, 5
    base = rng.standard_normal((groups, d)).astype(np.float32)
    G = np.repeat(base, r, axis=0)
    odd = rng.choice(groups, size=500, replace=False)
    G[odd * r + 1, 2] += 1.0                                   # two members that differ: no majority
    ref_w = oracle.majority_filter(G, r)
    assert (ref_w < 0).sum() == 500
    Gd = dev_matrix(G)
    w, Zhat = dx.detox_filter_block_mean(Gd, r, 101)
    assert host(w).tolist() == ref_w.tolist()
    assert host(Zhat).tobytes() == oracle.block_mean(G, ref_w, 101).tobytes()
    too_many = torch.zeros(((groups + 1) * r, d), device="cuda:0")
    with pytest.raises(dx.DetoxError) as e:
        dx.detox_majority_filter(too_many, r)
    assert e.value.code == 1
