"""GPU parity: the whole parameter-server step (filter -> block means -> aggregator) on the
five workload shapes, against the oracle pipeline."""
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


def _run(dx, w, spec, ld=None, materialise=True, G=None, group_rows=None, vote_perm=None):
    G = w.matrix() if G is None else G
    kw = {k: v for k, v in spec.items() if k not in ("B", "aggregator")}
    ref_out, ref_w, ref_Zh = oracle.detox_step(G, w.r, spec["B"], spec["aggregator"], group_rows=group_rows,
                                               vote_perm=vote_perm, **kw)
    b = dx.detox_step(dev_matrix(G, ld), w.r, w.q, spec["B"], spec["aggregator"], f=spec.get("f", -1),
                      m=spec.get("m", -1), iters=spec.get("iters", 50), eps=spec.get("eps", 1e-8),
                      group_rows=group_rows, vote_perm=vote_perm, materialise=materialise)
    assert host(b.winner).tolist() == ref_w.tolist()
    if materialise:
        assert host(b.Zhat).tobytes() == ref_Zh.tobytes()
    else:
        assert b.Zhat is None
    got = host(b.out)
    if spec["aggregator"] == "coord_median":
        assert got.tobytes() == ref_out.tobytes()
    elif spec["aggregator"] == "trimmed_mean":
        assert rel_l2(got, ref_out) <= TOL
    else:
        assert rel_l2(got, ref_out) <= TOL
    if spec["aggregator"] == "multikrum":
        ref_sel = oracle.multikrum(ref_Zh, spec["f"], spec["m"])[1]
        assert host(b.selected)[: spec["m"]].tolist() == ref_sel.tolist()
    if spec["aggregator"] == "bulyan":
        ref_sel = oracle.bulyan(ref_Zh, spec["f"])[1]
        assert host(b.selected)[: len(ref_sel)].tolist() == ref_sel.tolist()


@pytest.mark.parametrize("idx,d", [(1, 4096), (2, 1 << 20), (3, 300007), (4, 200003), (5, 100001)])
def test_step_on_each_workload(dx, idx, d):
    w = workloads.config(idx, d=d)
    for spec in w.detox:
        for materialise in (True, False):
            _run(dx, w, spec, materialise=materialise)
            _run(dx, w, spec, ld=(d + 63) // 64 * 64, materialise=materialise)


AGGS = [dict(B=5, aggregator="multikrum", f=1, m=3), dict(B=15, aggregator="multikrum", f=2, m=9),
        dict(B=5, aggregator="coord_median"), dict(B=3, aggregator="coord_median"),
        dict(B=15, aggregator="coord_median"), dict(B=4, aggregator="coord_median"),
        dict(B=7, aggregator="bulyan", f=1), dict(B=15, aggregator="bulyan", f=2),
        dict(B=5, aggregator="geomedian"), dict(B=15, aggregator="geomedian", iters=20),
        dict(B=5, aggregator="trimmed_mean", f=1), dict(B=15, aggregator="trimmed_mean", f=3),
        dict(B=7, aggregator="trimmed_mean", f=-1)]


@pytest.mark.parametrize("spec", AGGS, ids=lambda s: f"{s['aggregator']}-B{s['B']}")
@pytest.mark.parametrize("materialise", [True, False])
def test_step_with_votes_without_majority_and_permutations(dx, spec, materialise):
    """Groups without a majority (zero votes), a Byzantine-majority group, scattered node groups
    and a vote permutation: the one-pass results must be redone exactly where needed."""
    w = workloads.config(3, d=30011)
    G = w.matrix()
    d = w.d
    G[3, d // 2:] += 1; G[5, : d // 2] += 2          # group 1: piecewise agreement only
    G[12] = 7; G[13] = 8; G[14] = 9                  # group 4: three different rows
    G[18] = -3; G[20] = -3                           # group 6: two colluding Byzantine rows
    rng = np.random.default_rng(11)
    _run(dx, w, spec, G=G, materialise=materialise)
    order = rng.permutation(15)
    group_rows = np.concatenate([3 * g + rng.permutation(3) for g in order]).astype(np.int32)
    vote_perm = rng.permutation(15).astype(np.int32)
    _run(dx, w, spec, G=G, materialise=materialise, group_rows=group_rows, vote_perm=vote_perm)
    _run(dx, w, spec, G=G, ld=d + 1, materialise=materialise, vote_perm=vote_perm)


def test_step_derives_f_and_m(dx):
    # q = 5, r = 3: at most 5 // 2 = 2 Byzantine votes survive the filter (Appendix B.1 uses
    # the same count to state Bulyan's requirement 4*2+3 = 11 <= 15)
    w = workloads.config(3, d=20011)
    G = w.matrix()
    Gd = dev_matrix(G)
    ref_out, _, ref_Zh = oracle.detox_step(G, 3, 15, "bulyan", f=2)
    b = dx.detox_step(Gd, 3, 5, 15, "bulyan")
    assert rel_l2(host(b.out), ref_out) <= TOL
    ref_out, _, _ = oracle.detox_step(G, 3, 7, "multikrum", f=2, m=5)     # 7 = 2*2+3 rows: just enough
    b = dx.detox_step(Gd, 3, 5, 7, "multikrum")
    assert rel_l2(host(b.out), ref_out) <= TOL
    # 5 rows admit only f = 1 < 2: refused rather than run with a smaller f (Appendix B.1's requirements)
    with pytest.raises(dx.DetoxError) as err:
        dx.detox_step(Gd, 3, 5, 5, "multikrum")
    assert err.value.code == 2
    with pytest.raises(dx.DetoxError) as err:
        dx.detox_step(Gd, 3, 5, 7, "bulyan")
    assert err.value.code == 2


def test_step_output_ignores_byzantine_content(dx):
    w = workloads.config(3, d=40009)
    spec = w.detox[0]
    a = host(dx.detox_step(dev_matrix(w.matrix()), 3, 5, spec["B"], "multikrum", f=1, m=3).out).copy()
    rng = np.random.default_rng(0)
    for i in list(w.byz):
        w.byz[i] = rng.standard_normal(w.d).astype(np.float32)
    b = host(dx.detox_step(dev_matrix(w.matrix()), 3, 5, spec["B"], "multikrum", f=1, m=3).out)
    assert a.tobytes() == b.tobytes()


def test_no_attack_is_the_plain_mean(dx):
    w = workloads.config(3, d=40009)
    w.byz.clear()
    b = dx.detox_step(dev_matrix(w.matrix()), 3, 0, 5, "multikrum", f=0, m=5)
    assert rel_l2(host(b.out), w.honest_mean()) <= TOL


def test_full_size_resnet18_shape(dx):
    """n = 45, r = 3, q = 5, d = 11,173,962 in the layout the benchmark times (rows padded to a
    multiple of 64 floats): DETOX Multi-Krum and vanilla Multi-Krum against the oracle."""
    w = workloads.config(3)
    G = w.matrix()
    ld = (w.d + 63) // 64 * 64
    Gd = w.to_device(ld=ld)
    spec = w.detox[0]
    ref_out, ref_w, ref_Zh = oracle.detox_step(G, 3, spec["B"], "multikrum", f=spec["f"], m=spec["m"])
    b = dx.detox_step(Gd, 3, 5, spec["B"], "multikrum", f=spec["f"], m=spec["m"])
    assert host(b.winner).tolist() == ref_w.tolist()
    assert host(b.Zhat).tobytes() == ref_Zh.tobytes()
    assert rel_l2(host(b.out), ref_out) <= TOL
    b2 = dx.detox_step(Gd, 3, 5, spec["B"], "multikrum", f=spec["f"], m=spec["m"], materialise=False)
    assert host(b2.out).tobytes() == host(b.out).tobytes()      # the launch configuration bench.py times
    # the one-pass median and trimmed mean (results held back in LDS and registers until a
    # workgroup's last trip): every column
    ref_med = oracle.detox_step(G, 3, spec["B"], "coord_median")[0]
    med = dx.detox_step(Gd, 3, 5, spec["B"], "coord_median", materialise=False)
    assert host(med.out).tobytes() == ref_med.tobytes()
    ref_tm = oracle.detox_step(G, 3, spec["B"], "trimmed_mean", f=1)[0]
    tm = dx.detox_step(Gd, 3, 5, spec["B"], "trimmed_mean", f=1, materialise=False)
    assert rel_l2(host(tm.out), ref_tm) <= TOL
    assert np.abs(host(tm.out) - ref_tm).max() <= 1e-5 * np.abs(ref_tm).max()
    v = w.vanilla[0]
    ref_out, ref_sel, ref_scores = oracle.multikrum(G, v["f"], v["m"])
    out, sel, scores = dx.robust_multikrum(Gd, v["f"], v["m"])
    assert host(sel).tolist() == ref_sel.tolist()
    np.testing.assert_allclose(host(scores), ref_scores, rtol=3e-6)
    assert rel_l2(host(out), ref_out) <= TOL


@pytest.mark.parametrize("r,groups,B,d", [(3, 3, 3, 1_048_577), (3, 3, 3, 7_340_033), (2, 4, 4, 8_400_001),
                                          (5, 5, 5, 3_500_003), (7, 2, 2, 9_000_001)])
def test_one_pass_median_and_trimmed_mean_at_middle_sizes(dx, r, groups, B, d):
    """The one-pass kernels keep a workgroup's results in LDS for its first seven trips and in
    registers for up to twelve more: sizes of 2 to 9 trips per workgroup on a 256-CU chip, with
    a ragged last chunk, every column against the oracle (one group without a majority, so the
    repair pass runs as well)."""
    rng = np.random.default_rng(d)
    base = (rng.standard_normal((groups, d)) * 0.05).astype(np.float32)
    G = np.repeat(base, r, axis=0)
    G[0] = 3.0                                       # a Byzantine row inside group 0
    if r >= 3:
        G[r + 1, d // 3:] += 1.0; G[r + 2, : d // 3] -= 1.0   # group 1: no vector majority
    Gd = dev_matrix(G)
    ref, ref_w, _ = oracle.detox_step(G, r, B, "coord_median")
    got = dx.detox_step(Gd, r, 1, B, "coord_median", materialise=False)
    assert host(got.winner).tolist() == ref_w.tolist()
    assert host(got.out).tobytes() == ref.tobytes()
    ref = oracle.detox_step(G, r, B, "trimmed_mean", f=(B - 1) // 2)[0]
    got = dx.detox_step(Gd, r, 1, B, "trimmed_mean", f=(B - 1) // 2, materialise=False)
    assert np.abs(host(got.out) - ref).max() <= 1e-5 * np.abs(ref).max()


def _sample_columns(d, width=4096, pieces=6, seed=0):
    """Column windows spread over [0, d), including both ends (the ragged tail too) and, where
    d reaches that far, the column at which the averaging kernels start their second launch on
    a 256-CU chip (1536 workgroups x 8 chunks x 1024 columns)."""
    rng = np.random.default_rng(seed)
    starts = [0, d - width] + [int(x) for x in rng.integers(0, d - width, size=pieces - 2)]
    seam = 1536 * 8 * 1024
    if d > seam + width:
        starts.append(seam - width // 2)
    return [(s, s + width) for s in sorted(starts)]


def test_full_size_heavy_tailed_shape(dx):
    """n = 45, r = 3, q = 5, d = 25,000,000 (Student-t gradients, uniform Byzantine rows):
    DETOX median (5 vote groups, one pass) bit-exact on sampled column windows; DETOX Bulyan over
    the 15 votes and vanilla Bulyan over the 45 rows: selections exact (the oracle computes the
    full-size distances), outputs on sampled windows within 1e-5."""
    w = workloads.config(4)
    G = w.matrix()
    Gd = w.to_device()
    wins = _sample_columns(w.d)
    ref_w = oracle.majority_filter(G, 3)
    med = dx.detox_step(Gd, 3, 5, 5, "coord_median", materialise=False)
    assert host(med.winner).tolist() == ref_w.tolist()
    got = host(med.out)
    # also the columns of workgroup 0's trips around the points where the one-pass kernel changes
    # where it keeps its results (LDS up to trip 6, registers up to trip 18, stored at once after)
    trips = [(t << 20, (t << 20) + 4096) for t in (5, 6, 7, 8, 12, 17, 18, 19, 20, 23)]
    for a, b in wins + trips:
        sub = np.ascontiguousarray(G[:, a:b])
        ref = oracle.detox_step(sub, 3, 5, "coord_median")[0]
        assert got[a:b].tobytes() == ref.tobytes()
    # Bulyan over the votes: selection from full-size distances of the 15 honest votes
    votes = np.ascontiguousarray(G[ref_w])
    ref_sel = oracle.bulyan_select(oracle.pairwise_sqdist(votes), 1)
    bul = dx.detox_step(Gd, 3, 5, 15, "bulyan", f=1, materialise=False)
    assert host(bul.selected)[:13].tolist() == ref_sel.tolist()
    got = host(bul.out)
    for a, b in wins:
        ref = oracle.bulyan_trim(np.ascontiguousarray(votes[:, a:b]), ref_sel, 11)
        assert rel_l2(got[a:b], ref) <= TOL
    del votes
    # vanilla Bulyan over all 45 rows
    ref_sel = oracle.bulyan_select(oracle.pairwise_sqdist(G), 5)
    out, sel = dx.robust_bulyan(Gd, 5)
    assert host(sel).tolist() == ref_sel.tolist()
    got = host(out)
    for a, b in wins:
        ref = oracle.bulyan_trim(np.ascontiguousarray(G[:, a:b]), ref_sel, 25)
        assert rel_l2(got[a:b], ref) <= TOL


def test_full_size_105_node_shape(dx):
    """n = 105, r = 5, q = 10 (two per group), d = 25,000,000: DETOX geometric median over 7 block
    means against the full oracle; vanilla coordinate median bit-exact on sampled windows; vanilla
    Multi-Krum selection against full-size oracle distances."""
    w = workloads.config(5)
    G = w.matrix()
    Gd = w.to_device()
    spec = w.detox[0]
    ref_out, ref_w, _ = oracle.detox_step(G, 5, 7, "geomedian", iters=spec["iters"], eps=spec["eps"])
    b = dx.detox_step(Gd, 5, 10, 7, "geomedian", iters=spec["iters"], eps=spec["eps"], materialise=False)
    assert host(b.winner).tolist() == ref_w.tolist()
    assert rel_l2(host(b.out), ref_out) <= TOL
    wins = _sample_columns(w.d)
    got = host(dx.robust_coord_median(Gd))
    for a, c in wins:
        assert got[a:c].tobytes() == oracle.coord_median(np.ascontiguousarray(G[:, a:c])).tobytes()
    v = w.vanilla[1]
    ref_sel, ref_scores = oracle.multikrum_from_dist(oracle.pairwise_sqdist(G), v["f"], v["m"])
    out, sel, scores = dx.robust_multikrum(Gd, v["f"], v["m"])
    assert host(sel).tolist() == ref_sel.tolist()
    np.testing.assert_allclose(host(scores), ref_scores, rtol=3e-6)
    got = host(out)
    for a, c in wins:
        ref = G[ref_sel][:, a:c].astype(np.float64).sum(axis=0) / v["m"]
        assert rel_l2(got[a:c], ref) <= TOL


@pytest.mark.parametrize("d", [1, 2, 3, 5, 63, 64, 255, 257, 1023, 1025])
def test_tiny_dimensions(dx, d):
    """Every entry point on dimensions smaller than one workgroup's columns, including d = 1."""
    w = workloads.config(3, d=d)
    G = w.matrix()
    for materialise in (True, False):
        for spec in (dict(B=5, aggregator="multikrum", f=1, m=3), dict(B=5, aggregator="coord_median"),
                     dict(B=15, aggregator="bulyan", f=2), dict(B=5, aggregator="geomedian", iters=10)):
            _run(dx, w, spec, G=G, materialise=materialise)
    Gd = dev_matrix(G)
    ref_out, ref_sel, _ = oracle.multikrum(G, 5, 40)
    out, sel, _ = dx.robust_multikrum(Gd, 5, 40)
    # at tiny d different honest groups can tie exactly or nearly; compare what is unique
    D = oracle.pairwise_sqdist(G)
    scores = oracle.krum_scores(D, 5)
    assert np.allclose(np.sort(scores[host(sel)]), np.sort(scores[ref_sel]), rtol=1e-5, atol=1e-12)
    # ... and that what is valid holds: 40 different rows, and the output is their mean
    picked = host(sel)
    assert len(set(picked.tolist())) == 40 and picked.min() >= 0 and picked.max() < G.shape[0]
    assert rel_l2(host(out), G[picked].astype(np.float64).sum(axis=0) / 40.0) <= TOL
    assert host(dx.robust_coord_median(Gd)).tobytes() == oracle.coord_median(G).tobytes()


def test_single_group_and_single_row(dx):
    X = workloads.distinct_rows(1, 1, 300)
    assert host(dx.robust_coord_median(dev_matrix(X))).tobytes() == X[0].tobytes()
    assert rel_l2(host(dx.robust_geomedian(dev_matrix(X))), X[0]) <= TOL
    G = np.repeat(X, 3, axis=0)
    b = dx.detox_step(dev_matrix(G), 3, 0, 1, "coord_median")
    assert host(b.winner).tolist() == [0] and host(b.out).tobytes() == X[0].tobytes()
    b = dx.detox_step(dev_matrix(G), 3, 0, 1, "geomedian", materialise=False)
    assert rel_l2(host(b.out), X[0]) <= TOL


ROBUST_BLOCKS = [("multikrum", 2, 2, 3), ("multikrum", 2, 1, -1), ("multikrum", 1, 5, 8), ("multikrum", 3, 1, 2),
                 ("bulyan", 1, 2, -1), ("bulyan", 1, 3, -1), ("bulyan", 2, 1, -1), ("bulyan", 3, 0, -1)]


@pytest.mark.parametrize("a0,B,f,m", ROBUST_BLOCKS)
def test_robust_aggregator_inside_vote_groups(dx, a0, B, f, m):
    """The hierarchy of Section 5.2 (A0 robust, A1 mean), e.g. Multi-Krum on 7 + 8 votes and Bulyan
    on all 15 (Appendix B.1), with a group without majority and a vote permutation."""
    w = workloads.config(3, d=40009)
    rng = np.random.default_rng(B * 10 + f)
    # with and without a group that has no majority (its vote is the zero vector; the Gram matrix
    # formed in the filter pass is then replaced), with and without a vote permutation, on rows
    # that start on 16-byte boundaries and on rows that do not
    for broken, vote_perm, ld in ((True, None, None), (True, rng.permutation(15).astype(np.int32), 40064),
                                  (False, None, 40064), (False, rng.permutation(15).astype(np.int32), 40064),
                                  (False, None, None), (False, None, 40065), (True, None, 40065)):
        G = w.matrix()
        if broken:
            G[12] = 7; G[13] = 8; G[14] = 9
        ref_out, ref_w, ref_blocks, ref_sels = oracle.detox_step_robust_blocks(G, 3, B, a0, f, m, vote_perm=vote_perm)
        for _ in range(1):
            out, winner, blocks, selected = dx.detox_step_robust_blocks(dev_matrix(G, ld), 3, B, a0, f, m, vote_perm=vote_perm)
            assert host(winner).tolist() == ref_w.tolist()
            sel = host(selected)
            for b, rs in enumerate(ref_sels):
                lo = (b * 15) // B
                assert sel[lo: lo + len(rs)].tolist() == rs.tolist()
            if B > 1:
                assert rel_l2(host(blocks), ref_blocks) <= TOL
            assert rel_l2(host(out), ref_out) <= TOL


@pytest.mark.parametrize("groups,r", [(9, 3), (11, 5), (13, 3), (16, 3), (16, 1), (10, 2)])
@pytest.mark.parametrize("aggregator", ["multikrum", "bulyan", "geomedian"])
def test_gram_of_the_votes_formed_in_the_filter_pass(dx, groups, r, aggregator):
    """9 to 16 votes, every vote its own block, block means not materialised: the filter pass
    forms the Gram matrix of the votes on the matrix cores.  Every group has a majority here, so
    those tiles are the ones used (the repair path is covered by the test above); two replicated
    votes must give exactly tied distances, which the selections make visible."""
    import torch
    rng = np.random.default_rng(100 * groups + r)
    d = 70_003
    base = rng.standard_normal((groups, d)).astype(np.float32) * np.float32(0.05)
    base[3] = base[1]                                  # two identical votes: exact ties
    G = np.repeat(base, r, axis=0)
    if r >= 3:
        G[0] = 5.0                                     # one Byzantine member, outvoted
        G[r * 4 + 1] = -5.0
    w = workloads.Workload("votes", groups * r, r, 2, d, base, {})
    f = 1 if groups < 11 else 2
    spec = dict(B=groups, aggregator=aggregator)
    if aggregator == "multikrum":
        spec.update(f=f, m=groups - f - 1)
    if aggregator == "bulyan":
        spec.update(f=f)
    vote_perm = rng.permutation(groups).astype(np.int32)
    for ld, vp in ((None, None), (d + 1, None), ((d + 63) // 64 * 64, vote_perm)):
        _run(dx, w, spec, G=G, ld=ld, materialise=False, vote_perm=vp)
    with dx.trace() as tr:
        dx.detox_step(dev_matrix(G, (d + 3) // 4 * 4), r, 2, groups, aggregator, f=spec.get("f", -1),
                      m=spec.get("m", -1), materialise=False)
        names = [n for n, _ in tr.records()]
    assert "filter_votes_gram" in names and "gram_mfma_bf16x3" not in names


@pytest.mark.parametrize("k", [10, 100, 1000])
@pytest.mark.parametrize("aggregator", ["multikrum", "bulyan", "geomedian"])
def test_step_over_15_votes_with_a_common_offset(dx, aggregator, k):
    """The Gram matrix of the 15 votes formed in the filter pass, on votes that share a component
    k times their spread, with Byzantine members far away: selections as the oracle's."""
    d, sigma = 70_003, 0.03
    rng = np.random.default_rng(k)
    base = (rng.standard_normal((15, d)) * sigma + k * sigma).astype(np.float32)
    G = np.repeat(base, 3, axis=0)
    G[0] = -50.0; G[3 * 7 + 2] = 80.0                    # outvoted
    G[3 * 11] = G[3 * 11 + 1] = 1000.0                   # a Byzantine vote survives the filter
    w = workloads.Workload("votes", 45, 3, 4, d, base, {})
    spec = dict(B=15, aggregator=aggregator)
    if aggregator == "multikrum":
        spec.update(f=2, m=11)
    if aggregator == "bulyan":
        spec.update(f=2)
    _run(dx, w, spec, G=G, ld=(d + 63) // 64 * 64, materialise=False)
    _run(dx, w, spec, G=G, materialise=False, vote_perm=rng.permutation(15).astype(np.int32))


WIDE = [dict(aggregator="multikrum", f=2, m=5), dict(aggregator="bulyan", f=1), dict(aggregator="coord_median"),
        dict(aggregator="geomedian", iters=20), dict(aggregator="trimmed_mean", f=-1)]


@pytest.mark.parametrize("spec", WIDE, ids=lambda s: s["aggregator"])
@pytest.mark.parametrize("n,r,B", [(105, 5, 9), (105, 5, 10), (105, 5, 16), (105, 5, 17), (105, 5, 20), (105, 5, 21),
                                   (45, 3, 9), (45, 3, 12), (96, 3, 32), (96, 3, 31)])
def test_step_with_9_to_32_vote_groups_and_no_block_means_in_memory(dx, spec, n, r, B):
    """Algorithm 2 with any number of vote groups up to 32 while the block means stay out of memory
    (Zhat = NULL): the pass only votes, later kernels (Gram matrix, order statistics, averages)
    re-form the means from the winner rows.  With a group without
    majority (repair path), a Byzantine vote that survives, a vote permutation, and once with the
    means written out as well."""
    import torch
    groups = n // r
    d = 40_003
    rng = np.random.default_rng(1000 * n + B)
    base = (rng.standard_normal((groups, d)) * 0.05 + 0.5).astype(np.float32)
    w = workloads.Workload("wide", n, r, 4, d, base, {})
    spec = dict(spec, B=B)
    if spec["aggregator"] == "trimmed_mean":
        spec["f"] = B // 4
    ld = (d + 63) // 64 * 64
    for broken in (False, True):
        G = np.repeat(base, r, axis=0)
        G[0] = 3.0                                       # outvoted (r >= 3)
        G[r * 2] = G[r * 2 + 1] = -2.0                   # two colluding members: a Byzantine vote (majority only if r = 3)
        if broken:
            for k in range(r):
                G[r * 5 + k] = float(k)                  # group 5: all members differ
        vote_perm = rng.permutation(groups).astype(np.int32)
        _run(dx, w, spec, G=G, ld=ld, materialise=False)
        _run(dx, w, spec, G=G, ld=ld, materialise=False, vote_perm=vote_perm)
    _run(dx, w, spec, G=G, ld=ld, materialise=True, vote_perm=vote_perm)
    # rows off the 16-byte grid (ld = d odd, and ld = 2 mod 4)
    _run(dx, w, spec, G=G, materialise=False, vote_perm=vote_perm)
    _run(dx, w, spec, G=G, ld=d + 3, materialise=False)


@pytest.mark.parametrize("aggregator", ["multikrum", "bulyan", "geomedian"])
@pytest.mark.parametrize("groups", [45, 70, 100])
@pytest.mark.parametrize("broken", [1, 2])
def test_step_over_many_votes_some_without_majority(dx, aggregator, groups, broken):
    """More than 32 votes as one block each (B = n/r), votes kept out of memory: the Gram matrix is
    formed over the winner rows, where a vote without majority stands for the zero vector.  broken = 1:
    a few such votes; broken = 2: two thirds of them, so that the row the Gram kernel centres on
    is itself a zero vector."""
    r, d = 3, 20_011
    rng = np.random.default_rng(groups + broken)
    base = (rng.standard_normal((groups, d)) * 0.05 + 0.5).astype(np.float32)
    G = np.repeat(base, r, axis=0)
    bad = [1, 7, groups - 1] if broken == 1 else [g for g in range(groups) if g % 3 != 0]
    for g in bad:
        for k in range(r):
            G[r * g + k] += float(k + 1)                 # all members differ
    G[r * 3] = 9.0                                        # outvoted
    w = workloads.Workload("many", groups * r, r, 4, d, base, {})
    spec = dict(aggregator=aggregator, B=groups)
    if aggregator == "multikrum":
        spec.update(f=4, m=groups - 6)
    if aggregator == "bulyan":
        spec.update(f=4)
    if aggregator == "geomedian":
        spec.update(iters=20)
    _run(dx, w, spec, G=G, ld=(d + 63) // 64 * 64, materialise=False)
    _run(dx, w, spec, G=G, materialise=False, vote_perm=rng.permutation(groups).astype(np.int32))
