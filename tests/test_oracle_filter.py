"""Pins for the oracle's majority-vote filter (Section 3; Algorithm 1, filtering step)."""
import numpy as np
import pytest

import oracle
import workloads
from conftest import read_golden


def _rows(*rows):
    return np.array(rows, dtype=np.float32)


def test_honest_majority_returns_base_bit_exactly():
    # Section 3.1: a group with more honest than Byzantine members votes its true gradient.
    for idx, d in ((1, 4096), (2, 3000), (3, 1237), (4, 999), (5, 640)):
        w = workloads.config(idx, d=d)
        G = w.matrix()
        winner, Z = oracle.majority_filter(G, w.r, materialise=True)
        assert (winner >= 0).all()
        assert Z.tobytes() == w.base.tobytes()
        for j, win in enumerate(winner):
            honest = [i for i in range(j * w.r, (j + 1) * w.r) if i not in w.byz]
            assert win == honest[0]          # lowest row of the agreeing set


def test_two_colluding_byzantines_win_a_group_of_three():
    g, b = [1.0, 2.0, 3.0], [9.0, 9.0, 9.0]
    winner, Z = oracle.majority_filter(_rows(b, g, b), 3, materialise=True)
    assert winner.tolist() == [0] and Z[0].tolist() == b


def test_no_majority_gives_zero_vote():
    # "If there is no majority, we set z_j = 0."
    G = _rows([1, 2], [1, 3], [4, 2], [5, 5], [5, 5], [0, 0])
    winner, Z = oracle.majority_filter(G, 3, materialise=True)
    assert winner.tolist() == [-1, 3]
    assert Z[0].tobytes() == np.zeros(2, np.float32).tobytes()
    assert Z[1].tolist() == [5, 5]


def test_piecewise_agreement_is_not_a_majority():
    # rows agree pairwise on different halves: every coordinate has a majority value but no
    # whole vector does
    G = _rows([1, 1, 2, 2], [1, 1, 3, 3], [4, 4, 3, 3])
    assert oracle.majority_filter(G, 3).tolist() == [-1]


def test_equality_is_bitwise():
    pz, nz = np.float32(0.0), np.float32(-0.0)
    G = np.array([[pz], [nz], [nz]], dtype=np.float32)
    assert oracle.majority_filter(G, 3).tolist() == [1]
    G = np.array([[pz], [nz], [np.float32(1)]], dtype=np.float32)
    assert oracle.majority_filter(G, 3).tolist() == [-1]
    # NaNs with the same payload are equal, with different payloads they are not
    a = np.array([0x7FC00000, 0x7FC00000, 0x7FC00001], dtype=np.uint32).view(np.float32)
    assert oracle.majority_filter(a.reshape(3, 1), 3).tolist() == [0]
    b = np.array([0x7FC00000, 0x7FC00002, 0x7FC00001], dtype=np.uint32).view(np.float32)
    assert oracle.majority_filter(b.reshape(3, 1), 3).tolist() == [-1]


def test_difference_in_last_coordinate_only_is_seen():
    d = 1000
    a = np.arange(d, dtype=np.float32)
    b = a.copy(); b[-1] += 1
    c = a.copy(); c[0] += 1
    assert oracle.majority_filter(np.stack([a, b, c]), 3).tolist() == [-1]
    assert oracle.majority_filter(np.stack([b, a, b]), 3).tolist() == [0]


def test_even_r_needs_strict_majority_and_r1_is_identity():
    G = _rows([1], [1], [2], [2])
    assert oracle.majority_filter(G, 4).tolist() == [-1]
    assert oracle.majority_filter(_rows([1], [2], [1], [1]), 4).tolist() == [0]
    assert oracle.majority_filter(G, 2).tolist() == [0, 2]
    assert oracle.majority_filter(G, 1).tolist() == [0, 1, 2, 3]


def test_r_must_divide_n():
    with pytest.raises(oracle.OracleError):
        oracle.majority_filter(_rows([1], [1], [2], [2]), 3)


def test_permuting_members_and_groups():
    w = workloads.config(3, d=257)
    G = w.matrix()
    ref_w, ref_Z = oracle.majority_filter(G, 3, materialise=True)
    rng = np.random.default_rng(5)
    group_order = rng.permutation(w.groups)
    group_rows = np.concatenate([rng.permutation(3) + 3 * g for g in group_order]).astype(np.int32)
    win, Z = oracle.majority_filter(G, 3, group_rows=group_rows, materialise=True)
    assert win.tolist() == ref_w[group_order].tolist()
    assert Z.tobytes() == ref_Z[group_order].tobytes()


def test_strided_rows():
    w = workloads.config(1, d=100)
    G = w.matrix(ld=128)
    assert G.strides[0] == 512
    assert oracle.majority_filter(G, 3).tolist() == oracle.majority_filter(np.ascontiguousarray(G), 3).tolist()


@pytest.mark.parametrize("row", read_golden("expected_byzantine_votes.txt"))
def test_expected_number_of_byzantine_votes(row):
    """Monte-Carlo over uniformly random node partitions against the closed form of Appendix A.1.
    Colluding Byzantine nodes all send the same vector, so a group votes Byzantine exactly when
    they hold its majority."""
    n, q, r, expect = int(row[0]), int(row[1]), int(row[2]), float(row[3])
    rng = np.random.default_rng(n * 1000 + q * 10 + r)
    trials = 20000
    groups = n // r
    total = 0
    sq = 0
    for _ in range(trials):
        perm = rng.permutation(n)                     # perm[slot] = node placed in that slot
        G = np.empty((n, 2), dtype=np.float32)
        slot_group = np.arange(n) // r
        G[:, 0] = slot_group
        G[:, 1] = -slot_group
        G[perm < q] = (-7.0, 7.0)                     # nodes 0..q-1 are the Byzantine ones
        winner = oracle.majority_filter(G, r)
        # a vote is honest iff it equals its group's own value in both coordinates
        bad = int(sum(1 for j, wj in enumerate(winner) if wj < 0 or G[wj, 0] != j or G[wj, 1] != -j))
        total += bad
        sq += bad * bad
    mean = total / trials
    var = max(sq / trials - mean * mean, 1e-12)
    assert abs(mean - expect) < 4.5 * np.sqrt(var / trials) + 1e-9
