"""Pins for the oracle's vote-group means (Algorithm 2 with A0 = mean)."""
import numpy as np
import pytest

import oracle
import workloads
from conftest import read_golden


def _sizes(votes, B):
    G = np.eye(votes, dtype=np.float32)             # vote j = e_j, so a block mean shows its members
    Zh = oracle.block_mean(G, np.arange(votes, dtype=np.int32), B)
    return [int((row != 0).sum()) for row in Zh], Zh


def test_split_examples_of_appendix_b1():
    for row in read_golden("appendix_b1_examples.txt"):
        if row[0] not in ("uneven_split", "even_split"):
            continue
        votes = int(row[1].split("=")[1]); B = int(row[2].split("=")[1])
        expect = [int(x) for x in row[3:]]
        sizes, Zh = _sizes(votes, B)
        assert sizes == expect
        # consecutive, disjoint, covering
        members = [np.nonzero(r)[0].tolist() for r in Zh]
        assert sum(members, []) == list(range(votes))


def test_blocks_of_one_return_votes_bit_exactly():
    w = workloads.config(2, d=999)
    G = w.matrix()
    G[0, :3] = [-0.0, np.float32(1e-45), np.float32(3.4e38)]
    G[1] = G[0]; G[2] = G[0]
    winner, Z = oracle.majority_filter(G, 3, materialise=True)
    Zh = oracle.block_mean(G, winner, w.groups)
    assert Zh.tobytes() == Z.tobytes()


def test_matches_fp64_mean_and_numpy():
    w = workloads.config(3, d=4001)
    G = w.matrix()
    winner, Z = oracle.majority_filter(G, 3, materialise=True)
    Zh32 = oracle.block_mean(G, winner, 5)
    Zh64 = oracle.block_mean(G, winner, 5, fp64=True)
    ref = Z.astype(np.float64).reshape(5, 3, -1).mean(axis=1)
    np.testing.assert_allclose(Zh64, ref, rtol=1e-15, atol=0)
    rel = np.linalg.norm(Zh32 - ref) / np.linalg.norm(ref)
    assert rel < 1e-6
    # the fp32 version is exactly: two rounded adds, one rounded division
    manual = ((Z[0::3] + Z[1::3]) + Z[2::3]) / np.float32(3)
    assert manual.dtype == np.float32 and Zh32.tobytes() == manual.tobytes()


def test_zero_vote_counts_in_the_denominator():
    G = np.array([[3, 6], [3, 6], [3, 6], [1, 0], [2, 0], [3, 0]], dtype=np.float32)
    winner = oracle.majority_filter(G, 3)
    assert winner.tolist() == [0, -1]
    assert oracle.block_mean(G, winner, 1).tolist() == [[1.5, 3.0]]


def test_no_attack_single_block_is_plain_mean():
    w = workloads.config(5, d=777)
    w.byz.clear()
    G = w.matrix()
    winner = oracle.majority_filter(G, w.r)
    Zh = oracle.block_mean(G, winner, 1, fp64=True)
    np.testing.assert_allclose(Zh[0], w.honest_mean(), rtol=1e-14)
    np.testing.assert_allclose(Zh[0], G.astype(np.float64).mean(axis=0), rtol=1e-12, atol=1e-18)


def test_vote_permutation():
    w = workloads.config(3, d=65)
    G = w.matrix()
    winner = oracle.majority_filter(G, 3)
    perm = np.random.default_rng(1).permutation(15).astype(np.int32)
    Zh = oracle.block_mean(G, winner, 5, vote_perm=perm, fp64=True)
    ref = w.base.astype(np.float64)[perm].reshape(5, 3, -1).mean(axis=1)
    np.testing.assert_allclose(Zh, ref, rtol=1e-15)


def test_bad_arguments():
    G = np.zeros((3, 4), dtype=np.float32)
    with pytest.raises(oracle.OracleError):
        oracle.block_mean(G, np.array([0], dtype=np.int32), 2)      # more blocks than votes
