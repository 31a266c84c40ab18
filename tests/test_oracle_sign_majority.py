"""Pins for the oracle's signSGD pairing (Section 5.2, setup 4): filter, then coordinate-wise
majority vote inside vote groups and across them."""
import numpy as np
import pytest

import oracle
import workloads


def test_packing_layout():
    X = np.array([[1.0, -2.0, 0.0, -0.5] + [3.0] * 30], dtype=np.float32)      # 34 coordinates
    S = workloads.pack_signs(X)
    assert S.shape == (1, 2)
    assert S[0, 0] == (0xFFFFFFFF & ~0b1010) and S[0, 1] == 0b11               # unused bits zero


def test_no_attack_is_sign_of_summed_signs_by_numpy():
    w = workloads.config(3, d=1000)
    w.byz.clear()
    S = workloads.pack_signs(w.matrix())
    signs = np.where(w.base >= 0, 1, -1)
    out, winner = oracle.sign_majority(S, w.d, 3, 15)          # groups of one vote: plain signSGD vote
    assert (winner == np.arange(15) * 3).all()
    assert (out == np.sign(signs.sum(axis=0))).all()
    out, _ = oracle.sign_majority(S, w.d, 3, 5)                # 5 groups of 3: majority of majorities
    inner = np.sign(signs.reshape(5, 3, -1).sum(axis=1))
    assert (out == np.sign(inner.sum(axis=0))).all()
    out, _ = oracle.sign_majority(S, w.d, 3, 2)                # 7 + 8: even size -> ties give 0
    inner = np.stack([np.sign(signs[:7].sum(axis=0)), np.sign(signs[7:].sum(axis=0))])
    assert (inner[1] == 0).any()
    assert (out == np.sign(inner.sum(axis=0))).all()


def test_constant_attack_is_filtered_and_zero_votes_abstain():
    # Section 5.2's constant attack: Byzantine nodes send all -1
    w = workloads.config(3, d=640)
    X = w.matrix()
    for i in w.byz:
        X[i] = -1.0
    ref, _ = oracle.sign_majority(workloads.pack_signs(np.repeat(w.base, 3, axis=0)), w.d, 3, 5)
    out, winner = oracle.sign_majority(workloads.pack_signs(X), w.d, 3, 5)
    assert (winner >= 0).all() and (out == ref).all()
    # a group without majority abstains: same result as dropping that vote
    X2 = np.repeat(w.base, 3, axis=0)
    X2[0] = -X2[0]; X2[1, :320] = -X2[1, :320]      # group 0: three different sign rows
    out2, winner2 = oracle.sign_majority(workloads.pack_signs(X2), w.d, 3, 5)
    assert winner2[0] == -1
    signs = np.where(w.base >= 0, 1, -1); signs[0] = 0
    inner = np.sign(signs.reshape(5, 3, -1).sum(axis=1))
    assert (out2 == np.sign(inner.sum(axis=0))).all()


def test_vote_permutation_and_brute_force_small():
    rng = np.random.default_rng(3)
    base = rng.standard_normal((6, 70)).astype(np.float32)
    G = np.repeat(base, 5, axis=0)
    G[3] = -G[3]; G[4] = rng.standard_normal(70)                # two Byzantine of five: honest majority
    perm = rng.permutation(6).astype(np.int32)
    out, winner = oracle.sign_majority(workloads.pack_signs(G), 70, 5, 3, vote_perm=perm)
    signs = np.where(base >= 0, 1, -1)[perm]
    inner = np.sign(signs.reshape(3, 2, -1).sum(axis=1))
    assert (out == np.sign(inner.sum(axis=0))).all()
