"""GPU parity: DETOX paired with signSGD (bit-packed signs, two levels of coordinate-wise
majority vote) against the CPU oracle, bit for bit."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dx():
    import torch
    assert torch.cuda.is_available()
    import paper_1907_12205_amd as dx
    return dx


def _run(dx, S, d, r, B, vote_perm=None, ldw=None):
    import torch
    ref, ref_w = oracle.sign_majority(S, d, r, B, vote_perm=vote_perm)
    n, words = S.shape
    ldw = words if ldw is None else ldw
    buf = torch.zeros((n, ldw), dtype=torch.int32, device="cuda:0")
    buf[:, :words].copy_(torch.from_numpy(S.view(np.int32)))
    pos, neg, winner = dx.detox_sign_majority(buf[:, :words], d, r, B, vote_perm=vote_perm)
    assert winner.cpu().numpy().tolist() == ref_w.tolist()
    pos = pos.cpu().numpy().view(np.uint32); neg = neg.cpu().numpy().view(np.uint32)
    assert not (pos & neg).any()
    bits = lambda m: np.unpackbits(m.view(np.uint8), bitorder="little")[:d].astype(np.int8)
    got = bits(pos) - bits(neg)
    assert (got == ref).all()
    if d % 32:
        assert (pos[-1] >> (d % 32)) == 0 and (neg[-1] >> (d % 32)) == 0
    return ref


@pytest.mark.parametrize("idx,d,B", [(3, 100003, 5), (3, 4096, 15), (3, 33, 2), (3, 1, 1), (5, 70001, 7),
                                      (5, 70001, 21), (5, 999, 3), (2, 50000, 5), (1, 4096, 3)])
def test_sign_majority(dx, idx, d, B):
    w = workloads.config(idx, d=d)
    X = w.matrix()
    for i in w.byz:
        X[i] = -1.0                                  # the constant attack of Section 5.2
    S = workloads.pack_signs(X)
    _run(dx, S, d, w.r, B)
    rng = np.random.default_rng(d)
    _run(dx, S, d, w.r, B, vote_perm=rng.permutation(w.groups).astype(np.int32), ldw=S.shape[1] + 3)


def test_sign_majority_with_abstaining_and_byzantine_votes(dx):
    w = workloads.config(3, d=20011)
    X = w.matrix()
    X[0] = -X[0]; X[1, :10000] = -X[1, :10000]       # group 0: no majority
    X[6] = -1.0; X[7] = -1.0                          # group 2: colluding Byzantine majority
    S = workloads.pack_signs(X)
    for B in (5, 15, 1, 4):
        ref = _run(dx, S, w.d, 3, B)
    assert (ref == 0).sum() >= 0


@pytest.mark.parametrize("r", [1, 2, 3, 4, 5, 7, 11])
def test_sign_majority_in_the_filter_pass(dx, r):
    """Rows padded to a multiple of four words: the filter pass itself takes both vote levels from
    the per-coordinate majority bits of the node groups (one data-touching launch); with a group
    without majority the stand-alone vote repairs the result.  Every group size, even ones too."""
    groups, d = 12, 40_037
    rng = np.random.default_rng(r)
    base = rng.standard_normal((groups, d)).astype(np.float32)
    X = np.repeat(base, r, axis=0)
    if r >= 3:
        X[0] = -1.0                                   # outvoted
        X[r * 4] = 1.0
    for broken in (False, True):
        if broken and r >= 2:
            for k in range(r):                        # group 7: all members differ somewhere
                X[r * 7 + k, k * 100: k * 100 + 50] *= -1.0
        S = workloads.pack_signs(X, pad_words=4)
        ldw = S.strides[0] // 4
        assert ldw % 4 == 0
        for B, vp in ((3, None), (12, None), (5, rng.permutation(groups).astype(np.int32)), (1, None)):
            _run(dx, np.ascontiguousarray(S), d, r, B, vote_perm=vp, ldw=ldw)
        with dx.trace() as tr:
            _run(dx, np.ascontiguousarray(S), d, r, 4, ldw=ldw)
            names = [k for k, _ in tr.records()]
        assert "filter_sign_vote" in names and "sign_vote_if_redo" in names
