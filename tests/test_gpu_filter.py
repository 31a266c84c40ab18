"""GPU parity: majority-vote filter and block means against the CPU oracle, bit for bit."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import dev_matrix, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dx():
    import torch
    assert torch.cuda.is_available()
    import paper_1907_12205_amd as dx
    return dx


def _check_filter(dx, G, r, group_rows=None, ld=None, offset=0):
    ref_w, ref_Z = oracle.majority_filter(G, r, group_rows=group_rows, materialise=True)
    Gd = dev_matrix(G, ld, offset)
    w, Z = dx.detox_majority_filter(Gd, r, group_rows=group_rows, materialise=True)
    assert host(w).tolist() == ref_w.tolist()
    assert host(Z).tobytes() == ref_Z.tobytes()
    w2 = dx.detox_majority_filter(Gd, r, group_rows=group_rows)
    assert host(w2).tolist() == ref_w.tolist()
    return ref_w


@pytest.mark.parametrize("idx,d", [(1, 4096), (2, 70001), (3, 50003), (4, 33333), (5, 20002)])
@pytest.mark.parametrize("layout", ["ld=d", "padded", "odd-offset"])
def test_filter_configs(dx, idx, d, layout):
    w = workloads.config(idx, d=d)
    G = w.matrix()
    ld = None if layout != "padded" else (d + 63) // 64 * 64
    offset = 1 if layout == "odd-offset" else 0
    winners = _check_filter(dx, G, w.r, ld=ld, offset=offset)
    assert (winners >= 0).all()


@pytest.mark.parametrize("r", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11])
def test_filter_all_group_sizes_and_outcomes(dx, r):
    rng = np.random.default_rng(r)
    groups, d = 12, 3001
    base = rng.standard_normal((groups, d)).astype(np.float32)
    G = np.repeat(base, r, axis=0)
    # corrupt a varying number of members per group, some colluding, some each on their own
    for g in range(groups):
        k = g % (r + 1)
        members = rng.permutation(r)[:k]
        collude = g % 2 == 0
        bad = rng.standard_normal(d).astype(np.float32)
        for m in members:
            G[g * r + m] = bad if collude else rng.standard_normal(d).astype(np.float32)
    _check_filter(dx, G, r)
    # scattered groups
    perm = rng.permutation(groups * r).astype(np.int32)
    _check_filter(dx, G, r, group_rows=perm)


def test_filter_single_word_differences(dx):
    d = 5000
    a = np.arange(d, dtype=np.float32)
    for pos in (0, 1, 1023, 1024, 4095, d - 2, d - 1):
        b = a.copy(); b[pos] = -1
        c = a.copy(); c[(pos + 7) % d] = -2
        assert _check_filter(dx, np.stack([a, b, c]), 3).tolist() == [-1]
        assert _check_filter(dx, np.stack([b, a, b]), 3).tolist() == [0]
        assert _check_filter(dx, np.stack([a, b, a]), 3).tolist() == [0]


def test_filter_bitwise_equality(dx):
    d = 300
    z = np.zeros(d, dtype=np.float32)
    nz = -z
    assert _check_filter(dx, np.stack([z, nz, nz]), 3).tolist() == [1]
    assert _check_filter(dx, np.stack([z, nz, z + 1]), 3).tolist() == [-1]
    nan_a = np.full(d, 0x7FC00000, dtype=np.uint32).view(np.float32)
    nan_b = np.full(d, 0x7FC00001, dtype=np.uint32).view(np.float32)
    assert _check_filter(dx, np.stack([nan_a, nan_a.copy(), nan_b]), 3).tolist() == [0]
    assert _check_filter(dx, np.stack([nan_a, nan_b, z]), 3).tolist() == [-1]


def test_filter_piecewise_agreement(dx):
    d = 4096
    a = np.ones(d, dtype=np.float32); b = a.copy(); c = a.copy()
    b[d // 2:] = 2; a[d // 2:] = 3          # a==b==c on the first half, only b!=a!=c after
    c[d // 2:] = 2; c[: d // 2] = 5         # c agrees with b on the second half only
    assert _check_filter(dx, np.stack([a, b, c]), 3).tolist() == [-1]


@pytest.mark.parametrize("idx,d,B", [(3, 50003, 5), (3, 4099, 2), (3, 777, 15), (4, 10001, 5),
                                      (5, 9999, 7), (5, 1025, 4), (2, 70001, 5), (1, 4096, 3)])
@pytest.mark.parametrize("layout", ["ld=d", "padded"])
def test_block_mean_and_fused(dx, idx, d, B, layout):
    w = workloads.config(idx, d=d)
    G = w.matrix()
    ld = None if layout != "padded" else (d + 63) // 64 * 64
    Gd = dev_matrix(G, ld)
    ref_w = oracle.majority_filter(G, w.r)
    rng = np.random.default_rng(d)
    for perm in (None, rng.permutation(w.groups).astype(np.int32)):
        ref = oracle.block_mean(G, ref_w, B, vote_perm=perm)
        wd = dx.detox_majority_filter(Gd, w.r)
        got = dx.detox_block_mean(Gd, wd, B, vote_perm=perm)
        assert host(got).tobytes() == ref.tobytes()
        w2, fused = dx.detox_filter_block_mean(Gd, w.r, B, vote_perm=perm)
        assert host(w2).tolist() == ref_w.tolist()
        assert host(fused).tobytes() == ref.tobytes()
        ref64 = oracle.block_mean(G, ref_w, B, vote_perm=perm, fp64=True)
        assert np.linalg.norm(host(fused) - ref64) <= 1e-5 * np.linalg.norm(ref64)


def test_fused_redoes_blocks_with_a_vote_without_majority(dx):
    # group 1 has no majority (piecewise agreement: every coordinate has a majority value),
    # group 4 has none at all, group 6 is taken over by two colluding Byzantine rows
    w = workloads.config(3, d=6007)
    G = w.matrix()
    d = w.d
    G[3, d // 2:] += 1; G[5, : d // 2] += 2
    G[12] = 7; G[13] = 8; G[14] = 9
    G[18] = -3; G[20] = -3
    ref_w = oracle.majority_filter(G, 3)
    assert ref_w[1] == -1 and ref_w[4] == -1 and ref_w[6] == 18
    Gd = dev_matrix(G)
    for B in (5, 15, 1, 4):
        ref = oracle.block_mean(G, ref_w, B)
        w2, fused = dx.detox_filter_block_mean(Gd, 3, B)
        assert host(w2).tolist() == ref_w.tolist()
        assert host(fused).tobytes() == ref.tobytes()


def test_repeated_calls_are_bit_identical(dx):
    w = workloads.config(3, d=30011)
    Gd = dev_matrix(w.matrix())
    a = dx.detox_filter_block_mean(Gd, 3, 5)
    b = dx.detox_filter_block_mean(Gd, 3, 5)
    assert host(a[1]).tobytes() == host(b[1]).tobytes() and host(a[0]).tolist() == host(b[0]).tolist()


def test_many_groups_take_the_general_kernel(dx):
    """More than 1024 node groups: the per-group flag words with integer atomics (grid.y = vote
    group) instead of the persistent kernel; also exercised with block means and the whole step."""
    rng = np.random.default_rng(77)
    groups, r, d = 1500, 3, 2301          # wider than the rows the row-parallel kernels take
    base = rng.standard_normal((groups, d)).astype(np.float32)
    G = np.repeat(base, r, axis=0)
    for g in rng.choice(groups, size=200, replace=False):
        kind = g % 3
        if kind == 0:
            G[g * r + int(rng.integers(r))] = rng.standard_normal(d).astype(np.float32)     # one Byzantine member
        elif kind == 1:
            bad = rng.standard_normal(d).astype(np.float32)                                 # two colluding
            G[g * r] = bad; G[g * r + 2] = bad
        else:
            G[g * r + 1, d // 2:] += 1; G[g * r + 2, : d // 2] -= 1                        # no majority
    ref_w = _check_filter(dx, G, r)
    assert (ref_w < 0).sum() > 10
    Gd = dev_matrix(G)
    for B in (10, 1500, 7):
        ref = oracle.block_mean(G, ref_w, B)
        w2, fused = dx.detox_filter_block_mean(Gd, r, B)
        assert host(w2).tolist() == ref_w.tolist()
        assert host(fused).tobytes() == ref.tobytes()
    ref_out, _, _ = oracle.detox_step(G, r, 10, "coord_median")
    b = dx.detox_step(Gd, r, 100, 10, "coord_median")
    assert host(b.out).tobytes() == ref_out.tobytes()
    ref_out, _, _ = oracle.detox_step(G, r, 20, "multikrum", f=2, m=10)
    b = dx.detox_step(Gd, r, 100, 20, "multikrum", f=2, m=10)
    assert np.linalg.norm(host(b.out) - ref_out) <= 1e-5 * np.linalg.norm(ref_out)
