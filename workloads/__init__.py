"""Seeded synthetic inputs shaped like the paper's parameter-server workloads.

This module only *makes inputs*: an n x d fp32 matrix of node gradients in which
the honest members of a node group hold bitwise-identical rows (Section 3: they
evaluate the same gradient on the same samples) and the Byzantine rows follow
one of the attack models of Section 5.2.  It contains none of the aggregation
arithmetic and is the only code shared by the CPU oracle's tests and the GPU
path's tests.  The paper's real inputs are ResNet-18 / VGG13-BN gradients from
45 workers; those models and datasets are not available here, so these
generators stand in for them with the same shapes.

Random numbers come from numpy's counter-based Philox generator keyed by
(seed, stream), so every vector is reproducible on its own.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

DEFAULT_SEED = 20190712

# stream identifiers for Philox keys
_S_PLACEMENT = 1
_S_BASE = 1000
_S_BYZ = 2000


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


@dataclass
class Workload:
    name: str
    n: int
    r: int
    q: int
    d: int
    base: np.ndarray                     # (n/r) x d fp32: the honest gradient of each group
    byz: Dict[int, np.ndarray]           # row index -> Byzantine vector (d fp32)
    detox: List[dict] = field(default_factory=list)    # pipelines run after the filter
    vanilla: List[dict] = field(default_factory=list)  # aggregators run on all n rows
    attack: str = ""

    @property
    def groups(self) -> int:
        return self.n // self.r

    def row(self, i: int) -> np.ndarray:
        return self.byz[i] if i in self.byz else self.base[i // self.r]

    def matrix(self, ld: Optional[int] = None) -> np.ndarray:
        """Dense n x d host matrix (a view of an n x ld buffer when ld is given)."""
        ld = self.d if ld is None else ld
        buf = np.zeros((self.n, ld), dtype=np.float32)
        buf[:, : self.d] = np.repeat(self.base, self.r, axis=0)
        for i, v in self.byz.items():
            buf[i, : self.d] = v
        return buf[:, : self.d]

    def honest_mean(self) -> np.ndarray:
        """fp64 mean of the group base gradients (what DETOX approximates without attack)."""
        return self.base.astype(np.float64).mean(axis=0)

    def to_device(self, device="cuda:0", ld: Optional[int] = None):
        """Upload as an n x d view of an n x ld torch buffer; replicas are device copies."""
        import torch

        ld = self.d if ld is None else ld
        buf = torch.zeros((self.n, ld), dtype=torch.float32, device=device)
        G = buf[:, : self.d]
        for g in range(self.groups):
            src = torch.from_numpy(self.base[g]).to(device)
            for k in range(self.r):
                i = g * self.r + k
                if i not in self.byz:
                    G[i].copy_(src)
            del src
        for i, v in self.byz.items():
            G[i].copy_(torch.from_numpy(v).to(device))
        torch.cuda.synchronize()
        return G


def place_byzantine(seed: int, n: int, r: int, q: int, max_per_group: int) -> List[int]:
    """q distinct rows packed max_per_group to a node group (the last group may get fewer)."""
    rng = _rng(seed, _S_PLACEMENT)
    groups = n // r
    if max_per_group > r or q > groups * max_per_group:
        raise ValueError("too many Byzantine nodes for this placement rule")
    rows = []
    left = q
    for g in rng.permutation(groups):
        if left == 0:
            break
        take = min(max_per_group, left)
        members = rng.permutation(r)[:take]
        rows += [int(g) * r + int(k) for k in members]
        left -= take
    return sorted(rows)


def _base_normal(seed, groups, d, sigma):
    base = np.empty((groups, d), dtype=np.float32)
    for g in range(groups):
        base[g] = _rng(seed, _S_BASE + g).standard_normal(d, dtype=np.float32) * np.float32(sigma)
    return base


def _base_student_t(seed, groups, d, nu, scale):
    base = np.empty((groups, d), dtype=np.float32)
    step = 1 << 22
    for g in range(groups):
        rng = _rng(seed, _S_BASE + g)
        for c0 in range(0, d, step):
            c1 = min(d, c0 + step)
            base[g, c0:c1] = (rng.standard_t(nu, c1 - c0) * scale).astype(np.float32)
    return base


def _alie_vector(base, r, byz_rows, z):
    """mean + z * std per coordinate over the honest rows (the ALIE attack of Section 5.2)."""
    groups, d = base.shape
    honest = np.full(groups, r, dtype=np.float64)
    for i in byz_rows:
        honest[i // r] -= 1
    total = honest.sum()
    out = np.empty(d, dtype=np.float32)
    step = 1 << 20
    for c0 in range(0, d, step):
        blk = base[:, c0:c0 + step].astype(np.float64)
        mu = (honest[:, None] * blk).sum(axis=0) / total
        var = (honest[:, None] * (blk - mu) ** 2).sum(axis=0) / total
        out[c0:c0 + step] = (mu + z * np.sqrt(var)).astype(np.float32)
    return out


def config(index: int, seed: int = DEFAULT_SEED, d: Optional[int] = None) -> Workload:
    """The five workloads (index 1..5).  `d` overrides the dimension, keeping the structure."""
    if index == 1:
        n, r, q, d = 9, 3, 1, d or 4096
        base = _base_normal(seed, n // r, d, 1.0)
        rows = place_byzantine(seed, n, r, q, 1)
        byz = {i: np.full(d, -100.0, dtype=np.float32) for i in rows}
        return Workload("cfg1", n, r, q, d, base, byz, attack="constant -100",
                        detox=[dict(B=3, aggregator="coord_median")])
    if index == 2:
        n, r, q, d = 15, 3, 2, d or (1 << 20)
        base = _base_normal(seed, n // r, d, 0.1)
        rows = place_byzantine(seed, n, r, q, 1)
        byz = {i: (np.float32(-10.0) * base[i // r]) for i in rows}
        return Workload("cfg2", n, r, q, d, base, byz, attack="reverse gradient, c=10",
                        detox=[dict(B=5, aggregator="multikrum", f=1, m=3)],
                        vanilla=[dict(aggregator="multikrum", f=2, m=13)])
    if index == 3:
        n, r, q, d = 45, 3, 5, d or 11_173_962
        base = _base_normal(seed, n // r, d, np.sqrt(1e-3))
        rows = place_byzantine(seed, n, r, q, 1)
        v = _alie_vector(base, r, rows, 1.5)
        byz = {i: v for i in rows}
        return Workload("cfg3", n, r, q, d, base, byz, attack="ALIE, z=1.5",
                        detox=[dict(B=5, aggregator="multikrum", f=1, m=3)],
                        vanilla=[dict(aggregator="multikrum", f=5, m=40)])
    if index == 4:
        n, r, q, d = 45, 3, 5, d or 25_000_000
        base = _base_student_t(seed, n // r, d, 3, 1e-3)
        rows = place_byzantine(seed, n, r, q, 1)
        byz = {i: _rng(seed, _S_BYZ + i).uniform(-1.0, 1.0, d).astype(np.float32) for i in rows}
        return Workload("cfg4", n, r, q, d, base, byz, attack="uniform [-1,1]",
                        detox=[dict(B=15, aggregator="bulyan", f=1),
                               dict(B=5, aggregator="coord_median")],
                        vanilla=[dict(aggregator="bulyan", f=5)])
    if index == 5:
        n, r, q, d = 105, 5, 10, d or 25_000_000
        base = _base_normal(seed, n // r, d, np.sqrt(1e-3))
        rows = place_byzantine(seed, n, r, q, 2)
        signs = _rng(seed, _S_BYZ).integers(0, 2, size=len(rows)) * 2 - 1
        byz = {i: np.full(d, 100.0 * s, dtype=np.float32) for i, s in zip(rows, signs)}
        return Workload("cfg5", n, r, q, d, base, byz, attack="constant +-100",
                        detox=[dict(B=7, aggregator="geomedian", iters=50, eps=1e-8)],
                        vanilla=[dict(aggregator="coord_median"),
                                 dict(aggregator="multikrum", f=10, m=95)])
    raise ValueError("config index must be 1..5")


def mean_estimation(d: int, seed: int = DEFAULT_SEED, n: int = 220_000, r: int = 11,
                    q: Optional[int] = None, batch: int = 20, norm: float = 100.0) -> Workload:
    """The synthetic mean-estimation setting of Section 5.3: n = 220000 nodes in groups of
    r = 11, q = floor(e^r / 3) Byzantine nodes placed uniformly at random; every node group
    holds the mean of `batch` = 20 iid N(0, I_d) samples (honest members bitwise identical);
    every Byzantine node sends the same constant vector of l2 norm 100.  The true mean is 0, so
    the error of an estimate is its l2 norm."""
    import math

    if q is None:
        q = int(math.floor(math.exp(r) / 3.0))
    groups = n // r
    base = np.empty((groups, d), dtype=np.float32)
    rng = _rng(seed, _S_BASE)
    step = 4096
    for g0 in range(0, groups, step):
        g1 = min(groups, g0 + step)
        x = rng.standard_normal((g1 - g0, batch, d), dtype=np.float32)
        base[g0:g1] = x.mean(axis=1, dtype=np.float64).astype(np.float32)
    rows = np.sort(_rng(seed, _S_PLACEMENT).choice(n, size=q, replace=False))
    v = np.full(d, norm / math.sqrt(d), dtype=np.float32)
    byz = {int(i): v for i in rows}
    B = 65
    return Workload(f"mean_estimation_d{d}", n, r, q, d, base, byz,
                    attack=f"constant vector of norm {norm:g}",
                    detox=[dict(B=B, aggregator="coord_median"),
                           dict(B=B, aggregator="geomedian", iters=50, eps=1e-8)],
                    vanilla=[dict(aggregator="coord_median"),
                             dict(aggregator="geomedian", iters=50, eps=1e-8)])


def distinct_rows(seed: int, count: int, d: int, sigma: float = 1.0, mean: float = 0.0):
    """count independent N(mean, sigma^2) rows (the vanilla setting: every node its own batch)."""
    X = np.empty((count, d), dtype=np.float32)
    for i in range(count):
        X[i] = _rng(seed, _S_BASE + i).standard_normal(d, dtype=np.float32) * np.float32(sigma)
    if mean:
        X += np.float32(mean)
    return X


def integer_rows(seed: int, count: int, d: int, lo: int = -8, hi: int = 8):
    """Rows of small integers: every sum and product is exact in fp32 and fp64."""
    return _rng(seed, _S_BASE).integers(lo, hi + 1, size=(count, d)).astype(np.float32)


def pack_signs(X, pad_words: int = 1):
    """Bit-pack the signs of a float matrix for the signSGD pairing (input preparation only):
    bit (c % 32) of word (c // 32) set <=> X[i, c] >= 0; unused bits of the last word are zero.
    pad_words: the row stride is rounded up to a multiple of it (4: rows stay 16-byte aligned);
    the result is the n x ceil(d/32) view of that buffer."""
    n, d = X.shape
    words = (d + 31) // 32
    ldw = (words + pad_words - 1) // pad_words * pad_words
    out = np.zeros((n, ldw), dtype=np.uint32)[:, :words]
    for i in range(n):
        bits = np.zeros(words * 32, dtype=np.uint8)
        bits[:d] = X[i] >= 0
        out[i] = np.packbits(bits.reshape(words, 32), axis=-1, bitorder="little").view(np.uint32).reshape(words)
    return out
