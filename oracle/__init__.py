"""CPU oracle for the DETOX parameter-server step (numpy-facing wrapper).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
benchmark's ``cpu_baseline`` leg.  The GPU package never imports this module
and this module never imports the GPU package.

Every function takes and returns host numpy arrays and calls the plain C
implementation in ``detox_oracle.c`` (built by ``oracle.build()``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "detox_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

OK, EINVAL, EPRECOND, ENOMEM = 0, 1, 2, 3


class OracleError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"oracle: {where} returned {code}")
        self.code = code


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (IEEE arithmetic: no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra", "-shared",
               "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


_i64 = ctypes.c_int64
_int = ctypes.c_int


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _rows(X: np.ndarray):
    """Return (array, count, d, ld) for a 2-D fp32 matrix whose rows are contiguous."""
    if X.dtype != np.float32 or X.ndim != 2 or X.strides[1] != 4 or X.strides[0] % 4:
        raise ValueError("expected a 2-D float32 array with unit column stride")
    return X, X.shape[0], X.shape[1], X.strides[0] // 4


def _i32(a, n=None):
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.int32)
    if n is not None and a.size != n:
        raise ValueError("index array has the wrong length")
    return a


def _check(rc: int, where: str):
    if rc != OK:
        raise OracleError(rc, where)


def majority_filter(G, r, group_rows=None, materialise=False):
    """Votes of the node groups.  Returns winner[n/r] (row index or -1), and Z if asked."""
    G, n, d, ld = _rows(G)
    if r < 1 or n % r:
        raise OracleError(EINVAL, "majority_filter")
    gr = _i32(group_rows, n)
    winner = np.empty(n // r, dtype=np.int32)
    Z = np.empty((n // r, d), dtype=np.float32) if materialise else None
    rc = lib().oracle_majority_filter(_p(G), _i64(n), _i64(d), _i64(ld), _int(r), _p(gr),
                                      _p(winner), _p(Z), _i64(d))
    _check(rc, "majority_filter")
    return (winner, Z) if materialise else winner


def block_mean(G, winner, B, vote_perm=None, fp64=False):
    """Means of the B vote groups (A0 = mean); fp32 sequential by default, fp64 on request."""
    G, n, d, ld = _rows(G)
    winner = _i32(winner)
    V = winner.size
    vp = _i32(vote_perm, V)
    out = np.empty((B, d), dtype=np.float64 if fp64 else np.float32)
    fn = lib().oracle_block_mean_f64 if fp64 else lib().oracle_block_mean
    rc = fn(_p(G), _i64(d), _i64(ld), _p(winner), _i64(V), _i64(B), _p(vp), _p(out), _i64(d))
    _check(rc, "block_mean")
    return out


def coord_median(X):
    X, count, d, ld = _rows(X)
    out = np.empty(d, dtype=np.float32)
    _check(lib().oracle_coord_median(_p(X), _i64(count), _i64(d), _i64(ld), _p(out)),
           "coord_median")
    return out


def trimmed_mean(X, g):
    """Coordinate-wise trimmed mean dropping the g smallest and g largest values."""
    X, count, d, ld = _rows(X)
    out = np.empty(d, dtype=np.float32)
    _check(lib().oracle_trimmed_mean(_p(X), _i64(count), _i64(d), _i64(ld), _i64(g), _p(out)),
           "trimmed_mean")
    return out


def pairwise_sqdist(X):
    X, count, d, ld = _rows(X)
    D = np.empty((count, count), dtype=np.float64)
    _check(lib().oracle_pairwise_sqdist(_p(X), _i64(count), _i64(d), _i64(ld), _p(D)),
           "pairwise_sqdist")
    return D


def krum_scores(D, f):
    D = np.ascontiguousarray(D, dtype=np.float64)
    count = D.shape[0]
    s = np.empty(count, dtype=np.float64)
    _check(lib().oracle_krum_scores(_p(D), _i64(count), _int(f), _p(s)), "krum_scores")
    return s


def multikrum_from_dist(D, f, m):
    D = np.ascontiguousarray(D, dtype=np.float64)
    count = D.shape[0]
    sel = np.empty(max(m, 1), dtype=np.int32)
    s = np.empty(count, dtype=np.float64)
    _check(lib().oracle_multikrum_from_dist(_p(D), _i64(count), _int(f), _int(m), _p(sel), _p(s)),
           "multikrum_from_dist")
    return sel, s


def multikrum(X, f, m):
    """Returns (out[d] fp32, selected[m] int32, scores[count] fp64)."""
    X, count, d, ld = _rows(X)
    out = np.empty(d, dtype=np.float32)
    sel = np.empty(max(m, 1), dtype=np.int32)
    s = np.empty(count, dtype=np.float64)
    rc = lib().oracle_multikrum(_p(X), _i64(count), _i64(d), _i64(ld), _int(f), _int(m), _p(out),
                                _p(sel), _p(s))
    _check(rc, "multikrum")
    return out, sel, s


def bulyan_select(D, f):
    D = np.ascontiguousarray(D, dtype=np.float64)
    count = D.shape[0]
    sel = np.empty(max(count - 2 * f, 1), dtype=np.int32)
    _check(lib().oracle_bulyan_select(_p(D), _i64(count), _int(f), _p(sel)), "bulyan_select")
    return sel


def bulyan_trim(X, rows, beta):
    X, count, d, ld = _rows(X)
    rows = _i32(rows)
    out = np.empty(d, dtype=np.float32)
    rc = lib().oracle_bulyan_trim(_p(X), _i64(d), _i64(ld), _p(rows), _i64(rows.size), _i64(beta),
                                  _p(out))
    _check(rc, "bulyan_trim")
    return out


def bulyan(X, f):
    """Returns (out[d] fp32, selected[count-2f] int32 in selection order)."""
    X, count, d, ld = _rows(X)
    out = np.empty(d, dtype=np.float32)
    sel = np.empty(max(count - 2 * f, 1), dtype=np.int32)
    rc = lib().oracle_bulyan(_p(X), _i64(count), _i64(d), _i64(ld), _int(f), _p(out), _p(sel))
    _check(rc, "bulyan")
    return out, sel


def geomedian(X, iters=50, eps=1e-8, with_objective=False):
    X, count, d, ld = _rows(X)
    out = np.empty(d, dtype=np.float32)
    obj = np.empty(iters + 1, dtype=np.float64) if with_objective else None
    rc = lib().oracle_geomedian(_p(X), _i64(count), _i64(d), _i64(ld), _int(iters),
                                ctypes.c_double(eps), _p(out), _p(obj))
    _check(rc, "geomedian")
    return (out, obj) if with_objective else out


def detox_step(G, r, B, aggregator, f=0, m=1, iters=50, eps=1e-8, group_rows=None,
               vote_perm=None):
    """Filter -> block means -> robust aggregator over the block means (Algorithms 1 and 2)."""
    winner = majority_filter(G, r, group_rows)
    Zhat = block_mean(G, winner, B, vote_perm)
    if aggregator == "multikrum":
        out = multikrum(Zhat, f, m)[0]
    elif aggregator == "bulyan":
        out = bulyan(Zhat, f)[0]
    elif aggregator == "coord_median":
        out = coord_median(Zhat)
    elif aggregator == "geomedian":
        out = geomedian(Zhat, iters, eps)
    elif aggregator == "trimmed_mean":
        out = trimmed_mean(Zhat, f if f >= 0 else B // 4)
    else:
        raise ValueError(aggregator)
    return out, winner, Zhat


def sign_majority(S, d, r, B, group_rows=None, vote_perm=None):
    """DETOX paired with signSGD: returns (out[d] int8 in {-1,0,+1}, winner[n/r])."""
    if S.dtype != np.uint32 or S.ndim != 2 or S.strides[1] != 4:
        raise ValueError("expected a 2-D uint32 array with unit column stride")
    n, ldw = S.shape[0], S.strides[0] // 4
    if r < 1 or n % r:
        raise OracleError(EINVAL, "sign_majority")
    winner = np.empty(n // r, dtype=np.int32)
    out = np.empty(d, dtype=np.int8)
    gr, vp = _i32(group_rows, n), _i32(vote_perm, n // r)
    rc = lib().oracle_sign_majority(_p(S), _i64(n), _i64(d), _i64(ldw), _int(r), _p(gr), _i64(B), _p(vp),
                                    _p(winner), _p(out))
    _check(rc, "sign_majority")
    return out, winner


def detox_step_robust_blocks(G, r, B, a0, f, m=-1, group_rows=None, vote_perm=None):
    """Algorithm 2 as deployed in Section 5.2 (setups 2 and 3): A0 = Multi-Krum / Bulyan inside
    every vote group, A1 = mean of the group results (fp64 sum in group order, cast once).
    Returns (out, winner, block_out[B x d], selections: list of per-group index arrays)."""
    winner, Z = majority_filter(G, r, group_rows, materialise=True)
    V = winner.size
    order = np.arange(V) if vote_perm is None else np.asarray(vote_perm)
    outs, sels = [], []
    for b in range(B):
        lo, hi = (b * V) // B, ((b + 1) * V) // B
        X = np.ascontiguousarray(Z[order[lo:hi]])
        if a0 == "multikrum":
            o, sel, _ = multikrum(X, f, (hi - lo) - f if m < 0 else m)
        elif a0 == "bulyan":
            o, sel = bulyan(X, f)
        else:
            raise ValueError(a0)
        outs.append(o)
        sels.append(sel)
    block_out = np.stack(outs)
    acc = np.zeros(G.shape[1], dtype=np.float64)
    for o in outs:
        acc += o.astype(np.float64)
    out = (acc / B).astype(np.float32) if B > 1 else outs[0]
    return out, winner, block_out, sels
