"""ctypes binding of libdetox.so.  Names and argument order follow include/detox.h."""
from __future__ import annotations

import contextlib
import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdetox.so")

OP = dict(filter=0, block_mean=1, pairwise_sqdist=2, multikrum=3, bulyan=4, coord_median=5,
          geomedian=6, step=7, coord_median_many=8, geomedian_many=9, step_robust_blocks=10)
AGG = dict(multikrum=0, bulyan=1, coord_median=2, geomedian=3, trimmed_mean=4)

EXPORTS = ["detox_strerror", "detox_last_hip_error", "detox_workspace_bytes",
           "detox_majority_filter", "detox_block_mean", "detox_filter_block_mean",
           "robust_pairwise_sqdist", "robust_multikrum", "robust_bulyan", "robust_coord_median",
           "robust_geomedian", "robust_trimmed_mean", "robust_coord_median_many",
           "robust_geomedian_many", "detox_step", "detox_step_static", "detox_step_robust_blocks", "detox_sign_majority", "detox_probe_stream_read", "detox_probe_mfma_f32", "detox_trace_enable",
           "detox_trace_read"]


class DetoxError(RuntimeError):
    def __init__(self, code: int, where: str):
        super().__init__(f"{where}: {strerror(code)} (status {code}, hip error {lib().detox_last_hip_error()})")
        self.code = code


class _TraceRecord(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_char_p), ("ms", ctypes.c_float)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Loads the in-tree library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: run `python -m paper_1907_12205_amd.build` "
                               "(or __graft_entry__.build()) first; there is no CPU fallback")
        L = ctypes.CDLL(_LIB_PATH)
        i64, i32, vp, sz, dbl = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_double
        L.detox_strerror.restype = ctypes.c_char_p
        L.detox_strerror.argtypes = [i32]
        L.detox_last_hip_error.restype = i32
        L.detox_workspace_bytes.restype = sz
        L.detox_workspace_bytes.argtypes = [i32, i64, i64, i64]
        L.detox_majority_filter.argtypes = [vp, i64, i64, i64, i32, vp, vp, vp, i64, vp, sz, vp]
        L.detox_block_mean.argtypes = [vp, i64, i64, vp, i64, i64, vp, vp, i64, vp]
        L.detox_filter_block_mean.argtypes = [vp, i64, i64, i64, i32, vp, i64, vp, vp, vp, i64, vp, sz, vp]
        L.robust_pairwise_sqdist.argtypes = [vp, i64, i64, i64, vp, vp, sz, vp]
        L.robust_multikrum.argtypes = [vp, i64, i64, i64, i32, i32, vp, vp, vp, vp, sz, vp]
        L.robust_bulyan.argtypes = [vp, i64, i64, i64, i32, vp, vp, vp, sz, vp]
        L.robust_coord_median.argtypes = [vp, i64, i64, i64, vp, vp]
        L.robust_trimmed_mean.argtypes = [vp, i64, i64, i64, i32, vp, vp]
        L.robust_trimmed_mean.restype = i32
        L.robust_geomedian.argtypes = [vp, i64, i64, i64, i32, dbl, vp, vp, sz, vp]
        L.robust_coord_median_many.argtypes = [vp, i64, i64, i64, vp, vp, sz, vp]
        L.robust_coord_median_many.restype = i32
        L.robust_geomedian_many.argtypes = [vp, i64, i64, i64, i32, dbl, vp, vp, sz, vp]
        L.robust_geomedian_many.restype = i32
        L.detox_step.argtypes = [vp, i64, i64, i64, i32, i32, vp, i64, vp, i32, i32, i32, i32, dbl,
                                 vp, vp, i64, vp, vp, vp, sz, vp]
        L.detox_step_static.argtypes = [vp, i64, i64, i64, i32, i32, vp, i64, vp, i32, i32, i32, i32, dbl,
                                        vp, vp, i64, vp, vp, vp]
        L.detox_step_static.restype = i32
        L.detox_step_robust_blocks.argtypes = [vp, i64, i64, i64, i32, vp, i64, vp, i32, i32, i32, vp, vp, i64,
                                               vp, vp, vp, sz, vp]
        L.detox_step_robust_blocks.restype = i32
        L.detox_sign_majority.argtypes = [vp, i64, i64, i64, i32, vp, i64, vp, vp, vp, vp, vp, sz, vp]
        L.detox_sign_majority.restype = i32
        L.detox_probe_stream_read.argtypes = [vp, sz, vp, vp]
        L.detox_probe_stream_read.restype = i32
        L.detox_probe_mfma_f32.argtypes = [i32, vp, ctypes.POINTER(dbl), vp]
        L.detox_probe_mfma_f32.restype = i32
        L.detox_trace_enable.argtypes = [i32]
        L.detox_trace_enable.restype = None
        L.detox_trace_read.argtypes = [ctypes.POINTER(_TraceRecord), i32]
        for name in ("detox_majority_filter", "detox_block_mean", "detox_filter_block_mean",
                     "robust_pairwise_sqdist", "robust_multikrum", "robust_bulyan",
                     "robust_coord_median", "robust_geomedian", "robust_trimmed_mean", "robust_coord_median_many",
           "robust_geomedian_many", "detox_step", "detox_trace_read"):
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().detox_strerror(int(code)).decode()


def workspace_bytes(op: str, count: int, d: int, aux: int = 0) -> int:
    return int(lib().detox_workspace_bytes(OP[op], count, d, aux))


# ---- marshalling helpers ------------------------------------------------------------------
def _torch():
    import torch
    return torch


def _matrix(X):
    """(pointer, rows, d, ld) of a 2-D fp32 device tensor with unit column stride."""
    torch = _torch()
    if X.dtype != torch.float32 or X.dim() != 2 or X.stride(1) != 1 or not X.is_cuda:
        raise ValueError("expected a 2-D float32 device tensor with unit column stride")
    return X.data_ptr(), X.shape[0], X.shape[1], X.stride(0)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _i32(t, device):
    if t is None:
        return None
    torch = _torch()
    t = torch.as_tensor(t, dtype=torch.int32).to(device).contiguous()
    return t


def _stream():
    return _torch().cuda.current_stream().cuda_stream


def _ws(ws, need: int, device):
    torch = _torch()
    if need == 0:
        return None, 0
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws, ws.numel()


def _check(rc: int, where: str):
    if rc != 0:
        raise DetoxError(rc, where)


# ---- entry points --------------------------------------------------------------------------
def detox_majority_filter(G, r: int, group_rows=None, materialise: bool = False, ws=None):
    """winner[n/r] (int32: row index or -1), and the votes Z when materialise is set."""
    torch = _torch()
    p, n, d, ld = _matrix(G)
    gr = _i32(group_rows, G.device)
    groups = n // max(r, 1)
    winner = torch.empty(max(groups, 1), dtype=torch.int32, device=G.device)
    Z = torch.empty((groups, d), dtype=torch.float32, device=G.device) if materialise else None
    ws, nb = _ws(ws, workspace_bytes("filter", max(groups, 1), d), G.device)
    rc = lib().detox_majority_filter(p, n, d, ld, r, _ptr(gr), _ptr(winner), _ptr(Z), d, _ptr(ws), nb, _stream())
    _check(rc, "detox_majority_filter")
    return (winner, Z) if materialise else winner


def detox_block_mean(G, winner, B: int, vote_perm=None, out=None):
    torch = _torch()
    p, n, d, ld = _matrix(G)
    vp = _i32(vote_perm, G.device)
    if out is None:
        out = torch.empty((B, d), dtype=torch.float32, device=G.device)
    rc = lib().detox_block_mean(p, d, ld, _ptr(winner), winner.numel(), B, _ptr(vp), _ptr(out), out.stride(0), _stream())
    _check(rc, "detox_block_mean")
    return out


def detox_filter_block_mean(G, r: int, B: int, group_rows=None, vote_perm=None, out=None, winner=None, ws=None):
    """Fused filter + block means: returns (winner, Zhat)."""
    torch = _torch()
    p, n, d, ld = _matrix(G)
    gr, vp = _i32(group_rows, G.device), _i32(vote_perm, G.device)
    groups = n // max(r, 1)
    if winner is None:
        winner = torch.empty(max(groups, 1), dtype=torch.int32, device=G.device)
    if out is None:
        out = torch.empty((B, d), dtype=torch.float32, device=G.device)
    ws, nb = _ws(ws, workspace_bytes("filter", max(groups, 1), d), G.device)
    rc = lib().detox_filter_block_mean(p, n, d, ld, r, _ptr(gr), B, _ptr(vp), _ptr(winner), _ptr(out),
                                       out.stride(0), _ptr(ws), nb, _stream())
    _check(rc, "detox_filter_block_mean")
    return winner, out


def robust_pairwise_sqdist(X, ws=None):
    torch = _torch()
    p, count, d, ld = _matrix(X)
    D = torch.empty((count, count), dtype=torch.float64, device=X.device)
    ws, nb = _ws(ws, workspace_bytes("pairwise_sqdist", count, d), X.device)
    _check(lib().robust_pairwise_sqdist(p, count, d, ld, _ptr(D), _ptr(ws), nb, _stream()), "robust_pairwise_sqdist")
    return D


def robust_multikrum(X, f: int, m: int, out=None, ws=None, with_scores: bool = True):
    """Returns (out[d], selected[m], scores[count] or None)."""
    torch = _torch()
    p, count, d, ld = _matrix(X)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=X.device)
    sel = torch.empty(max(m, 1), dtype=torch.int32, device=X.device)
    scores = torch.empty(count, dtype=torch.float64, device=X.device) if with_scores else None
    ws, nb = _ws(ws, workspace_bytes("multikrum", count, d), X.device)
    rc = lib().robust_multikrum(p, count, d, ld, f, m, _ptr(out), _ptr(sel), _ptr(scores), _ptr(ws), nb, _stream())
    _check(rc, "robust_multikrum")
    return out, sel, scores


def robust_bulyan(X, f: int, out=None, ws=None):
    """Returns (out[d], selected[count-2f])."""
    torch = _torch()
    p, count, d, ld = _matrix(X)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=X.device)
    sel = torch.empty(max(count - 2 * f, 1), dtype=torch.int32, device=X.device)
    ws, nb = _ws(ws, workspace_bytes("bulyan", count, d), X.device)
    rc = lib().robust_bulyan(p, count, d, ld, f, _ptr(out), _ptr(sel), _ptr(ws), nb, _stream())
    _check(rc, "robust_bulyan")
    return out, sel


def robust_coord_median(X, out=None):
    torch = _torch()
    p, count, d, ld = _matrix(X)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=X.device)
    _check(lib().robust_coord_median(p, count, d, ld, _ptr(out), _stream()), "robust_coord_median")
    return out


def robust_trimmed_mean(X, g: int, out=None):
    torch = _torch()
    p, count, d, ld = _matrix(X)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=X.device)
    _check(lib().robust_trimmed_mean(p, count, d, ld, g, _ptr(out), _stream()), "robust_trimmed_mean")
    return out


def robust_geomedian(X, iters: int = 50, eps: float = 1e-8, out=None, ws=None):
    torch = _torch()
    p, count, d, ld = _matrix(X)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=X.device)
    ws, nb = _ws(ws, workspace_bytes("geomedian", count, d), X.device)
    rc = lib().robust_geomedian(p, count, d, ld, iters, float(eps), _ptr(out), _ptr(ws), nb, _stream())
    _check(rc, "robust_geomedian")
    return out


def robust_coord_median_many(X, out=None, ws=None):
    """Coordinate-wise median of any number of rows (radix selection on transposed keys)."""
    torch = _torch()
    p, count, d, ld = _matrix(X)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=X.device)
    ws, nb = _ws(ws, workspace_bytes("coord_median_many", count, d), X.device)
    rc = lib().robust_coord_median_many(p, count, d, ld, _ptr(out), _ptr(ws), nb, _stream())
    _check(rc, "robust_coord_median_many")
    return out


def robust_geomedian_many(X, iters: int = 50, eps: float = 1e-8, out=None, ws=None):
    """Geometric median of any number of short rows (streamed Weiszfeld iterations)."""
    torch = _torch()
    p, count, d, ld = _matrix(X)
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=X.device)
    ws, nb = _ws(ws, workspace_bytes("geomedian_many", count, d), X.device)
    rc = lib().robust_geomedian_many(p, count, d, ld, iters, float(eps), _ptr(out), _ptr(ws), nb,
                                     _stream())
    _check(rc, "robust_geomedian_many")
    return out


class StepBuffers:
    """Outputs and workspace of detox_step, allocated once and reused across steps."""

    def __init__(self, n, d, r, B, device, ldo: Optional[int] = None, materialise: bool = True,
                 workspace: bool = True):
        """materialise=False: the block means are not written to memory (Zhat = NULL);
        workspace=False: outputs only (for detox_step_static)."""
        torch = _torch()
        ldo = ldo or ((d + 63) // 64 * 64)
        self.winner = torch.empty(n // r, dtype=torch.int32, device=device)
        self.Zhat = None
        if materialise:
            self.Zhat_buf = torch.empty((B, ldo), dtype=torch.float32, device=device)
            self.Zhat = self.Zhat_buf[:, :d]
        self.selected = torch.full((max(B, 1),), -1, dtype=torch.int32, device=device)
        self.out = torch.empty(d, dtype=torch.float32, device=device)
        self.ws = (torch.empty(max(workspace_bytes("step", n, d, B), 256), dtype=torch.uint8, device=device)
                   if workspace else None)


def detox_step(G, r: int, q: int, B: int, aggregator: str, f: int = -1, m: int = -1, iters: int = 50,
               eps: float = 1e-8, group_rows=None, vote_perm=None, buffers: Optional[StepBuffers] = None,
               materialise: bool = True):
    """The whole step.  Returns the StepBuffers holding out, winner, Zhat (or None) and selected."""
    p, n, d, ld = _matrix(G)
    gr, vp = _i32(group_rows, G.device), _i32(vote_perm, G.device)
    if buffers is None:
        buffers = StepBuffers(n, d, max(r, 1), B, G.device, materialise=materialise)
    b = buffers
    rc = lib().detox_step(p, n, d, ld, r, q, _ptr(gr), B, _ptr(vp), AGG[aggregator], f, m, iters, float(eps),
                          _ptr(b.winner), _ptr(b.Zhat), b.Zhat.stride(0) if b.Zhat is not None else 0,
                          _ptr(b.selected), _ptr(b.out),
                          _ptr(b.ws), b.ws.numel(), _stream())
    _check(rc, "detox_step")
    return b


def detox_step_static(G, r: int, q: int, B: int, aggregator: str, buffers: StepBuffers, f: int = -1, m: int = -1,
                      iters: int = 50, eps: float = 1e-8, group_rows=None, vote_perm=None):
    """detox_step on the library's own scratch array: no workspace, nothing allocated.  `buffers`
    holds the outputs (StepBuffers(..., workspace=False)); index arrays must be device tensors."""
    p, n, d, ld = _matrix(G)
    b = buffers
    rc = lib().detox_step_static(p, n, d, ld, r, q, _ptr(group_rows), B, _ptr(vote_perm), AGG[aggregator], f, m,
                                 iters, float(eps), _ptr(b.winner), _ptr(b.Zhat),
                                 b.Zhat.stride(0) if b.Zhat is not None else 0, _ptr(b.selected), _ptr(b.out),
                                 _stream())
    _check(rc, "detox_step_static")
    return b


def robust_blocks_workspace_bytes(n: int, d: int, r: int, B: int) -> int:
    """Workspace of detox_step_robust_blocks."""
    return workspace_bytes("step_robust_blocks", n // max(r, 1), d, B)


def detox_step_robust_blocks(G, r: int, B: int, a0: str, f: int, m: int = -1, group_rows=None, vote_perm=None,
                             out=None, ws=None):
    """Robust aggregator inside every vote group, mean over the groups.
    Returns (out[d], winner[n/r], block_out[B x d] or None, selected[n/r])."""
    torch = _torch()
    p, n, d, ld = _matrix(G)
    gr, vp = _i32(group_rows, G.device), _i32(vote_perm, G.device)
    groups = n // max(r, 1)
    winner = torch.empty(max(groups, 1), dtype=torch.int32, device=G.device)
    selected = torch.full((max(groups, 1),), -1, dtype=torch.int32, device=G.device)
    block_out = torch.empty((B, d), dtype=torch.float32, device=G.device) if B > 1 else None
    if out is None:
        out = torch.empty(d, dtype=torch.float32, device=G.device)
    ws, nb = _ws(ws, robust_blocks_workspace_bytes(n, d, r, B), G.device)
    rc = lib().detox_step_robust_blocks(p, n, d, ld, r, _ptr(gr), B, _ptr(vp), AGG[a0], f, m, _ptr(winner),
                                        _ptr(block_out), d, _ptr(selected), _ptr(out), _ptr(ws), nb, _stream())
    _check(rc, "detox_step_robust_blocks")
    return out, winner, block_out, selected


def detox_sign_majority(S, d: int, r: int, B: int, group_rows=None, vote_perm=None, ws=None, out=None):
    """signSGD pairing: S is an n x words int32/uint32 device tensor of bit-packed signs.
    Returns (out_pos[words], out_neg[words], winner[n/r]) as int32 tensors holding the bit masks."""
    torch = _torch()
    if S.dim() != 2 or S.stride(1) != 1 or S.element_size() != 4 or not S.is_cuda:
        raise ValueError("expected a 2-D device tensor of 32-bit words with unit column stride")
    n, ldw = S.shape[0], S.stride(0)
    words = (d + 31) // 32
    gr, vp = _i32(group_rows, S.device), _i32(vote_perm, S.device)
    groups = n // max(r, 1)
    winner = torch.empty(max(groups, 1), dtype=torch.int32, device=S.device)
    if out is None:
        out = torch.empty((2, words), dtype=torch.int32, device=S.device)
    ws, nb = _ws(ws, workspace_bytes("filter", max(groups, 1), words), S.device)
    rc = lib().detox_sign_majority(S.data_ptr(), n, d, ldw, r, _ptr(gr), B, _ptr(vp), _ptr(winner),
                                   out[0].data_ptr(), out[1].data_ptr(), _ptr(ws), nb, _stream())
    _check(rc, "detox_sign_majority")
    return out[0], out[1], winner


def probe_stream_read(buf, sink):
    """Enqueues one read of every byte of the device tensor `buf` (the caller times it)."""
    _check(lib().detox_probe_stream_read(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream()),
           "detox_probe_stream_read")


def probe_mfma_f32(iters: int, sink) -> float:
    """Enqueues the fp32 MFMA probe; returns the number of floating-point operations it performs."""
    flop = ctypes.c_double(0.0)
    _check(lib().detox_probe_mfma_f32(int(iters), sink.data_ptr(), ctypes.byref(flop), _stream()), "detox_probe_mfma_f32")
    return float(flop.value)


@contextlib.contextmanager
def trace():
    """Per-kernel timing: `with trace() as t: ...; t.records()` -> [(kernel, ms), ...]."""
    class _T:
        def records(self, cap: int = 4096):
            _torch().cuda.synchronize()
            buf = (_TraceRecord * cap)()
            k = lib().detox_trace_read(buf, cap)
            return [(buf[i].kernel.decode(), float(buf[i].ms)) for i in range(k)]
    lib().detox_trace_enable(1)
    try:
        yield _T()
    finally:
        lib().detox_trace_enable(0)
