"""Helpers shared by the GPU parity tests: host<->device plumbing only."""
import numpy as np


def dev_matrix(X: np.ndarray, ld=None, offset=0):
    """Upload a host matrix as a (rows x d) view of a device buffer with row stride ld; `offset`
    (in elements) shifts the base pointer to exercise the narrower-load paths."""
    import torch

    rows, d = X.shape
    ld = d if ld is None else ld
    buf = torch.zeros(rows * ld + offset + 8, dtype=torch.float32, device="cuda:0")
    view = buf[offset: offset + rows * ld].view(rows, ld)[:, :d]
    view.copy_(torch.from_numpy(np.ascontiguousarray(X)))
    return view


def host(t):
    return t.detach().cpu().numpy()


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64); b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return np.linalg.norm(a - b) / (den if den > 0 else 1.0)
