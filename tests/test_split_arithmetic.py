"""The arithmetic behind the Gram kernels of more than 8 rows, checked on the CPU with numpy: an
fp32 operand cut into three bf16 pieces (each the rounded rest of the one before) is represented
exactly, and the six products the kernels keep differ from the full product by less than
3 * 2^-24 of its magnitude (the three products left out).  This pins the reading, not the kernels:
nothing here calls the library."""
import numpy as np


def bf16_round(x):
    """Round-to-nearest-even of fp32 values to bf16, returned as fp32."""
    u = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32)


def cut(x):
    h = bf16_round(x)
    r1 = (x - h).astype(np.float32)
    m = bf16_round(r1)
    r2 = (r1 - m).astype(np.float32)
    l = bf16_round(r2)
    return h, m, l, r1, r2


def sample(seed, n):
    rng = np.random.default_rng(seed)
    mant = rng.standard_normal(n).astype(np.float32)
    scale = np.float32(2.0) ** rng.integers(-60, 60, n).astype(np.float32)
    x = (mant * scale).astype(np.float32)
    x[:8] = [0.0, -0.0, 1.0, -1.0, 3.0e38, -3.0e38, 1.17549435e-38, 16777215.0]
    return x


def test_three_pieces_represent_the_operand_exactly():
    x = sample(1, 200_000)
    h, m, l, r1, r2 = cut(x)
    # each subtraction is exact (the rest is representable), and the last rest fits a bf16
    assert np.array_equal(r1.astype(np.float64), x.astype(np.float64) - h.astype(np.float64))
    assert np.array_equal(r2.astype(np.float64), r1.astype(np.float64) - m.astype(np.float64))
    assert np.array_equal(l, r2)
    assert np.array_equal(h.astype(np.float64) + m.astype(np.float64) + l.astype(np.float64), x.astype(np.float64))
    # sizes of the pieces: each at most 2^-8 of the one before (round to nearest: 2^-9 of it)
    ax = np.abs(x.astype(np.float64))
    assert (np.abs(m.astype(np.float64)) <= ax * 2.0 ** -8).all()
    assert (np.abs(l.astype(np.float64)) <= ax * 2.0 ** -16).all()


def test_the_six_products_kept_are_within_three_units_of_2_to_the_minus_24():
    x, y = sample(2, 100_000), sample(3, 100_000)
    x, y = np.clip(x, -1e18, 1e18), np.clip(y, -1e18, 1e18)      # keep the products finite
    hx, mx, lx, _, _ = cut(x)
    hy, my, ly, _, _ = cut(y)
    f = lambda a: a.astype(np.float64)
    kept = f(mx) * f(my) + f(hx) * f(ly) + f(lx) * f(hy) + f(hx) * f(my) + f(mx) * f(hy) + f(hx) * f(hy)
    full = f(x) * f(y)
    assert (np.abs(kept - full) <= 3.0 * 2.0 ** -24 * np.abs(full) + 1e-300).all()


def test_distances_from_the_kept_products_match_fp64():
    rng = np.random.default_rng(4)
    for count, d, mean in ((45, 20_000, 0.0), (45, 20_000, 30.0), (105, 5_000, 0.5)):
        X = (rng.standard_normal((count, d)) * 0.03 + mean).astype(np.float32)
        Xc = (X - X[3]).astype(np.float32)                       # centred on a reference row, in fp32
        h, m, l, _, _ = cut(Xc)
        H, M, L = h.astype(np.float64), m.astype(np.float64), l.astype(np.float64)
        G = M @ M.T + (H @ L.T + L @ H.T) + (H @ M.T + M @ H.T) + H @ H.T
        g = np.diag(G)
        D = g[:, None] + g[None, :] - 2.0 * G
        Xd = X.astype(np.float64)
        ref = ((Xd[:, None, :] - Xd[None, :, :]) ** 2).sum(-1) if count <= 45 else None
        if ref is None:
            Ge = Xd @ Xd.T
            ge = np.diag(Ge)
            ref = ge[:, None] + ge[None, :] - 2.0 * Ge
            tol = 1e-7                                            # the fp64 identity itself at this offset
        else:
            tol = 1e-8
        assert np.abs(D - ref).max() <= tol * ref.max()
