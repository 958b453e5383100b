"""Helpers shared by the GPU parity tests: device tensors from NumPy arrays, seeded small problems."""
import numpy as np


def to_dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def bf16_bits_to_dev(bits):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def correlated_problem(n, p, N, seed, sigma_w=0.02, outliers=0):
    """A seeded layer with log-normal channel scales and neighbour-correlated channels (fp32 X)."""
    rng = np.random.default_rng(seed)
    s = np.exp(rng.standard_normal(n))
    if outliers:
        s[rng.choice(n, outliers, replace=False)] *= 20.0
    X = rng.standard_normal((N, n)).astype(np.float32)
    X[:, 1:] += np.float32(0.5) * X[:, :-1]
    X = (X * s.astype(np.float32)).astype(np.float32)
    W0 = (sigma_w * rng.standard_normal((n, p))).astype(np.float32)
    return X, W0


def assert_differs_only_at_midpoints(k, k64, Wt, d, sc, zr, g):
    """fp32 codes k against the float64 projection k64 of eq. 10.  The kernel forms t = ((W + V/rho)/d_i - z0)/delta
    from three reciprocals and five further fp32 operations; the error that reaches t is a few units of 2^-24 of
    (|x| + |z0|)/delta, x the unscaled target (the subtraction x - z0 keeps the absolute error of x).  So the two
    may differ only where float64's t lies within 2^-22 (|x| + |z0|)/delta of a rounding midpoint, about 1e-6 to
    1e-5 for these grids; a fraction of about twice that band of all entries lies that near a midpoint at all."""
    n = k.shape[0]
    gg = n if g == 0 else g
    diff = k64 != k
    if diff.any():
        x = Wt / d[:, None].astype(np.float64)
        ze = np.repeat(zr.astype(np.float64), gg, 0)
        se = np.repeat(sc.astype(np.float64), gg, 0)
        live = se[diff] > 0
        assert live.all()                                   # a degenerate group's codes are 0 on both sides
        t = (x[diff] - ze[diff]) / se[diff]
        band = 2.0 ** -22 * (np.abs(x[diff]) + np.abs(ze[diff])) / se[diff]
        assert np.all(np.abs(t - np.floor(t) - 0.5) < band)
        assert np.all(np.abs(k64[diff] - k[diff].astype(np.int64)) == 1)
    assert diff.sum() <= max(2, 1e-5 * diff.size)
