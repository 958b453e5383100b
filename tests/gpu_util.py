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
