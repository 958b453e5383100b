"""Pins for the oracle's pair-swap local search (Sec. 3.5): eq. 11 against recomputed objectives,
gradient maintenance, monotone descent, separable case, and exhaustive enumeration on tiny layers."""
import itertools

import numpy as np
import pytest

from oracle import admmq_oracle as orc


def small_problem(n, p, bits, seed, g=0, N=None):
    rng = np.random.default_rng(seed)
    N = N or 3 * n
    X = rng.standard_normal((N, n)) * np.exp(0.7 * rng.standard_normal(n))
    X[:, 1:] += 0.6 * X[:, :-1]                      # correlated channels: off-diagonal H matters
    W0 = rng.standard_normal((n, p))
    Hd, _ = orc.damp_hessian(orc.hessian([X]))
    grid = orc.Grid.fit(W0, bits, g)
    return Hd, W0, grid


def test_eq11_equals_recomputed_objective_difference_for_every_candidate():
    Hd, W0, grid = small_problem(8, 5, 3, seed=1, g=4)
    rng = np.random.default_rng(7)
    codes = rng.integers(0, 8, size=W0.shape)
    Wq = grid.dequant(codes)
    G = Hd @ (W0 - Wq)
    base = np.array([(Wq[:, j] - W0[:, j]) @ Hd @ (Wq[:, j] - W0[:, j]) for j in range(5)])
    for i1, i2 in itertools.permutations(range(8), 2):
        dL, d1, d2 = orc.pair_gains(Hd, G, codes, grid, i1, i2)
        for c, (s1, s2) in enumerate(((1, 1), (1, -1), (-1, 1), (-1, -1))):
            for j in range(5):
                k = codes[:, j].copy()
                k[i1] += s1
                k[i2] += s2
                if k[i1] < 0 or k[i1] > 7 or k[i2] < 0 or k[i2] > 7:
                    assert np.isinf(dL[c, j])
                    continue
                col = grid.dequant(np.repeat(k[:, None], 5, axis=1))[:, j]
                new = (col - W0[:, j]) @ Hd @ (col - W0[:, j])
                assert dL[c, j] == pytest.approx(new - base[j], rel=1e-9, abs=1e-9)


def test_gradient_maintenance_monotone_descent_and_bookkeeping():
    Hd, W0, grid = small_problem(24, 9, 3, seed=2, g=8)
    k0, Wq0 = orc.rtn(W0, grid)
    j0 = orc.objective(Hd, W0, Wq0)
    res = orc.local_search(Hd, W0, k0, grid, rounds=3, pairs_per_batch=16, seed=5)
    assert res.moves > 0
    Wq = grid.dequant(res.codes)
    assert np.allclose(res.G, Hd @ (W0 - Wq), rtol=1e-10, atol=1e-10)
    j1 = orc.objective(Hd, W0, Wq)
    assert j1 < j0
    assert j0 - j1 == pytest.approx(res.objective_drop, rel=1e-9)
    assert res.codes.min() >= 0 and res.codes.max() <= 7
    assert all(a[5] > 0 for a in res.applied)
    assert np.count_nonzero(res.codes != k0) <= res.entries_changed
    # replay: every applied pair lowers the objective by exactly its recorded total
    again = orc.local_search(Hd, W0, k0, grid, rounds=3, pairs_per_batch=16, seed=5)
    assert np.array_equal(again.codes, res.codes)


def test_diagonal_hessian_rtn_is_fixed_point():
    rng = np.random.default_rng(4)
    n, p = 10, 6
    Hd = np.diag(np.exp(rng.standard_normal(n)))
    W0 = rng.standard_normal((n, p))
    grid = orc.Grid.fit(W0, 3, 0)
    k0, _ = orc.rtn(W0, grid)
    res = orc.local_search(Hd, W0, k0, grid, rounds=2, pairs_per_batch=32, seed=1)
    assert res.moves == 0 and np.array_equal(res.codes, k0)


def all_pairs(n):
    return lambda r, m: list(itertools.permutations(range(n), 2))


def enumerate_columns(Hd, W0, grid, n, bits):
    """Exhaustive minimum of eq. 2 over all (2^b)^n code vectors, per column."""
    L = 2 ** bits
    combos = np.array(list(itertools.product(range(L), repeat=n)))          # [L^n][n]
    best = []
    for j in range(W0.shape[1]):
        vals = grid.z0[0, j] + combos * grid.delta[0, j]
        E = vals - W0[:, j][None, :]
        obj = np.einsum("ci,ij,cj->c", E, Hd, E)
        best.append((float(obj.min()), combos[int(np.argmin(obj))]))
    return best


@pytest.mark.parametrize("n,seed", [(4, 0), (5, 1), (6, 2), (6, 3)])
def test_tiny_layers_against_exhaustive_enumeration(n, seed):
    bits, p = 2, 3
    Hd, W0, grid = small_problem(n, p, bits, seed=seed, N=4 * n)
    best = enumerate_columns(Hd, W0, grid, n, bits)
    j_opt = sum(b[0] for b in best)
    # (a) from RTN, run to exhaustion with every pair in every batch: never below the optimum,
    #     never above the start
    k0, Wq0 = orc.rtn(W0, grid)
    res = orc.local_search(Hd, W0, k0, grid, rounds=200, batches_per_round=1, pairs_fn=all_pairs(n))
    j_ls = orc.objective(Hd, W0, grid.dequant(res.codes))
    assert j_opt <= j_ls * (1 + 1e-12) <= orc.objective(Hd, W0, Wq0) * (1 + 1e-12)
    # (b) at exhaustion no pair move of the neighbourhood lowers any column's loss
    G = Hd @ (W0 - grid.dequant(res.codes))
    for i1, i2 in itertools.permutations(range(n), 2):
        dL, _, _ = orc.pair_gains(Hd, G, res.codes, grid, i1, i2)
        assert np.all(dL >= -1e-12)
    # (c) the global optimum is a fixed point
    kopt = np.stack([b[1] for b in best], axis=1)
    fix = orc.local_search(Hd, W0, kopt, grid, rounds=3, batches_per_round=1, pairs_fn=all_pairs(n))
    assert fix.moves == 0 and np.array_equal(fix.codes, kopt)


def test_layer_end_to_end_ordering_small():
    rng = np.random.default_rng(8)
    n, p, N = 48, 16, 200
    X = rng.standard_normal((N, n)) * np.exp(rng.standard_normal(n))
    X[:, 2:] += 0.5 * X[:, :-2]
    W0 = 0.02 * rng.standard_normal((n, p))
    H = orc.hessian([X])
    res = orc.quantize_layer(H, W0, bits=3, group_size=16, T=80, ls_rounds=3, ls_pairs=16, seed=3)
    assert res.j_damp <= res.j_damp_admm <= res.j_damp_rtn
    assert res.j_damp == pytest.approx(orc.objective(orc.damp_hessian(H)[0], W0, res.Wq), rel=1e-12)
    assert res.j_recon == pytest.approx(float(np.sum((X @ (res.Wq - W0)) ** 2)), rel=1e-9)
    assert res.codes.min() >= 0 and res.codes.max() <= 7
    assert np.allclose(res.Wq, np.repeat(res.zeros, 16, axis=0) + res.codes * np.repeat(res.scales, 16, axis=0))
