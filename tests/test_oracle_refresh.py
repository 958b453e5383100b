"""Pins for the oracle's grid refresh (paper Sec. 3.3 "Grid refresh", App. B): acceptance by eq. 12, dual
consistency, the key inequality of App. C through the refresh iteration, and "at most one accepted refresh"."""
import numpy as np
import pytest

from oracle import admmq_oracle as orc


def problem(seed=3, n=40, p=12, N=120, bits=3, g=0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, n)) * np.exp(0.8 * rng.standard_normal(n))
    X[:, 1:] += 0.7 * X[:, :-1]
    W0 = rng.standard_normal((n, p)) * 0.02
    Hd, _ = orc.damp_hessian(orc.hessian([X]))
    return Hd, W0, orc.Grid.fit(W0, bits, g)


@pytest.mark.parametrize("g", [0, 8])
def test_refresh_acceptance_is_eq12_and_state_is_consistent(g):
    Hd, W0, grid = problem(g=g)
    T, it = 40, 6
    base = orc.admm(Hd, W0, grid, T=it)                      # state just before the attempt
    res = orc.admm(Hd, W0, grid, T=T, refresh_iter=it)
    assert res.refresh_tried == 1
    accepted = res.refresh_accepted_at == it
    assert accepted == (res.refresh_err_new <= res.refresh_err_old)
    # independent recomputation of the attempt from the state of a run stopped at `it`
    d, Hs, Ws = orc.scale_problem(Hd, W0)
    lam, U = np.linalg.eigh(Hs)
    # replay iterations 0..it-1 by hand to get D, V (unrolled eqs. 7-9; no refresh before `it`)
    D, V, rho = Ws.copy(), np.zeros_like(Ws), 0.1
    for t in range(it):
        W = np.linalg.solve(Hs + rho * np.eye(len(d)), Hs @ Ws + rho * D - V)
        Wt = W + V / rho
        k = grid.codes(Wt / d[:, None])
        Dn = d[:, None] * grid.dequant(k)
        V = V + rho * (W - Dn)
        D, rho = Dn, rho * 1.1
    assert np.array_equal(grid.codes(D / d[:, None]), base.codes)
    W = np.linalg.solve(Hs + rho * np.eye(len(d)), Hs @ Ws + rho * D - V)
    Wt = W + V / rho
    x = Wt / d[:, None]
    gg = x.shape[0] if g == 0 else g
    xg = x.reshape(x.shape[0] // gg, gg, -1)
    new = orc.Grid(delta=(xg.max(1) - xg.min(1)) / 7.0, z0=xg.min(1), bits=3, degenerate=xg.max(1) <= xg.min(1))
    D_old = d[:, None] * grid.dequant(grid.codes(x))
    D_new = d[:, None] * new.dequant(new.codes(x))
    assert res.refresh_err_old == pytest.approx(float(np.sum((D_old - Wt) ** 2)), rel=1e-9)
    assert res.refresh_err_new == pytest.approx(float(np.sum((D_new - Wt) ** 2)), rel=1e-9)
    if accepted:
        # the grid in force is the refitted one; it spans the target exactly (min and max are grid points)
        assert np.allclose(res.grid.z0, xg.min(1)) and np.allclose(res.grid.delta, new.delta)
    else:
        assert res.grid is grid
    # key inequality of App. C holds at every iteration after the first, the refresh iteration included
    for lhs, rhs in list(zip(res.key_lhs, res.key_rhs))[1:]:
        assert lhs <= rhs * (1 + 1e-12) + 1e-30
    assert res.primal[-1] < 1e-3 * res.primal[1]
    assert np.array_equal(res.codes, res.grid.codes(res.Wq))


def test_dual_after_accepted_refresh_equals_one_step_update():
    """V + rho (W - D_old) + rho (D_old - D_new) must be V + rho (W - D_new): the continued run from the
    refresh iteration with the new grid and the one-step dual gives the same trajectory."""
    Hd, W0, grid = problem(seed=5, g=8)
    it, T = 4, 30
    res = orc.admm(Hd, W0, grid, T=T, refresh_iter=it)
    if res.refresh_accepted_at < 0:
        pytest.skip("refresh rejected for this seed")
    d, Hs, Ws = orc.scale_problem(Hd, W0)
    D, V, rho = Ws.copy(), np.zeros_like(Ws), 0.1
    cur = grid
    for t in range(T):
        W = np.linalg.solve(Hs + rho * np.eye(len(d)), Hs @ Ws + rho * D - V)
        Wt = W + V / rho
        if t == it:
            cur = orc.refit_grid(Wt / d[:, None], grid)
        k = cur.codes(Wt / d[:, None])
        Dn = d[:, None] * cur.dequant(k)
        V = V + rho * (W - Dn)
        D, rho = Dn, rho * 1.1
    assert np.array_equal(k, res.codes)


def test_refresh_never_tried_by_default_and_only_once():
    Hd, W0, grid = problem(seed=7)
    a = orc.admm(Hd, W0, grid, T=20)
    assert a.refresh_tried == 0 and a.refresh_accepted_at == -1 and a.grid is grid
    b = orc.admm(Hd, W0, grid, T=20, refresh_iter=3)
    assert b.refresh_tried == 1


def test_layer_with_refresh_keeps_bookkeeping_consistent():
    rng = np.random.default_rng(8)
    n, p, N = 48, 16, 200
    X = rng.standard_normal((N, n)) * np.exp(rng.standard_normal(n))
    X[:, 2:] += 0.5 * X[:, :-2]
    W0 = 0.02 * rng.standard_normal((n, p))
    H = orc.hessian([X])
    res = orc.quantize_layer(H, W0, bits=3, group_size=16, T=60, ls_rounds=2, ls_pairs=16, seed=3, refresh_iter=10)
    assert np.allclose(res.Wq, np.repeat(res.zeros, 16, axis=0) + res.codes * np.repeat(res.scales, 16, axis=0))
    assert res.j_damp <= res.j_damp_admm
    assert res.j_damp == pytest.approx(orc.objective(orc.damp_hessian(H)[0], W0, res.Wq), rel=1e-12)


def test_a_late_refresh_amplifies_rounding_of_the_w_update():
    """Why an fp32 implementation cannot be held to the base algorithm's 0.5 % objective bar when the refresh is
    tried late: the refitted grid hangs on the two extreme entries of each group of the projection target, so a
    relative perturbation of 2e-6 of every W-update (a fifth of the 1e-5 the W-update is allowed) moves the
    float64 oracle's own end objective by close to 1 % with the attempt at iteration 12, against a few 1e-4
    without a refresh.  The GPU test of that case therefore carries a wider tolerance."""
    import sys
    import os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from gpu_util import correlated_problem
    n, p, N, bits, g, seed = 256, 130, 300, 4, 64, 5
    X, W0 = correlated_problem(n, p, N, seed, outliers=2)
    H = orc.hessian([X.astype(np.float64)])
    exact = orc.w_update
    spread = {}
    try:
        for it in (-1, 12):
            js = []
            for s in range(4):
                rng = np.random.default_rng(200 + s)
                orc.w_update = lambda *a, _r=rng: (lambda W: W * (1 + 2e-6 * _r.standard_normal(W.shape)))(exact(*a))
                js.append(orc.quantize_layer(H, W0.astype(np.float64), bits, g, T=80, ls_rounds=0,
                                             refresh_iter=it).j_damp_admm)
            spread[it] = (max(js) - min(js)) / np.mean(js)
    finally:
        orc.w_update = exact
    print(spread)
    assert spread[-1] < 1e-3
    assert spread[12] > 3 * spread[-1] and spread[12] > 2e-3
