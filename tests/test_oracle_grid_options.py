"""Pins for the oracle's symmetric grids and MSE clipping search (paper Sec. 3.4 "Clipping heuristics", App. D)."""
import numpy as np
import pytest

from oracle import admmq_oracle as orc


def weights(seed=0, n=32, p=6, heavy=True):
    rng = np.random.default_rng(seed)
    W = rng.standard_normal((n, p))
    if heavy:
        W[rng.integers(0, n, 3), rng.integers(0, p, 3)] *= 6.0      # a few outliers: clipping should pay
    return W


@pytest.mark.parametrize("g", [0, 8])
def test_no_options_is_the_plain_min_max_fit(g):
    W = weights()
    a = orc.Grid.fit(W, 3, g)
    d, z = orc.grid_fit_options(W, 3, g, False, 0)
    assert np.array_equal(a.delta, d) and np.array_equal(a.z0, z)


@pytest.mark.parametrize("bits,g", [(2, 0), (3, 8), (4, 16)])
def test_symmetric_levels_are_symmetric_about_zero_and_cover_the_data(bits, g):
    W = weights(seed=1)
    grid = orc.Grid.fit(W, bits, g, symmetric=True)
    L = 2 ** bits - 1
    n = W.shape[0]
    gg = n if g == 0 else g
    lo = grid.z0
    hi = grid.z0 + L * grid.delta
    assert np.allclose(lo, -hi)
    amax = np.abs(W.reshape(n // gg, gg, -1)).max(axis=1)
    assert np.allclose(hi, amax)
    k = grid.codes(W)
    assert np.allclose(grid.dequant(L - k), -grid.dequant(k))
    assert np.all(np.abs(grid.dequant(k) - W) <= 0.5 * np.repeat(grid.delta, gg, 0) + 1e-12)


@pytest.mark.parametrize("sym,g,bits", [(False, 0, 3), (True, 8, 2), (False, 16, 4)])
def test_clipping_search_picks_the_best_candidate_brute_force(sym, g, bits):
    W = weights(seed=2)
    n, p = W.shape
    gg = n if g == 0 else g
    P, shrink = 100, 0.8
    delta, z0 = orc.grid_fit_options(W, bits, g, sym, P, shrink)
    L = 2 ** bits - 1
    for r in range(n // gg):
        for j in range(p):
            x = W[r * gg:(r + 1) * gg, j]
            mn, mx = x.min(), x.max()
            if sym:
                a = max(abs(mn), abs(mx))
                mn, mx = -a, a
            errs = []
            for i in range(int(shrink * P)):
                rr = 1.0 - i / P
                levels = rr * mn + np.arange(L + 1) * (rr * (mx - mn) / L)
                errs.append(np.sum(np.min((levels[None, :] - x[:, None]) ** 2, axis=1)))
            best = int(np.argmin(errs))                                # argmin: first minimiser
            rr = 1.0 - best / P
            assert z0[r, j] == pytest.approx(rr * mn, rel=1e-12, abs=1e-15)
            assert delta[r, j] == pytest.approx(rr * (mx - mn) / L, rel=1e-12)
            assert errs[best] <= errs[0]
    assert np.any(delta < orc.grid_fit_options(W, bits, g, sym, 0)[0])   # the outliers make clipping win somewhere


def test_layer_runs_on_a_clipped_symmetric_grid():
    rng = np.random.default_rng(4)
    n, p, N = 32, 10, 120
    X = rng.standard_normal((N, n)) * np.exp(rng.standard_normal(n))
    W0 = 0.02 * weights(seed=3, n=n, p=p)
    H = orc.hessian([X])
    res = orc.quantize_layer(H, W0, 3, 8, T=40, ls_rounds=1, ls_pairs=8, symmetric=True, clip_points=100)
    assert res.codes.min() >= 0 and res.codes.max() <= 7
    assert res.j_damp <= res.j_damp_admm
    assert np.allclose(res.zeros, -3.5 * res.scales)
