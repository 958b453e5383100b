"""Pins for the oracle's other formats (Sec. 4.3): dual-grid and codebook projections."""
import itertools

import numpy as np
import pytest

import synth_inputs as si
from oracle import admmq_oracle as orc


def _problem(n=24, p=10, N=96, seed=3):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, n)) * np.exp(rng.standard_normal(n))
    W0 = rng.standard_normal((n, p)) * 0.02
    return X.T @ X, W0


def test_dual_grid_without_outliers_is_the_uniform_grid():
    _, W0 = _problem()
    mask = np.zeros(W0.shape, dtype=bool)
    for g in (0, 8):
        fmt = orc.DualGridProjection.fit(W0, 3, mask, g)
        grid = orc.Grid.fit(W0, 3, g)
        x = W0 * 1.3 + 0.001
        k, xq = fmt.project(x)
        np.testing.assert_array_equal(k, grid.codes(x))
        np.testing.assert_array_equal(xq, grid.dequant(grid.codes(x)))
        assert np.all(fmt.outlier.degenerate)            # nothing to fit: step 0, codes 0


def test_dual_grid_fits_each_subset_on_its_own_range():
    rng = np.random.default_rng(0)
    W0 = rng.standard_normal((16, 3))
    mask = np.abs(W0) > 1.0
    fmt = orc.DualGridProjection.fit(W0, 2, mask, 8)
    for gi in range(2):
        for j in range(3):
            blk, m = W0[gi * 8:(gi + 1) * 8, j], mask[gi * 8:(gi + 1) * 8, j]
            for sel, gr in ((~m, fmt.inlier), (m, fmt.outlier)):
                if sel.any():
                    assert gr.z0[gi, j] == blk[sel].min()
                    assert gr.delta[gi, j] == (blk[sel].max() - blk[sel].min()) / 3
                else:
                    assert gr.delta[gi, j] == 0.0 and gr.z0[gi, j] == 0.0
    # every entry lands on the grid of its own subset, and W0's subset extremes are reproduced exactly
    k, xq = fmt.project(W0)
    lo_in = np.where(~mask, W0, np.inf).reshape(2, 8, 3).min(axis=1)
    assert np.all(np.isin(lo_in[np.isfinite(lo_in)], xq))
    # brute force: nearest level of the entry's own grid
    for i, j in itertools.product(range(16), range(3)):
        gr = fmt.outlier if mask[i, j] else fmt.inlier
        levels = gr.z0[i // 8, j] + gr.delta[i // 8, j] * np.arange(4)
        assert abs(W0[i, j] - xq[i, j]) <= np.min(np.abs(W0[i, j] - levels)) + 1e-15


def test_dual_grid_beats_one_grid_on_heavy_tails():
    # the outliers no longer stretch the inliers' range: the plain projection error can only go down
    rng = np.random.default_rng(1)
    W0 = rng.standard_normal((64, 6)) * 0.02
    W0[rng.integers(0, 64, 6), np.arange(6)] *= 12.0
    mask = si.outlier_mask(W0, 0.05)
    assert mask.sum(axis=0).tolist() == [4] * 6
    one = orc.Grid.fit(W0, 3)
    two = orc.DualGridProjection.fit(W0, 3, mask)
    e1 = np.sum((one.dequant(one.codes(W0)) - W0) ** 2)
    e2 = np.sum((two.project(W0)[1] - W0) ** 2)
    assert e2 < 0.5 * e1


def test_codebook_on_uniform_levels_is_the_uniform_grid():
    _, W0 = _problem()
    grid = orc.Grid.fit(W0, 3)
    cb = grid.z0 + grid.delta * np.arange(8)[:, None]           # [8][p]
    fmt = orc.CodebookProjection(cb)
    rng = np.random.default_rng(5)
    x = W0 + rng.standard_normal(W0.shape) * 0.01                # includes values outside the range: clamped
    k, xq = fmt.project(x)
    kg = grid.codes(x)
    # away from exact midpoints (where rint rounds to even and the codebook rule goes down) both agree
    t = (x - grid.z0) / grid.delta
    clear = np.abs(t - np.floor(t) - 0.5) > 1e-9
    np.testing.assert_array_equal(k[clear], kg[clear])
    np.testing.assert_allclose(xq[clear], grid.dequant(kg)[clear], rtol=0, atol=1e-15)


def test_codebook_projection_is_the_nearest_level_and_idempotent():
    rng = np.random.default_rng(2)
    W0 = rng.standard_normal((40, 5))
    cb = si.column_codebook(W0, 3).astype(np.float64)
    assert np.all(np.diff(cb, axis=0) > 0)
    fmt = orc.CodebookProjection(cb)
    x = rng.standard_normal((40, 5)) * 1.5
    k, xq = fmt.project(x)
    for i, j in itertools.product(range(40), range(5)):
        dist = [abs(x[i, j] - cb[l, j]) for l in range(8)]
        assert k[i, j] == int(np.argmin(dist))
        assert xq[i, j] == cb[k[i, j], j]
    k2, xq2 = fmt.project(xq)
    np.testing.assert_array_equal(k2, k)
    np.testing.assert_array_equal(xq2, xq)
    # a tie goes to the lower level
    mid = 0.5 * (cb[2, 0] + cb[3, 0])
    if abs(mid - cb[2, 0]) == abs(cb[3, 0] - mid):
        assert fmt.project(np.full((1, 5), mid))[0][0, 0] == 2


def test_kept_entries_pass_through_and_carry_no_dual():
    H, W0 = _problem()
    free = si.outlier_mask(W0, 0.1)
    fmt = orc.CodebookProjection(si.column_codebook(W0, 2).astype(np.float64), free)
    x = W0 * 1.1
    k, xq = fmt.project(x)
    np.testing.assert_array_equal(xq[free], x[free])
    assert np.all(k[free] == 0)
    a, j_admm, j_near = orc.quantize_layer_format(H, W0, fmt, T=30)
    # a kept entry has D = W + V/rho, hence V_new = V + rho (W - D) = 0: the residual there is zero from t = 1 on,
    # and the result's kept entries are whatever the continuous iterate holds, not a level
    levels = si.column_codebook(W0, 2).astype(np.float64)
    on_level = np.isclose(a.Wq[None], levels[:, None, :], rtol=0, atol=1e-12).any(axis=0)
    assert np.all(on_level[~free])
    assert not np.all(on_level[free])
    assert j_admm < j_near


@pytest.mark.parametrize("kind", ["dual", "codebook", "codebook_free"])
def test_key_inequality_and_gain_over_plain_projection(kind):
    H, W0 = _problem(n=32, p=12, N=128, seed=7)
    if kind == "dual":
        fmt = orc.DualGridProjection.fit(W0, 2, si.outlier_mask(W0, 0.07), 16)
    else:
        free = si.outlier_mask(W0, 0.05) if kind == "codebook_free" else None
        fmt = orc.CodebookProjection(si.column_codebook(W0, 2).astype(np.float64), free)
    a, j_admm, j_near = orc.quantize_layer_format(H, W0, fmt, T=60)
    # App. C: D^{t+1} is a projection of Wt, D^t is feasible, so ||D^{t+1} - Wt|| <= ||D^t - Wt|| from t = 1 on
    for t in range(1, 60):
        assert a.key_lhs[t] <= a.key_rhs[t] * (1 + 1e-12) + 1e-18
    assert j_admm < j_near
    # the first iterate is the plain projection of W0 (W^(1) = Ws, V = 0)
    k0, _ = orc.project_unscaled(fmt, W0)
    np.testing.assert_array_equal(a.first_codes, k0)


@pytest.mark.parametrize("kind", ["dual", "codebook_free"])
def test_fp32_mirror_follows_the_float64_projection(kind):
    rng = np.random.default_rng(11)
    n, p = 32, 12
    W0 = (rng.standard_normal((n, p)) * 0.02).astype(np.float32).astype(np.float64)
    d = np.exp(rng.standard_normal(n) * 0.3)
    if kind == "dual":
        fmt = orc.DualGridProjection.fit(W0, 3, si.outlier_mask(W0, 0.07), 16)
    else:
        fmt = orc.CodebookProjection(si.column_codebook(W0, 3).astype(np.float64), si.outlier_mask(W0, 0.05))
    W = (d[:, None] * W0 + rng.standard_normal((n, p)) * 0.003).astype(np.float32)
    V = (rng.standard_normal((n, p)) * 0.001).astype(np.float32)
    rho, rho_next = 0.3, 0.33
    k32, Vn, Bn, xq, ss = orc.project_dual_step_format_f32(W, V, rho, rho_next, d, fmt)
    k64, Dn, Wt = orc.d_update(W.astype(np.float64), V.astype(np.float64), rho, d.astype(np.float32).astype(np.float64), fmt)
    assert np.mean(k32 != k64) < 0.02                      # only entries within rounding of a boundary may differ
    same = k32 == k64
    V64 = V + rho * (W - Dn)
    scale = np.abs(W).max()
    np.testing.assert_allclose(Vn[same], V64[same], rtol=0, atol=2e-6 * scale)
    np.testing.assert_allclose(Bn[same], (Dn - V64 / rho_next)[same], rtol=0, atol=4e-6 * scale)
    if kind == "codebook_free":
        assert np.all(Vn[fmt.free] == 0.0)
