"""Pins for the oracle's problem set-up and ADMM loop (none of them re-types the oracle's formula)."""
import itertools

import numpy as np
import pytest

import synth_inputs as si
from oracle import admmq_oracle as orc


def tiny_problem(n=12, p=5, N=40, seed=3, bits=3, g=0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((N, n)) * np.exp(rng.standard_normal(n))
    W0 = rng.standard_normal((n, p)) * 0.02
    return X, W0


def cfg1_problem():
    cfg = si.CONFIGS["cfg1"]
    H = orc.hessian(si.chunk_as_f64(cfg, xc) for _, xc in si.iter_x_chunks(cfg))
    W0 = si.layer_weights(cfg).astype(np.float64)
    return cfg, H, W0


def test_hessian_is_xtx_triple_loop_and_chunking():
    X, _ = tiny_problem(n=5, N=9)
    H = orc.hessian([X])
    ref = np.zeros((5, 5))
    for i in range(5):
        for j in range(5):
            for r in range(9):
                ref[i, j] += X[r, i] * X[r, j]
    assert np.allclose(H, ref, rtol=1e-13, atol=1e-13)
    assert np.array_equal(H, H.T)
    Hc = orc.hessian([X[:4], X[4:7], X[7:]])
    assert np.allclose(Hc, H, rtol=1e-13)


def test_damping_is_fraction_of_mean_diagonal():
    X, _ = tiny_problem()
    H = orc.hessian([X])
    Hd, lam = orc.damp_hessian(H, 0.01)
    assert lam == pytest.approx(0.01 * np.mean(np.sum(X * X, axis=0)))
    assert np.allclose(Hd - H, lam * np.eye(H.shape[0]))


def test_scaled_hessian_unit_diagonal_and_objective_invariance():
    X, W0 = tiny_problem()
    Hd, _ = orc.damp_hessian(orc.hessian([X]))
    d, Hs, Ws = orc.scale_problem(Hd, W0)
    assert np.allclose(np.diag(Hs), 1.0, rtol=0, atol=1e-14)
    # Sigma change of variables leaves the objective unchanged (eqs. 2 and 3)
    rng = np.random.default_rng(0)
    Wq = W0 + 0.003 * rng.standard_normal(W0.shape)
    j_unscaled = orc.objective(Hd, W0, Wq)
    j_scaled = orc.objective(Hs, Ws, Wq * d[:, None])
    assert j_scaled == pytest.approx(j_unscaled, rel=1e-12)
    # and equals the reconstruction form of eq. 1 (damped)
    lam = Hd[0, 0] - orc.hessian([X])[0, 0]
    direct = np.sum((X @ (Wq - W0)) ** 2) + lam * np.sum((Wq - W0) ** 2)
    assert j_unscaled == pytest.approx(direct, rel=1e-12)


def test_dead_channel_raises():
    X, W0 = tiny_problem()
    X[:] = 0.0
    Hd, _ = orc.damp_hessian(orc.hessian([X]))
    with pytest.raises(ValueError):
        orc.scale_problem(Hd, W0)


@pytest.mark.parametrize("bits,g", [(2, 0), (3, 4), (4, 0)])
def test_projection_is_nearest_level_brute_force(bits, g):
    rng = np.random.default_rng(5)
    n, p = 12, 7
    W0 = rng.standard_normal((n, p))
    grid = orc.Grid.fit(W0, bits, g)
    x = W0 + 0.6 * rng.standard_normal((n, p))          # some targets fall outside the range
    k = grid.codes(x)
    gg = n if g == 0 else g
    for i in range(n):
        for j in range(p):
            levels = grid.z0[i // gg, j] + np.arange(2 ** bits) * grid.delta[i // gg, j]
            assert k[i, j] == int(np.argmin(np.abs(levels - x[i, j])))
    # grid end points are the group's min and max
    Wg = W0.reshape(n // gg, gg, p)
    assert np.allclose(grid.z0, Wg.min(axis=1))
    assert np.allclose(grid.z0 + (2 ** bits - 1) * grid.delta, Wg.max(axis=1))


def test_degenerate_group_codes_zero():
    W0 = np.full((8, 3), 0.25)
    W0[:, 1] = np.linspace(-1, 1, 8)
    grid = orc.Grid.fit(W0, 3, 0)
    assert grid.degenerate.tolist() == [[True, False, True]]
    k = grid.codes(W0 + 5.0)
    assert np.all(k[:, 0] == 0) and np.all(k[:, 2] == 0)
    assert np.allclose(grid.dequant(k)[:, 0], 0.25)
    assert grid.delta[0, 0] == 0.0 and grid.delta[0, 1] > 0


def test_w_update_solves_eq7_linear_system():
    X, W0 = tiny_problem(n=40, p=6, N=100)
    Hd, _ = orc.damp_hessian(orc.hessian([X]))
    d, Hs, Ws = orc.scale_problem(Hd, W0)
    lam, U = np.linalg.eigh(Hs)
    rng = np.random.default_rng(1)
    D = Ws + 0.1 * rng.standard_normal(Ws.shape)
    V = 0.05 * rng.standard_normal(Ws.shape)
    for rho in (0.1, 3.0, 1e4):
        W = orc.w_update(U, lam, Hs @ Ws, D, V, rho)
        ref = np.linalg.solve(Hs + rho * np.eye(40), Hs @ Ws + rho * D - V)
        assert np.linalg.norm(W - ref) <= 1e-11 * np.linalg.norm(ref)


def test_first_iterate_is_dense_weights_and_rtn():
    """D0 = Ws, V0 = 0 make the first W-update return Ws exactly, so the first projection is
    round-to-nearest of W0 (Alg. 1 lines 4, 6, 7)."""
    cfg, H, W0 = cfg1_problem()
    Hd, _ = orc.damp_hessian(H)
    grid = orc.Grid.fit(W0, cfg.bits, cfg.group_size)
    res = orc.admm(Hd, W0, grid, T=1)
    # RTN computed here, directly in the unscaled space, by brute force over the levels
    levels = grid.z0[0][None, :, None] + np.arange(2 ** cfg.bits)[None, None, :] * grid.delta[0][None, :, None]
    k_rtn = np.argmin(np.abs(levels - W0[:, :, None]), axis=2)
    assert np.array_equal(res.first_codes, k_rtn)
    assert np.array_equal(orc.rtn(W0, grid)[0], k_rtn)


def test_second_iterate_in_closed_form_pins_the_dual_update_and_the_penalty_index():
    """Eqs. 7-9 over the first two iterations, written out from what the first iteration is known to be: the first
    W-update returns Ws (D0 = Ws, V0 = 0), so D1 = Sigma^{-1} RTN(W0), V1 = rho_0 (Ws - D1) by eq. 9, rho_1 = gamma
    rho_0, and W2 solves (Hs + rho_1 I) W2 = Hs Ws + rho_1 D1 - V1 (eq. 7, through a dense solve here, not the
    eigendecomposition).  The recorded residuals of a two-iteration run must be those of this closed form: a dual
    update with the sign flipped, with rho_1 in place of rho_0, or a W-update that takes the penalty of the wrong
    iteration, changes W2 and with it both residuals."""
    X, W0 = tiny_problem(n=24, p=7, N=70, seed=11)
    Hd, _ = orc.damp_hessian(orc.hessian([X]))
    grid = orc.Grid.fit(W0, 3, 0)
    rho0, gamma = 0.1, 1.1
    res = orc.admm(Hd, W0, grid, T=2, rho0=rho0, gamma=gamma)
    d = np.sqrt(np.diag(Hd))
    Hs = Hd / np.outer(d, d)
    Ws = W0 * d[:, None]
    levels = grid.z0[0][None, :, None] + np.arange(8)[None, None, :] * grid.delta[0][None, :, None]
    k1 = np.argmin(np.abs(levels - W0[:, :, None]), axis=2)               # round-to-nearest, brute force
    D1 = d[:, None] * np.take_along_axis(levels, k1[:, :, None], axis=2)[:, :, 0]
    V1 = rho0 * (Ws - D1)
    rho1 = gamma * rho0
    W2 = np.linalg.solve(Hs + rho1 * np.eye(len(d)), Hs @ Ws + rho1 * D1 - V1)
    x2 = (W2 + V1 / rho1) / d[:, None]
    k2 = np.argmin(np.abs(levels - x2[:, :, None]), axis=2)
    D2 = d[:, None] * np.take_along_axis(levels, k2[:, :, None], axis=2)[:, :, 0]
    assert res.rho == pytest.approx([rho0, rho1], rel=1e-15)
    assert res.primal[0] == pytest.approx(np.linalg.norm(Ws - D1), rel=1e-10)
    assert res.primal[1] == pytest.approx(np.linalg.norm(W2 - D2), rel=1e-9)
    assert res.dual[1] == pytest.approx(np.linalg.norm(D2 - D1), rel=1e-9)
    assert np.array_equal(res.codes, k2)
    assert np.any(k2 != k1)                                               # the second iterate has moved
    # the variants this is meant to catch do change the numbers (so the equalities above are not vacuous)
    for V_bad, rho_bad in ((-V1, rho1), (rho1 * (Ws - D1), rho1), (V1, rho0)):
        W_bad = np.linalg.solve(Hs + rho_bad * np.eye(len(d)), Hs @ Ws + rho_bad * D1 - V_bad)
        assert np.linalg.norm(W_bad - W2) > 1e-6 * np.linalg.norm(W2)


def test_key_inequality_residual_decay_and_rtn_no_worse_cfg1():
    cfg, H, W0 = cfg1_problem()
    Hd, _ = orc.damp_hessian(H)
    grid = orc.Grid.fit(W0, cfg.bits, cfg.group_size)
    res = orc.admm(Hd, W0, grid, T=200)
    # App. C key inequality, every iteration whose D^(t) is on the grid (D^(0) is the dense weights)
    for lhs, rhs in list(zip(res.key_lhs, res.key_rhs))[1:]:
        assert lhs <= rhs * (1 + 1e-12) + 1e-30
    # Thm. 1: rho_t * max(residuals) bounded, residual -> 0, codes freeze
    prim = np.array(res.primal)
    dual = np.array(res.dual)
    rho = np.array(res.rho)
    bound = rho * np.maximum(prim, dual)
    quarter = len(prim) // 4
    assert bound[quarter:].max() <= bound[:quarter].max()      # rho_t * residual stays below a constant
    assert prim[-1] <= 1e-3 * prim[1]
    assert np.all(dual[-20:] == 0.0)
    live = np.nonzero(prim > 1e-9 * prim[1])[0]                 # before the float64 round-off floor
    live = live[live >= np.argmax(bound)]
    slope = np.polyfit(np.log(rho[live]), np.log(prim[live]), 1)[0]
    assert slope <= -0.9
    # reconstruction objective no worse than RTN (expected from Fig. 3 / Table 6, not a theorem)
    j_admm = orc.objective(Hd, W0, res.Wq)
    j_rtn = orc.objective(Hd, W0, orc.rtn(W0, grid)[1])
    assert j_admm <= j_rtn
    j_admm_u = orc.objective(H, W0, res.Wq)
    assert j_admm_u <= orc.objective(H, W0, orc.rtn(W0, grid)[1])


def test_quiet_stop_ends_where_the_dual_residual_history_says_the_codes_froze():
    """The opt-in stopping rule (not in Alg. 1): stop once the codes have been constant for K iterations.  Pinned
    against the full run's own record of ||D^(t+1) - D^(t)||_F (zero exactly when no code changed): the stop falls at
    the first iteration that closes K zero entries in a row, and - the discrete iterates having converged there
    (Thm. 1) - the codes are those of the full run.  K = 0 changes nothing."""
    cfg, H, W0 = cfg1_problem()
    Hd, _ = orc.damp_hessian(H)
    grid = orc.Grid.fit(W0, cfg.bits, cfg.group_size)
    full = orc.admm(Hd, W0, grid, T=120)
    assert full.iters == 120
    same = orc.admm(Hd, W0, grid, T=120, quiet_stop=0)
    assert np.array_equal(same.codes, full.codes) and same.iters == 120
    dual = np.array(full.dual)
    for K in (1, 3, 8):
        run, expect = 0, None
        for t in range(1, len(dual)):
            run = run + 1 if dual[t] == 0.0 else 0
            if run >= K:
                expect = t + 1
                break
        assert expect is not None and expect < 120
        early = orc.admm(Hd, W0, grid, T=120, quiet_stop=K)
        assert early.iters == expect
        assert len(early.primal) == expect and early.primal == full.primal[:expect]
        if np.all(dual[expect:] == 0.0):                    # nothing moved afterwards in the full run
            assert np.array_equal(early.codes, full.codes)
    # a window that never closes runs all T iterations
    assert orc.admm(Hd, W0, grid, T=6, quiet_stop=50).iters == 6
    lay = orc.quantize_layer(H, W0, cfg.bits, cfg.group_size, T=120, ls_rounds=0, quiet_stop=3)
    assert lay.admm.iters < 120 and np.array_equal(lay.codes, full.codes)


def test_codes_invariant_under_hessian_rescaling_and_column_separable():
    cfg, H, W0 = cfg1_problem()
    grid = orc.Grid.fit(W0, cfg.bits, cfg.group_size)
    a = orc.admm(orc.damp_hessian(H)[0], W0, grid, T=30)
    b = orc.admm(orc.damp_hessian(4.0 * H)[0], W0, grid, T=30)   # power of two: exact rescale
    assert np.array_equal(a.codes, b.codes)
    cols = slice(5, 21)
    gs = orc.Grid.fit(W0[:, cols], cfg.bits, cfg.group_size)
    c = orc.admm(orc.damp_hessian(H)[0], W0[:, cols], gs, T=30)
    assert np.array_equal(c.codes, a.codes[:, cols])


def test_diagonal_hessian_makes_rtn_optimal_and_admm_returns_it():
    rng = np.random.default_rng(11)
    n, p = 10, 4
    Hd = np.diag(np.exp(rng.standard_normal(n)))
    W0 = rng.standard_normal((n, p))
    grid = orc.Grid.fit(W0, 2, 0)
    res = orc.admm(Hd, W0, grid, T=40)
    assert np.array_equal(res.codes, orc.rtn(W0, grid)[0])


def test_fp32_mirror_agrees_with_float64_projection_away_from_midpoints():
    cfg, H, W0 = cfg1_problem()
    Hd, _ = orc.damp_hessian(H)
    d, Hs, Ws = orc.scale_problem(Hd, W0)
    grid = orc.Grid.fit(W0, cfg.bits, cfg.group_size)
    rng = np.random.default_rng(2)
    W = (Ws + 0.2 * np.abs(Ws).mean() * rng.standard_normal(Ws.shape)).astype(np.float32)
    V = (0.01 * np.abs(Ws).mean() * rng.standard_normal(Ws.shape)).astype(np.float32)
    rho, rho_next = 0.5, 0.55
    k32, Vn, Bn, ss = orc.project_dual_step_f32(W, V, rho, rho_next, d, grid.delta, grid.z0,
                                                grid.degenerate, cfg.bits)
    k64, Dn, Wt = orc.d_update(W.astype(np.float64), V.astype(np.float64), rho, d, grid)
    t = (Wt / d[:, None] - grid.z0) / grid.delta
    near_mid = np.abs(t - np.floor(t) - 0.5) < 1e-4
    assert np.all((k32 == k64) | near_mid)
    assert np.mean(k32 != k64) < 1e-3
    ok = k32 == k64
    Vref = V.astype(np.float64) + rho * (W.astype(np.float64) - Dn)
    wmax = float(np.abs(W).max())
    assert np.allclose(Vn[ok], Vref[ok], rtol=1e-5, atol=2e-6 * wmax)
    Bref = Dn - Vref / rho_next
    assert np.allclose(Bn[ok], Bref[ok], rtol=1e-4, atol=4e-6 * wmax)
    assert ss == pytest.approx(float(np.sum((W.astype(np.float64) - Dn)[ok] ** 2)) +
                               float(np.sum((W.astype(np.float64) - d[:, None] * grid.dequant(k32.astype(np.int64)))[~ok] ** 2)),
                               rel=1e-5)


def test_splitmix_matches_published_vectors_and_pairs_are_valid():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "splitmix64_vectors.txt")
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        tok = line.split()
        seed = int(tok[0], 0)
        s = seed
        for want in tok[1:]:
            assert orc._mix64(s) == int(want, 0)
            s = (s + 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
    seen = set()
    for n in (2, 3, 7, 128):
        for slot in range(200):
            i1, i2 = orc.sample_pair(9, 1, 4, slot, n)
            assert 0 <= i1 < n and 0 <= i2 < n and i1 != i2
            seen.add((n, i1, i2))
    assert orc.sample_pair(9, 1, 4, 3, 128) == orc.sample_pair(9, 1, 4, 3, 128)
    assert len({orc.sample_pair(9, r, b, 0, 4096) for r in range(3) for b in range(50)}) > 140
