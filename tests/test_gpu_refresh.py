"""GPU parity of the grid refresh (paper Sec. 3.3, App. B) against the oracle: the attempt on identical inputs
(refitted grid, both sides of eq. 12, the decision), and the whole layer with one refresh iteration."""
import numpy as np
import pytest

from oracle import admmq_oracle as orc
from gpu_util import to_dev, correlated_problem

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu
OBJ_TOL = 5e-3


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_11222_amd as admmq
    c = admmq.Context(0)
    yield c
    c.close()


@pytest.mark.parametrize("n,p,bits,g,seed", [(96, 40, 3, 0, 1), (128, 70, 3, 32, 2), (64, 1030, 4, 16, 3), (48, 9, 2, 0, 4)])
def test_refresh_attempt_matches_oracle(ctx, n, p, bits, g, seed):
    rng = np.random.default_rng(seed)
    W0 = (0.02 * rng.standard_normal((n, p))).astype(np.float32)
    d = np.exp(0.5 * rng.standard_normal(n)).astype(np.float32)
    scales, zeros = ctx.grid_init(to_dev(W0), bits, g)
    sc0, zr0 = scales.cpu().numpy().copy(), zeros.cpu().numpy().copy()
    Ws = W0 * d[:, None]
    # a target whose range differs from the dense weights' (shrunk for some seeds, widened for others)
    shrink = 0.8 if seed % 2 else 1.15
    W = (shrink * Ws + 0.02 * np.abs(Ws).mean() * rng.standard_normal((n, p))).astype(np.float32)
    rho = 0.7
    V = (rho * 0.02 * np.abs(Ws).mean() * rng.standard_normal((n, p))).astype(np.float32)
    acc, eo, en = ctx.grid_refresh(to_dev(W), to_dev(V), to_dev(d), bits, g, rho, scales, zeros)
    # oracle, float64, same inputs
    d64 = d.astype(np.float64)
    old = orc.Grid(sc0.astype(np.float64), zr0.astype(np.float64), bits, sc0 == 0)
    Wt = W.astype(np.float64) + V.astype(np.float64) / rho
    x = Wt / d64[:, None]
    new = orc.refit_grid(x, old)
    D_old = d64[:, None] * old.dequant(old.codes(x))
    D_new = d64[:, None] * new.dequant(new.codes(x))
    eo_ref, en_ref = float(np.sum((D_old - Wt) ** 2)), float(np.sum((D_new - Wt) ** 2))
    assert eo == pytest.approx(eo_ref, rel=2e-4)
    assert en == pytest.approx(en_ref, rel=2e-4)
    assert abs(en_ref - eo_ref) > 1e-3 * eo_ref            # the case is not a near-tie
    assert acc == (en_ref <= eo_ref)
    if acc:
        assert np.allclose(zeros.cpu().numpy(), new.z0, rtol=1e-6, atol=1e-9)
        assert np.allclose(scales.cpu().numpy(), new.delta, rtol=1e-5)
    else:
        assert np.array_equal(scales.cpu().numpy(), sc0) and np.array_equal(zeros.cpu().numpy(), zr0)
    print(f"n={n} p={p} g={g}: eq.12 old {eo:.6g} new {en:.6g} -> {'accepted' if acc else 'rejected'}")


@pytest.mark.parametrize("n,p,N,bits,g,it,seed", [(192, 64, 600, 3, 32, 6, 2), (160, 48, 500, 3, 0, 6, 3),
                                                   (256, 130, 300, 4, 64, 5, 5), (256, 130, 300, 4, 64, 12, 5)])
def test_layer_with_refresh_against_oracle(ctx, n, p, N, bits, g, it, seed):
    import paper_2605_11222_amd as admmq
    X, W0 = correlated_problem(n, p, N, seed, outliers=2)
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    T = 80
    sched = admmq.Schedule(T=T, ls_rounds=2, ls_pairs=16, seed=seed, refresh_iter=it)
    codes, scales, zeros, st = ctx.quantize_layer(to_dev(H32), to_dev(W0), bits, g, sched)
    ref = orc.quantize_layer(H32.astype(np.float64), W0.astype(np.float64), bits, g, T=T, ls_rounds=2, ls_pairs=16,
                             seed=seed, refresh_iter=it)
    print(f"n={n} g={g}: refresh gpu {st.refresh_accepted} ({st.refresh_err_new:.5g} vs {st.refresh_err_old:.5g}) oracle "
          f"{ref.admm.refresh_accepted_at >= 0} ({ref.admm.refresh_err_new:.5g} vs {ref.admm.refresh_err_old:.5g}); "
          f"J admm {st.j_damp_admm:.6g}/{ref.j_damp_admm:.6g} final {st.j_damp:.6g}/{ref.j_damp:.6g}")
    assert st.refresh_accepted == (ref.admm.refresh_accepted_at >= 0)
    # the two trajectories have drifted apart by a few near-midpoint roundings when the attempt is made:
    # the sides of eq. 12 agree loosely here (tightly in the step test above, on identical inputs)
    assert st.refresh_err_old == pytest.approx(ref.admm.refresh_err_old, rel=2e-2)
    assert st.refresh_err_new == pytest.approx(ref.admm.refresh_err_new, rel=2e-2)
    assert st.j_damp_rtn == pytest.approx(ref.j_damp_rtn, rel=1e-4)
    # A refitted grid hangs on the two extreme entries of each group of the projection target.  With the attempt
    # at iteration 12 of this case the float64 oracle's own end objective moves by 0.6-0.8 % when every W-update
    # is perturbed by 2e-6 (a fifth of what the W-update is allowed), against 2e-4 without a refresh and 8e-4
    # with an early one (tests/test_oracle_refresh.py::test_a_late_refresh_amplifies_rounding_of_the_w_update):
    # no fp32 W-update can be held to 0.5 % there, so the late attempt is compared at four times the bar.
    tol = OBJ_TOL if it <= 6 else 4 * OBJ_TOL
    assert abs(st.j_damp_admm - ref.j_damp_admm) <= tol * ref.j_damp_admm
    assert abs(st.j_damp - ref.j_damp) <= tol * ref.j_damp
    if st.refresh_accepted and it <= 6:
        assert np.allclose(scales.cpu().numpy(), ref.scales, rtol=2e-3)
    # reported objective equals the float64 recomputation from the returned codes and (refreshed) grid
    gg = n if g == 0 else g
    k = codes.cpu().numpy().astype(np.float64)
    Wq = np.repeat(zeros.cpu().numpy().astype(np.float64), gg, 0) + k * np.repeat(scales.cpu().numpy().astype(np.float64), gg, 0)
    Hd = H32.astype(np.float64) + st.lam * np.eye(n)
    assert st.j_damp == pytest.approx(orc.objective(Hd, W0.astype(np.float64), Wq), rel=1e-4)
