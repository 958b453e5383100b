"""GPU parity of the symmetric grid and the MSE clipping search (paper Sec. 3.4, App. D) against the oracle."""
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


def heavy_weights(n, p, seed):
    rng = np.random.default_rng(seed)
    W = (0.02 * rng.standard_normal((n, p))).astype(np.float32)
    idx = rng.integers(0, n, 12), rng.integers(0, p, 12)
    W[idx] *= 6.0
    return W


def group_error(W, delta, z0, bits, g):
    """float64 squared quantization error per group of the dense weights on a given grid."""
    n = W.shape[0]
    gg = n if g == 0 else g
    grid = orc.Grid(delta.astype(np.float64), z0.astype(np.float64), bits, delta == 0)
    E = (grid.dequant(grid.codes(W.astype(np.float64))) - W.astype(np.float64)) ** 2
    return E.reshape(n // gg, gg, -1).sum(axis=1)


@pytest.mark.parametrize("n,p,bits,g,sym,points", [(128, 70, 3, 0, True, 0), (96, 33, 4, 32, True, 0),
                                                     (128, 70, 3, 0, False, 100), (64, 1030, 2, 16, True, 100),
                                                     (256, 5, 4, 64, False, 50)])
def test_grid_fit_options_match_oracle(ctx, n, p, bits, g, sym, points):
    W = heavy_weights(n, p, n + p)
    scales, zeros = ctx.grid_fit(to_dev(W), bits, g, sym, points, 0.8)
    sc, zr = scales.cpu().numpy(), zeros.cpu().numpy()
    ref = orc.Grid.fit(W.astype(np.float64), bits, g, sym, points, 0.8)
    if points == 0:
        assert np.allclose(sc, ref.delta, rtol=3e-7) and np.allclose(zr, ref.z0, rtol=1e-7)
        return
    # the search compares fp32 error sums: near-ties between neighbouring candidates may fall the other way,
    # so compare what is unique - the achieved error - and check that the result is one of the candidates
    e_gpu = group_error(W, sc, zr, bits, g)
    e_ref = group_error(W, ref.delta, ref.z0, bits, g)
    assert np.all(e_gpu <= e_ref * (1 + 1e-4) + 1e-12)
    same = np.isclose(sc, ref.delta, rtol=1e-5)
    print(f"n={n} p={p} sym={sym}: identical candidate in {same.mean():.3f} of the groups")
    assert same.mean() > 0.95
    base = orc.Grid.fit(W.astype(np.float64), bits, g, sym, 0)
    ratio = sc / base.delta
    cand = 1.0 - np.arange(int(0.8 * points)) / points
    assert np.all(np.min(np.abs(ratio[..., None] - cand), axis=-1) < 1e-5)
    assert np.allclose(zr, ratio * base.z0, rtol=1e-5, atol=1e-9)


@pytest.mark.parametrize("sym,points", [(True, 0), (False, 100), (True, 100)])
def test_layer_on_optional_grids_against_oracle(ctx, sym, points):
    import paper_2605_11222_amd as admmq
    X, _ = correlated_problem(160, 48, 500, 61, outliers=2)
    W0 = heavy_weights(160, 48, 62)
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    sched = admmq.Schedule(T=60, ls_rounds=2, ls_pairs=16, seed=5, symmetric=sym, clip_points=points)
    codes, scales, zeros, st = ctx.quantize_layer(to_dev(H32), to_dev(W0), 3, 32, sched)
    ref = orc.quantize_layer(H32.astype(np.float64), W0.astype(np.float64), 3, 32, T=60, ls_rounds=2, ls_pairs=16, seed=5,
                             symmetric=sym, clip_points=points)
    print(f"sym={sym} clip={points}: J rtn {st.j_damp_rtn:.6g}/{ref.j_damp_rtn:.6g} admm {st.j_damp_admm:.6g}/"
          f"{ref.j_damp_admm:.6g} final {st.j_damp:.6g}/{ref.j_damp:.6g}")
    assert np.isclose(scales.cpu().numpy(), ref.scales, rtol=1e-5).mean() > 0.95
    assert abs(st.j_damp_rtn - ref.j_damp_rtn) <= OBJ_TOL * ref.j_damp_rtn
    assert abs(st.j_damp_admm - ref.j_damp_admm) <= OBJ_TOL * ref.j_damp_admm
    assert abs(st.j_damp - ref.j_damp) <= OBJ_TOL * ref.j_damp
    if sym:
        assert np.allclose(zeros.cpu().numpy(), -3.5 * scales.cpu().numpy(), rtol=1e-6)
