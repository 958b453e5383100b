"""GPU parity for the other formats (Sec. 4.3), through the C-ABI: the dual-grid fit, one projection + dual
pass against the oracle's fp32 mirror (codes bit-exact), and the whole ADMM loop against the float64 oracle
(objective within 0.5 %).  Outlier sets and codebooks are synthetic (largest magnitudes per column, column
quantiles): the paper takes them from other methods' artefacts, which are not available."""
import numpy as np
import pytest

import synth_inputs as si
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


def _state(n, p, seed):
    rng = np.random.default_rng(seed)
    W0 = (rng.standard_normal((n, p)) * 0.02).astype(np.float32)
    W0[rng.integers(0, n, p), np.arange(p)] *= 9.0
    d = np.exp(rng.standard_normal(n) * 0.4).astype(np.float32)
    W = (d[:, None] * W0 + rng.standard_normal((n, p)).astype(np.float32) * 0.004).astype(np.float32)
    V = (rng.standard_normal((n, p)) * 0.002).astype(np.float32)
    return W0, d, W, V


@pytest.mark.parametrize("n,p,bits,g", [(64, 40, 3, 0), (96, 130, 2, 32), (257, 33, 4, 0), (128, 1024, 3, 64)])
def test_dual_grid_fit_and_projection_bit_exact(ctx, n, p, bits, g):
    import paper_2605_11222_amd as admmq
    W0, d, W, V = _state(n, p, n + p)
    mask = si.outlier_mask(W0, 0.06)
    fmt = orc.DualGridProjection.fit(W0.astype(np.float64), bits, mask, g)
    flags = to_dev(mask.astype(np.uint8))
    scales, zeros = ctx.grid_init_dual(to_dev(W0), bits, flags, g)
    # the fit is min / max (exact in any precision) and one fp32 subtraction and division
    gg = g if g else n
    f32 = np.float32
    for s, (sel, gr) in enumerate(((~mask, fmt.inlier), (mask, fmt.outlier))):
        lo = np.where(sel, W0, np.inf).reshape(n // gg, gg, p).min(axis=1)
        hi = np.where(sel, W0, -np.inf).reshape(n // gg, gg, p).max(axis=1)
        empty = hi < lo
        lo = np.where(empty, 0, lo).astype(f32)
        hi = np.where(empty, 0, hi).astype(f32)
        np.testing.assert_array_equal(zeros[s].cpu().numpy(), lo)
        np.testing.assert_array_equal(lo, gr.z0.astype(f32))                       # and the oracle's fit agrees
        np.testing.assert_array_equal(scales[s].cpu().numpy(), ((hi - lo) / f32(2 ** bits - 1)).astype(f32))
        np.testing.assert_allclose(scales[s].cpu().numpy(), gr.delta, rtol=3e-7, atol=0)
    # mirror on the library's own fp32 grids
    sc, zr = scales.cpu().numpy(), zeros.cpu().numpy()
    fmt32 = orc.DualGridProjection(orc.Grid(sc[0], zr[0], bits, sc[0] == 0), orc.Grid(sc[1], zr[1], bits, sc[1] == 0),
                                   mask)
    rho, rho_next = 0.37, 0.407
    Vd = to_dev(V)
    codes, B, Xq, rs = ctx.project_dual_format(to_dev(W), Vd, to_dev(d), admmq.FORMAT_DUAL_GRID, bits, rho, rho_next,
                                               group_size=g, flags=flags, scales=scales, zeros=zeros)
    k, Vn, Bn, xq, ss = orc.project_dual_step_format_f32(W, V, rho, rho_next, d, fmt32)
    np.testing.assert_array_equal(codes.cpu().numpy(), k)
    np.testing.assert_array_equal(Vd.cpu().numpy(), Vn)
    np.testing.assert_array_equal(B.cpu().numpy(), Bn)
    np.testing.assert_array_equal(Xq.cpu().numpy(), xq)
    assert abs(rs - ss) <= 1e-5 * ss


@pytest.mark.parametrize("n,p,bits,kept", [(64, 40, 3, True), (96, 130, 2, False), (257, 33, 4, True),
                                           (128, 1024, 1, True), (33, 7, 3, False)])
def test_codebook_projection_bit_exact(ctx, n, p, bits, kept):
    import paper_2605_11222_amd as admmq
    W0, d, W, V = _state(n, p, 3 * n + p)
    cb = si.column_codebook(W0, bits)
    free = si.outlier_mask(W0, 0.03) if kept else None
    fmt = orc.CodebookProjection(cb, free)
    rho, rho_next = 0.21, 0.231
    Vd = to_dev(V)
    codes, B, Xq, rs = ctx.project_dual_format(to_dev(W), Vd, to_dev(d), admmq.FORMAT_CODEBOOK, bits, rho, rho_next,
                                               flags=to_dev(free.astype(np.uint8)) if kept else None,
                                               codebook=to_dev(cb))
    k, Vn, Bn, xq, ss = orc.project_dual_step_format_f32(W, V, rho, rho_next, d, fmt)
    np.testing.assert_array_equal(codes.cpu().numpy(), k)
    np.testing.assert_array_equal(Vd.cpu().numpy(), Vn)
    np.testing.assert_array_equal(B.cpu().numpy(), Bn)
    np.testing.assert_array_equal(Xq.cpu().numpy(), xq)
    assert abs(rs - ss) <= 1e-5 * ss
    # in-place form used by the loop: B written over W
    import ctypes as C
    from paper_2605_11222_amd import binding
    Wd, Vd2, dd, cb_d = to_dev(W), to_dev(V), to_dev(d), to_dev(cb)
    fl_d = to_dev(free.astype(np.uint8)) if kept else None
    f = binding._Format(admmq.FORMAT_CODEBOOK, bits, 0, binding._ptr(fl_d), binding._ptr(cb_d), None, None)
    binding._check(ctx._lib.admmq_project_dual_format(ctx._h, binding._ptr(Wd), binding._ptr(Vd2), n, p,
                                                      binding._ptr(dd), C.byref(f), rho, rho_next, None,
                                                      binding._ptr(Wd), None, None))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Wd.cpu().numpy(), Bn)


def test_codebook_must_ascend(ctx):
    import paper_2605_11222_amd as admmq
    W0, d, W, V = _state(32, 16, 5)
    cb = si.column_codebook(W0, 2)
    cb[2, 3] = cb[1, 3]                    # two equal levels in one column
    with pytest.raises(admmq.AdmmqError):
        ctx.project_dual_format(to_dev(W), to_dev(V), to_dev(d), admmq.FORMAT_CODEBOOK, 2, 0.2, 0.22,
                                codebook=to_dev(cb))
    cb = si.column_codebook(W0, 2)
    cb[0, 0] = np.nan
    H = to_dev(np.eye(32, dtype=np.float32))
    with pytest.raises(admmq.AdmmqError):
        ctx.quantize_layer_format(H, to_dev(W0), admmq.FORMAT_CODEBOOK, 2, codebook=to_dev(cb),
                                  sched=admmq.Schedule(T=3, ls_rounds=0))


@pytest.mark.parametrize("kind,n,p,N,bits,g,T", [("dual", 128, 64, 512, 3, 0, 50), ("dual", 256, 96, 1024, 2, 64, 60),
                                                  ("codebook", 128, 64, 512, 3, 0, 50),
                                                  ("codebook_kept", 256, 96, 1024, 2, 0, 60),
                                                  ("codebook_kept", 192, 130, 700, 4, 0, 40)])
@pytest.mark.parametrize("form", ["tridiag", "band"])      # both forms of the factorisation
def test_layer_with_another_format_matches_the_oracle(ctx, monkeypatch, kind, n, p, N, bits, g, T, form):
    import paper_2605_11222_amd as admmq
    monkeypatch.setenv("ADMMQ_FACTOR", form)
    X, W0 = correlated_problem(n, p, N, seed=n + T, outliers=2)
    rng = np.random.default_rng(1)
    W0[rng.integers(0, n, p), np.arange(p)] *= 8.0
    H = torch.zeros((n, n), dtype=torch.float32, device="cuda")
    ctx.accumulate_hessian(H, to_dev(X))
    torch.cuda.synchronize()
    H64 = H.cpu().numpy().astype(np.float64)
    sched = admmq.Schedule(T=T, ls_rounds=0)
    if kind == "dual":
        mask = si.outlier_mask(W0, 0.05)
        fmt = orc.DualGridProjection.fit(W0.astype(np.float64), bits, mask, g)
        codes, Wq, grids, st = ctx.quantize_layer_format(H, to_dev(W0), admmq.FORMAT_DUAL_GRID, bits, group_size=g,
                                                         flags=to_dev(mask.astype(np.uint8)), sched=sched,
                                                         want_history=True)
        free = None
    else:
        cb = si.column_codebook(W0, bits)
        free = si.outlier_mask(W0, 0.02) if kind == "codebook_kept" else None
        fmt = orc.CodebookProjection(cb.astype(np.float64), free)
        codes, Wq, grids, st = ctx.quantize_layer_format(H, to_dev(W0), admmq.FORMAT_CODEBOOK, bits,
                                                         flags=to_dev(free.astype(np.uint8)) if free is not None else None,
                                                         codebook=to_dev(cb), sched=sched, want_history=True)
    a, j_admm, j_near = orc.quantize_layer_format(H64, W0.astype(np.float64), fmt, T=T)
    assert abs(st.j_damp_rtn - j_near) <= 1e-4 * j_near
    assert abs(st.j_damp_admm - j_admm) <= OBJ_TOL * j_admm
    assert st.j_damp_admm < st.j_damp_rtn
    # the reported objective is the objective of the returned weights (float64, damped Hessian)
    Hd, _ = orc.damp_hessian(H64)
    Wq_h = Wq.cpu().numpy().astype(np.float64)
    assert abs(orc.objective(Hd, W0.astype(np.float64), Wq_h) - st.j_damp_admm) <= 1e-4 * st.j_damp_admm
    assert abs(orc.objective(H64, W0.astype(np.float64), Wq_h) - st.j_recon) <= 1e-4 * st.j_recon
    # the returned weights are feasible: every constrained entry is the level its code names
    k = codes.cpu().numpy()
    if kind == "dual":
        sc, zr = grids[0].cpu().numpy(), grids[1].cpu().numpy()
        gg = g if g else n
        sel = mask.astype(np.int64)
        rows = np.arange(n)[:, None] // gg
        cols = np.arange(p)[None, :]
        want = (k.astype(np.float32) * sc[sel, rows, cols] + zr[sel, rows, cols]).astype(np.float32)
        np.testing.assert_array_equal(Wq.cpu().numpy(), want)
        assert k.max() <= 2 ** bits - 1
    else:
        want = np.take_along_axis(cb, k.astype(np.int64), axis=0)
        got = Wq.cpu().numpy()
        con = np.ones((n, p), dtype=bool) if free is None else ~free
        np.testing.assert_array_equal(got[con], want[con])
        if free is not None:
            assert np.all(k[free] == 0)
            assert np.mean(got[free] == want[free]) < 0.5      # kept entries are not snapped to a level
    # residual history: the float64 loop's, within the drift of two fp32 / fp64 trajectories
    res = np.array(st.primal_res)
    ref = np.array(a.primal)
    assert res.shape == ref.shape
    early = slice(0, 5)
    np.testing.assert_allclose(res[early], ref[early], rtol=2e-3, atol=1e-6 * ref[0])


def test_format_layer_reuses_the_factorisation(ctx):
    import paper_2605_11222_amd as admmq
    n, p = 128, 48
    X, W0 = correlated_problem(n, p, 400, seed=21)
    H = torch.zeros((n, n), dtype=torch.float32, device="cuda")
    ctx.accumulate_hessian(H, to_dev(X))
    cb = si.column_codebook(W0, 3)
    first = ctx.quantize_layer_format(H, to_dev(W0), admmq.FORMAT_CODEBOOK, 3, codebook=to_dev(cb),
                                      sched=admmq.Schedule(T=20, ls_rounds=0))
    again = ctx.quantize_layer_format(H, to_dev(W0), admmq.FORMAT_CODEBOOK, 3, codebook=to_dev(cb),
                                      sched=admmq.Schedule(T=20, ls_rounds=0, reuse_factor=True))
    assert torch.equal(first[0], again[0]) and torch.equal(first[1], again[1])
    assert again[3].ms_factor < first[3].ms_factor
