"""GPU parity, step by step, through the C-ABI: each hot-path step on inputs identical to the
oracle's.  Integer codes must be bit-exact against the oracle's fp32 mirror; the W-update must be
within 1e-5 relative Frobenius error of the float64 literal form of eq. 7; the Hessian within fp32
accumulation error of the float64 X^T X."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import admmq_oracle as orc
from gpu_util import to_dev, bf16_bits_to_dev, correlated_problem, assert_differs_only_at_midpoints

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

W_UPDATE_TOL = 1e-5        # relative Frobenius error of the W-update (the workload's stated bar)


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_11222_amd as admmq
    c = admmq.Context(0)
    yield c
    c.close()


# ---------------------------------------------------------------------------------------------
# Hessian accumulation
# ---------------------------------------------------------------------------------------------
# (256, 96, f32) and (384, 1536, bf16) are whole tiles and whole k-stages in both chunks: the direct-load path of the
# fp32 matrix cores, for bf16 with the operands kept as bf16 in LDS; bf16 with n a multiple of 256 goes to the bf16
# matrix cores: whole stages only, with a tail of fewer than 32 tokens, a chunk too short for a stage, several
# token slices
@pytest.mark.parametrize("n,rows,dtype", [(128, 512, "f32"), (200, 333, "f32"), (384, 1000, "bf16"),
                                           (1030, 777, "bf16"), (64, 1, "f32"), (1, 5, "f32"),
                                           (512, 1536, "bf16"), (1024, 3072, "bf16"), (256, 96, "f32"),
                                           (384, 1536, "bf16"), (768, 1003, "bf16"), (256, 70, "bf16"),
                                           (2304, 4500, "bf16")])
def test_hessian_accumulate_matches_float64(ctx, n, rows, dtype):
    rng = np.random.default_rng(n + rows)
    X = (rng.standard_normal((rows, n)) * np.exp(rng.standard_normal(n))).astype(np.float32)
    if dtype == "bf16":
        bits = si.f32_to_bf16_bits(X)
        Xd = bf16_bits_to_dev(bits)
        X64 = si.bf16_bits_to_f32(bits).astype(np.float64)
    else:
        Xd = to_dev(X)
        X64 = X.astype(np.float64)
    H = torch.zeros((n, n), dtype=torch.float32, device="cuda")
    # two chunks (ragged split) accumulate into the same H
    cut = rows // 3
    got = 0
    if cut > 0:
        got += ctx.accumulate_hessian(H, Xd[:cut])
    got += ctx.accumulate_hessian(H, Xd[cut:])
    torch.cuda.synchronize()
    assert got == rows
    Href = orc.hessian([X64])
    Hg = H.cpu().numpy().astype(np.float64)
    assert np.array_equal(Hg, Hg.T)                                   # both triangles kept, exactly mirrored
    scale = np.sqrt(np.outer(np.diag(Href), np.diag(Href)))
    assert np.max(np.abs(Hg - Href) / scale) < 2e-6 * np.sqrt(max(rows, 16) / 16)


@pytest.mark.parametrize("col0", [0, 8, 4])
def test_hessian_of_a_column_window_of_wider_activations(ctx, col0):
    """X as a window of a wider bf16 tensor (row stride larger than n): columns from 0 and from 8 keep the rows
    16-byte aligned and take the bf16 matrix-core kernel, from 4 they are 8-byte aligned and take the fp32 product;
    all three must give the window's X^T X."""
    n, rows, wide = 512, 1000, 512 + 264
    rng = np.random.default_rng(col0 + 1)
    bits = si.f32_to_bf16_bits(rng.standard_normal((rows, wide)).astype(np.float32))
    Xw = bf16_bits_to_dev(bits)
    X64 = si.bf16_bits_to_f32(bits).astype(np.float64)[:, col0:col0 + n]
    H = torch.zeros((n, n), dtype=torch.float32, device="cuda")
    assert ctx.accumulate_hessian(H, Xw[:, col0:col0 + n]) == rows
    torch.cuda.synchronize()
    Href = orc.hessian([X64])
    scale = np.sqrt(np.outer(np.diag(Href), np.diag(Href)))
    assert np.max(np.abs(H.cpu().numpy() - Href) / scale) < 2e-6 * np.sqrt(rows / 16)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_hessian_in_a_callers_workspace_takes_fewer_token_slices(dtype):
    """A caller's workspace bounds the partial sums of the token slices: with room for two slices the result is the
    one an arena of the library's own gives, up to the order of the additions; with room for none the call fails
    with the workspace error and leaves H alone."""
    n, rows = 512, 8192
    rng = np.random.default_rng(5)
    X = rng.standard_normal((rows, n)).astype(np.float32)
    if dtype == "bf16":
        bits = si.f32_to_bf16_bits(X)
        Xd = bf16_bits_to_dev(bits)
        X64 = si.bf16_bits_to_f32(bits).astype(np.float64)
    else:
        Xd = to_dev(X)
        X64 = X.astype(np.float64)
    Href = orc.hessian([X64])
    import paper_2605_11222_amd as admmq
    c = admmq.Context(0)
    try:
        ws = torch.empty(2 * n * n * 4 + 16384, dtype=torch.uint8, device="cuda")
        c.set_workspace(ws)
        H = torch.zeros((n, n), dtype=torch.float32, device="cuda")
        assert c.accumulate_hessian(H, Xd) == rows
        torch.cuda.synchronize()
        scale = np.sqrt(np.outer(np.diag(Href), np.diag(Href)))
        assert np.max(np.abs(H.cpu().numpy() - Href) / scale) < 2e-6 * np.sqrt(rows / 16)
        tiny = torch.empty(n * n * 2, dtype=torch.uint8, device="cuda")
        c.set_workspace(tiny)
        H2 = torch.full((n, n), 7.0, dtype=torch.float32, device="cuda")
        with pytest.raises(admmq.AdmmqError) as err:
            c.accumulate_hessian(H2, Xd)
        assert err.value.code == 6                                   # ADMMQ_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert bool((H2 == 7.0).all())
    finally:
        c.close()


def test_hessian_cfg1_from_the_shared_generator(ctx):
    cfg = si.CONFIGS["cfg1"]
    H = torch.zeros((cfg.n, cfg.n), dtype=torch.float32, device="cuda")
    chunks = []
    for _, xc in si.iter_x_chunks(cfg):
        ctx.accumulate_hessian(H, to_dev(xc))
        chunks.append(si.chunk_as_f64(cfg, xc))
    Href = orc.hessian(chunks)
    rel = np.linalg.norm(H.cpu().numpy() - Href) / np.linalg.norm(Href)
    assert rel < 1e-6


# ---------------------------------------------------------------------------------------------
# grid fit and the fused projection / dual step
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,p,bits,g", [(128, 64, 4, 0), (96, 50, 3, 32), (64, 7, 2, 16), (256, 1028, 3, 64),
                                         (40, 1, 8, 0)])
def test_grid_init_matches_oracle(ctx, n, p, bits, g):
    rng = np.random.default_rng(n * p + bits)
    W0 = (0.02 * rng.standard_normal((n, p))).astype(np.float32)
    W0[:, 0] = 0.125 if p > 1 else W0[:, 0]                           # a degenerate column when p > 1
    scales, zeros = ctx.grid_init(to_dev(W0), bits, g)
    grid = orc.Grid.fit(W0.astype(np.float64), bits, g)
    assert np.array_equal(zeros.cpu().numpy(), grid.z0.astype(np.float32))
    # fp32 (max-min)/(2^b-1) against the float64 value: one rounding of the difference, one of the quotient
    assert np.allclose(scales.cpu().numpy(), grid.delta, rtol=3e-7, atol=0)
    if p > 1:
        assert np.all(scales.cpu().numpy()[:, 0] == 0.0)


@pytest.mark.parametrize("n,p,bits,g,rho", [(128, 64, 4, 0, 0.1), (96, 52, 3, 32, 2.5), (72, 7, 2, 8, 40.0),
                                             (512, 1028, 3, 64, 1.7e7), (33, 5, 4, 0, 0.3)])
def test_projection_codes_bit_exact_against_fp32_mirror(ctx, n, p, bits, g, rho):
    rng = np.random.default_rng(17 * n + p)
    W0 = (0.02 * rng.standard_normal((n, p))).astype(np.float32)
    if p > 4:
        W0[:, 3] = -0.5                                               # degenerate group(s)
    d = np.exp(0.5 * rng.standard_normal(n)).astype(np.float32)
    W0d = to_dev(W0)
    scales, zeros = ctx.grid_init(W0d, bits, g)
    sc, zr = scales.cpu().numpy(), zeros.cpu().numpy()
    Ws = (W0 * d[:, None]).astype(np.float32)
    W = (Ws + 0.3 * np.abs(Ws).mean() * rng.standard_normal((n, p))).astype(np.float32)
    V = (rho * 0.05 * np.abs(Ws).mean() * rng.standard_normal((n, p))).astype(np.float32)
    rho_next = rho * 1.1
    Vd = to_dev(V)
    codes, B, rs = ctx.project_dual(to_dev(W), Vd, to_dev(d), bits, g, scales, zeros, rho, rho_next)
    torch.cuda.synchronize()
    k, Vn, Bn, ss = orc.project_dual_step_f32(W, V, rho, rho_next, d, sc, zr, sc == 0, bits)
    assert np.array_equal(codes.cpu().numpy(), k)                     # integer work: bit-exact
    assert np.array_equal(Vd.cpu().numpy(), Vn)
    assert np.array_equal(B.cpu().numpy(), Bn)
    assert rs == pytest.approx(ss, rel=1e-5)
    # against the float64 projection: differences only next to a rounding midpoint
    grid = orc.Grid(sc.astype(np.float64), zr.astype(np.float64), bits, sc == 0)
    k64, _, Wt = orc.d_update(W.astype(np.float64), V.astype(np.float64), rho, d.astype(np.float64), grid)
    assert_differs_only_at_midpoints(k, k64, Wt, d, sc, zr, g)


def test_first_projection_of_dense_weights_is_round_to_nearest(ctx):
    """Alg. 1 with D0 = Ws, V0 = 0: the first projection is RTN of W0 (checked on the GPU path)."""
    cfg = si.CONFIGS["cfg1"]
    W0 = si.layer_weights(cfg)
    rng = np.random.default_rng(0)
    d = np.exp(0.3 * rng.standard_normal(cfg.n)).astype(np.float32)
    scales, zeros = ctx.grid_init(to_dev(W0), cfg.bits, 0)
    Ws = (W0 * d[:, None]).astype(np.float32)
    V = torch.zeros((cfg.n, cfg.p), dtype=torch.float32, device="cuda")
    codes, _, _ = ctx.project_dual(to_dev(Ws), V, to_dev(d), cfg.bits, 0, scales, zeros, 0.1, 0.11)
    grid = orc.Grid.fit(W0.astype(np.float64), cfg.bits, 0)
    k_rtn, _ = orc.rtn(W0.astype(np.float64), grid)
    k = codes.cpu().numpy().astype(np.int64)
    t = (W0.astype(np.float64) - grid.z0) / grid.delta
    near = np.abs(t - np.floor(t) - 0.5) < 1e-4
    assert np.all((k == k_rtn) | near) and np.mean(k != k_rtn) < 1e-3


# ---------------------------------------------------------------------------------------------
# factorisation + W-update (eq. 7)
# ---------------------------------------------------------------------------------------------
# the later shapes walk the product launcher's paths: whole 64 / 128 / 256 tiles filled by direct loads (256 x 1280,
# 1024 x 2048, 2048 x 2048), a ragged width on the staged path (1024 x 4100), a column split whose tail takes a
# smaller tile (768 x 5120: 3 x 20 tiles), and the tridiagonal solve's 8- and 16-column strips.
# Both forms of the factorisation at every shape (the library picks by size; the environment forces one): the
# tridiagonal form with its scalar recurrence, and the band form (block reflectors, 16 x 16 block elimination), for
# which the shapes also cover n below one band width, n = 17 .. 19 (no, one and two reflectors), n not a multiple of
# 16, a Hessian of rank n/3 + damping (640 x 130 with 400 tokens: panels close to rank-deficient) and the last
# panels' plain Householder path.
@pytest.mark.parametrize("form", ["tridiag", "band"])
@pytest.mark.parametrize("n,p,N,seed", [(128, 64, 512, 0), (300, 77, 900, 1), (3, 5, 10, 2), (2, 4, 9, 3),
                                         (1, 3, 4, 4), (1024, 256, 3000, 5), (640, 130, 400, 6),
                                         (256, 1280, 600, 7), (1024, 2048, 2100, 8), (1024, 4100, 2100, 9),
                                         (2048, 2048, 4200, 10), (768, 5120, 1600, 11),
                                         (17, 20, 60, 12), (18, 33, 60, 13), (19, 16, 70, 14), (100, 50, 300, 15)])
def test_w_update_matches_literal_eq7_in_float64(ctx, monkeypatch, n, p, N, seed, form):
    if form == "tridiag" and seed >= 12:
        pytest.skip("shapes added for the band form")
    monkeypatch.setenv("ADMMQ_FACTOR", form)
    X, W0 = correlated_problem(n, p, N, seed, outliers=2 if n > 100 else 0)   # N < n in the last case
    H64 = orc.hessian([X.astype(np.float64)])
    H32 = H64.astype(np.float32)
    d, lam = ctx.factorize(to_dev(H32), 0.01, True)
    Hd, lam64 = orc.damp_hessian(H32.astype(np.float64), 0.01)
    assert lam == pytest.approx(lam64, rel=1e-6)
    dref, Hs, _ = orc.scale_problem(Hd, W0.astype(np.float64))
    dg = d.cpu().numpy()
    assert np.allclose(dg, dref, rtol=2e-7)
    # the solver's scaled problem uses the fp32 d: build the oracle's operands from the same d
    d64 = dg.astype(np.float64)
    Hs = Hd / d64[:, None] / d64[None, :]
    Ws = (W0 * dg[:, None]).astype(np.float32)
    lam_e, U = np.linalg.eigh(Hs)
    lam_e = np.maximum(lam_e, 0)
    rng = np.random.default_rng(seed + 100)
    scale = np.abs(Ws).mean()
    worst = 0.0
    for rho in (0.1, 1.0, 37.0, 1.7e7):
        D = (Ws + 0.3 * scale * rng.standard_normal(Ws.shape)).astype(np.float32)
        V = (rho * 0.1 * scale * rng.standard_normal(Ws.shape)).astype(np.float32)
        Wg = ctx.w_update(to_dev(Ws), to_dev(D), to_dev(V), rho).cpu().numpy().astype(np.float64)
        Wref = orc.w_update(U, lam_e, Hs @ Ws.astype(np.float64), D.astype(np.float64), V.astype(np.float64), rho)
        err = np.linalg.norm(Wg - Wref) / np.linalg.norm(Wref)
        worst = max(worst, err)
        assert err < W_UPDATE_TOL, (rho, err)
    print(f"n={n} p={p} {form}: worst relative W-update error {worst:.2e}")


@pytest.mark.parametrize("n,p,N,seed", [(1024, 96, 3000, 21), (700, 64, 250, 22)])
def test_w_update_band_form_with_lower_triangle_passes(ctx, monkeypatch, n, p, N, seed):
    """The band reduction's two trailing passes read and update only the lower triangle while the trailing matrix
    is large (6144 rows and up by default); here the mode is switched on for small matrices, so that the step is
    compared with eq. 7 in float64 through that path too: squares of 4 x 4 tiles with ragged edges, the
    hand-over to the full-square kernels (upper triangle restored) at 128 rows, a Hessian of rank N < n."""
    monkeypatch.setenv("ADMMQ_FACTOR", "band")
    monkeypatch.setenv("ADMMQ_BAND_LOWER_MIN", "128")
    X, W0 = correlated_problem(n, p, N, seed, outliers=2)
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    d, lam = ctx.factorize(to_dev(H32), 0.01, True)
    Hd, _ = orc.damp_hessian(H32.astype(np.float64), 0.01)
    dg = d.cpu().numpy()
    d64 = dg.astype(np.float64)
    Hs = Hd / d64[:, None] / d64[None, :]
    Ws = (W0 * dg[:, None]).astype(np.float32)
    lam_e, U = np.linalg.eigh(Hs)
    lam_e = np.maximum(lam_e, 0)
    rng = np.random.default_rng(seed)
    scale = np.abs(Ws).mean()
    for rho in (0.1, 37.0):
        D = (Ws + 0.3 * scale * rng.standard_normal(Ws.shape)).astype(np.float32)
        V = (rho * 0.1 * scale * rng.standard_normal(Ws.shape)).astype(np.float32)
        Wg = ctx.w_update(to_dev(Ws), to_dev(D), to_dev(V), rho).cpu().numpy().astype(np.float64)
        Wref = orc.w_update(U, lam_e, Hs @ Ws.astype(np.float64), D.astype(np.float64), V.astype(np.float64), rho)
        assert np.linalg.norm(Wg - Wref) / np.linalg.norm(Wref) < W_UPDATE_TOL


def test_w_update_band_form_of_a_diagonal_hessian(ctx, monkeypatch):
    """Uncorrelated channels: every block below the band is zero, the Gram matrix of a panel is singular, and the
    reduction must fall back to plain Householder steps that find nothing to eliminate (Q = I).  eq. 7 is then
    diagonal and has a closed form to compare with."""
    monkeypatch.setenv("ADMMQ_FACTOR", "band")
    n, p = 200, 48
    rng = np.random.default_rng(5)
    hd = (0.5 + rng.random(n)).astype(np.float32)
    H32 = np.diag(hd).astype(np.float32)
    W0 = rng.standard_normal((n, p)).astype(np.float32)
    d, lam = ctx.factorize(to_dev(H32), 0.01, True)
    dg = d.cpu().numpy()
    Ws = (W0 * dg[:, None]).astype(np.float32)
    for rho in (0.1, 5.0):
        D = (Ws + 0.1 * rng.standard_normal(Ws.shape)).astype(np.float32)
        V = (rho * 0.05 * rng.standard_normal(Ws.shape)).astype(np.float32)
        Wg = ctx.w_update(to_dev(Ws), to_dev(D), to_dev(V), rho).cpu().numpy().astype(np.float64)
        # Hs = I: W = (Ws + rho D - V) / (1 + rho)
        Wref = (Ws.astype(np.float64) + rho * D.astype(np.float64) - V.astype(np.float64)) / (1.0 + rho)
        assert np.linalg.norm(Wg - Wref) / np.linalg.norm(Wref) < W_UPDATE_TOL


@pytest.mark.parametrize("n,p,N,taken", [(1024, 6400, 2100, True), (2048, 3328, 4200, True), (1024, 1792, 2100, False)])
def test_w_update_with_split_fp16_products_matches_literal_eq7(ctx, n, p, N, taken):
    """The opt-in split-fp16 products against the same float64 reference and bar: 4 x 25 tiles cut into two slices
    of the contraction, 8 x 13 tiles in two slices, and a shape the products do not take (28 tiles, too short a
    contraction to slice), which must come out exactly as without the switch."""
    import paper_2605_11222_amd as admmq
    X, W0 = correlated_problem(n, p, N, seed=n + p, outliers=2)
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    d, lam = ctx.factorize(to_dev(H32), 0.01, True)
    Hd, _ = orc.damp_hessian(H32.astype(np.float64), 0.01)
    dg = d.cpu().numpy()
    d64 = dg.astype(np.float64)
    Hs = Hd / d64[:, None] / d64[None, :]
    Ws = (W0 * dg[:, None]).astype(np.float32)
    lam_e, U = np.linalg.eigh(Hs)
    lam_e = np.maximum(lam_e, 0)
    HWs = Hs @ Ws.astype(np.float64)
    rng = np.random.default_rng(n)
    scale = np.abs(Ws).mean()
    assert (admmq.fast_products_bytes(n, p) > 0) == taken
    for rho in (0.1, 37.0):
        D = (Ws + 0.3 * scale * rng.standard_normal(Ws.shape)).astype(np.float32)
        V = (rho * 0.1 * scale * rng.standard_normal(Ws.shape)).astype(np.float32)
        W_fp32 = ctx.w_update(to_dev(Ws), to_dev(D), to_dev(V), rho)
        ctx.set_fast_products(True)
        try:
            W_fast = ctx.w_update(to_dev(Ws), to_dev(D), to_dev(V), rho)
        finally:
            ctx.set_fast_products(False)
        assert torch.equal(W_fp32, W_fast) == (not taken)
        Wref = orc.w_update(U, lam_e, HWs, D.astype(np.float64), V.astype(np.float64), rho)
        err = np.linalg.norm(W_fast.cpu().numpy().astype(np.float64) - Wref) / np.linalg.norm(Wref)
        print(f"n={n} p={p} rho={rho:g}: relative W-update error with the split-fp16 products {err:.2e}")
        assert err < W_UPDATE_TOL


@pytest.mark.parametrize("n,p,N,switch", [(300, 40, 900, 128), (1030, 64, 2100, 512), (640, 33, 400, 128),
                                          (200, 16, 500, 129)])
def test_factorisation_from_the_lower_triangle_matches_literal_eq7(ctx, monkeypatch, n, p, N, switch):
    """The factorisation's mode for large matrices (trailing products read the lower triangle only; the library
    enters it at sizes no test reaches by default) forced on from n down to `switch`, where it hands over to the
    ordinary mode: same bar as above, and the same W as the ordinary mode to rounding."""
    X, W0 = correlated_problem(n, p, N, seed=n, outliers=2)
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    Hd, _ = orc.damp_hessian(H32.astype(np.float64), 0.01)
    rng = np.random.default_rng(n)
    got = {}
    for mode, env in (("plain", "0"), ("lower", str(switch))):
        monkeypatch.setenv("ADMMQ_SYMV_MIN", env)
        d, lam = ctx.factorize(to_dev(H32), 0.01, True)
        dg = d.cpu().numpy()
        Ws = (W0 * dg[:, None]).astype(np.float32)
        if mode == "plain":
            scale = np.abs(Ws).mean()
            D = (Ws + 0.3 * scale * rng.standard_normal(Ws.shape)).astype(np.float32)
            V = (0.05 * scale * rng.standard_normal(Ws.shape)).astype(np.float32)
        got[mode] = [ctx.w_update(to_dev(Ws), to_dev(D), to_dev(V), rho).cpu().numpy().astype(np.float64)
                     for rho in (0.1, 5.0)]
    d64 = dg.astype(np.float64)
    Hs = Hd / d64[:, None] / d64[None, :]
    lam_e, U = np.linalg.eigh(Hs)
    lam_e = np.maximum(lam_e, 0)
    for idx, rho in enumerate((0.1, 5.0)):
        Wref = orc.w_update(U, lam_e, Hs @ Ws.astype(np.float64), D.astype(np.float64), V.astype(np.float64), rho)
        for mode in ("plain", "lower"):
            err = np.linalg.norm(got[mode][idx] - Wref) / np.linalg.norm(Wref)
            assert err < W_UPDATE_TOL, (mode, rho, err)
        assert np.linalg.norm(got["lower"][idx] - got["plain"][idx]) <= 2e-6 * np.linalg.norm(Wref)


def test_stream_copy_copies(ctx):
    """The plain copy kernel bench.py uses as its bandwidth reference: whole blocks, a ragged tail, a tiny size."""
    for count in (4 * 1024 * 37, 4 * 1024 * 3 + 52, 4):
        src = torch.randn(count, device="cuda")
        dst = torch.zeros(count + 8, device="cuda")
        ctx.stream_copy(dst[:count], src)
        torch.cuda.synchronize()
        assert torch.equal(dst[:count], src) and float(dst[count:].abs().sum()) == 0.0
