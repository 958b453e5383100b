"""GPU parity of the whole layer solver and of the local search against the float64 oracle.

The ADMM trajectory is a discrete dynamical system: one rounding that falls the other way near a
midpoint (fp32 against float64) changes later iterates, and the local search breaks near-ties by
floating-point totals.  Several final code matrices are therefore correct; what is unique is compared
(grid, first-iteration codes, objectives within 0.5 %), the rest is checked for validity (codes in
range, objective recomputed in float64 from the returned codes equals the reported one, local search
never raises the objective, determinism)."""
import itertools

import numpy as np
import pytest

import synth_inputs as si
from oracle import admmq_oracle as orc
from gpu_util import to_dev, correlated_problem

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

OBJ_TOL = 5e-3       # final layer objective within 0.5 % relative of the oracle's


@pytest.fixture(scope="module")
def ctx():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_11222_amd as admmq
    c = admmq.Context(0)
    yield c
    c.close()


def cfg1_inputs(ctx):
    cfg = si.CONFIGS["cfg1"]
    H = torch.zeros((cfg.n, cfg.n), dtype=torch.float32, device="cuda")
    chunks = []
    for _, xc in si.iter_x_chunks(cfg):
        ctx.accumulate_hessian(H, to_dev(xc))
        chunks.append(si.chunk_as_f64(cfg, xc))
    W0 = si.layer_weights(cfg)
    return cfg, H, W0, orc.hessian(chunks)


def f64_objective(H32, lam, W0, codes, scales, zeros, g):
    n = W0.shape[0]
    gg = n if g == 0 else g
    Wq = np.repeat(zeros.astype(np.float64), gg, 0) + codes.astype(np.float64) * np.repeat(scales.astype(np.float64), gg, 0)
    Hd = H32.astype(np.float64) + lam * np.eye(n)
    return orc.objective(Hd, W0.astype(np.float64), Wq)


def test_cfg1_whole_layer_against_oracle(ctx):
    import paper_2605_11222_amd as admmq
    cfg, H, W0, H64 = cfg1_inputs(ctx)
    sched = admmq.Schedule(T=cfg.T, ls_rounds=5, seed=0)
    codes, scales, zeros, st = ctx.quantize_layer(H, to_dev(W0), cfg.bits, cfg.group_size, sched, want_history=True)
    torch.cuda.synchronize()
    ref = orc.quantize_layer(H64, W0.astype(np.float64), cfg.bits, cfg.group_size, T=cfg.T, ls_rounds=5, seed=0)
    k = codes.cpu().numpy()
    assert k.max() <= 2 ** cfg.bits - 1
    assert np.array_equal(zeros.cpu().numpy(), ref.zeros.astype(np.float32))
    assert np.allclose(scales.cpu().numpy(), ref.scales, rtol=3e-7)
    # objectives: reported == recomputed in float64 from the returned codes; within 0.5 % of the oracle
    H32 = H.cpu().numpy()
    j64 = f64_objective(H32, st.lam, W0, k, scales.cpu().numpy(), zeros.cpu().numpy(), cfg.group_size)
    assert st.j_damp == pytest.approx(j64, rel=1e-4)
    # the reconstruction error ||X (Wq - W0)||_F^2 (undamped H): recomputed in float64, and against the oracle's
    assert st.j_recon == pytest.approx(f64_objective(H32, 0.0, W0, k, scales.cpu().numpy(), zeros.cpu().numpy(),
                                                     cfg.group_size), rel=1e-4)
    assert abs(st.j_recon - ref.j_recon) <= OBJ_TOL * ref.j_recon
    assert st.j_recon < st.j_damp
    assert st.j_damp_rtn == pytest.approx(ref.j_damp_rtn, rel=1e-4)
    assert abs(st.j_damp_admm - ref.j_damp_admm) <= OBJ_TOL * ref.j_damp_admm
    assert abs(st.j_damp - ref.j_damp) <= OBJ_TOL * ref.j_damp
    assert st.j_damp <= st.j_damp_admm * (1 + 1e-6) <= st.j_damp_rtn
    # residual history: same decay as the oracle's until the fp32 floor
    pr = np.array(st.primal_res)
    assert pr[0] == pytest.approx(ref.admm.primal[0], rel=1e-4)
    live = np.array(ref.admm.primal) > 1e-4 * ref.admm.primal[0]
    assert np.allclose(pr[live], np.array(ref.admm.primal)[live], rtol=0.05)
    assert st.code_flips[0] > 0 and st.code_flips[-1] == 0
    print(f"cfg1: J rtn {st.j_damp_rtn:.4f} admm {st.j_damp_admm:.4f} (oracle {ref.j_damp_admm:.4f}) "
          f"final {st.j_damp:.4f} (oracle {ref.j_damp:.4f}) moves {st.ls_moves} vs {ref.ls.moves}")


def test_one_iteration_returns_round_to_nearest(ctx):
    import paper_2605_11222_amd as admmq
    cfg, H, W0, H64 = cfg1_inputs(ctx)
    codes, scales, zeros, st = ctx.quantize_layer(H, to_dev(W0), cfg.bits, 0, admmq.Schedule(T=1, ls_rounds=0))
    grid = orc.Grid.fit(W0.astype(np.float64), cfg.bits, 0)
    k_rtn, _ = orc.rtn(W0.astype(np.float64), grid)
    k = codes.cpu().numpy().astype(np.int64)
    t = (W0.astype(np.float64) - grid.z0) / grid.delta
    near = np.abs(t - np.floor(t) - 0.5) < 1e-4
    assert np.all((k == k_rtn) | near) and np.mean(k != k_rtn) < 1e-3
    assert st.j_damp_admm == pytest.approx(st.j_damp_rtn, rel=1e-3)


@pytest.mark.parametrize("form", ["tridiag", "band"])      # both forms of the factorisation (the library picks by size)
@pytest.mark.parametrize("n,p,N,bits,g,T,seed", [(256, 96, 800, 3, 64, 120, 1), (384, 200, 1500, 2, 32, 150, 2),
                                                  (192, 130, 150, 4, 0, 100, 3)])
def test_layer_objective_parity_other_shapes(ctx, monkeypatch, n, p, N, bits, g, T, seed, form):
    import paper_2605_11222_amd as admmq
    monkeypatch.setenv("ADMMQ_FACTOR", form)
    X, W0 = correlated_problem(n, p, N, seed, outliers=3)
    H64 = orc.hessian([X.astype(np.float64)])
    H32 = H64.astype(np.float32)
    sched = admmq.Schedule(T=T, ls_rounds=2, ls_pairs=32, seed=seed)
    codes, scales, zeros, st = ctx.quantize_layer(to_dev(H32), to_dev(W0), bits, g, sched)
    ref = orc.quantize_layer(H32.astype(np.float64), W0.astype(np.float64), bits, g, T=T, ls_rounds=2, ls_pairs=32,
                             seed=seed)
    k = codes.cpu().numpy()
    assert k.max() <= 2 ** bits - 1
    j64 = f64_objective(H32, st.lam, W0, k, scales.cpu().numpy(), zeros.cpu().numpy(), g)
    assert st.j_damp == pytest.approx(j64, rel=1e-4)
    assert abs(st.j_damp_admm - ref.j_damp_admm) <= OBJ_TOL * ref.j_damp_admm
    assert abs(st.j_damp - ref.j_damp) <= OBJ_TOL * ref.j_damp
    assert st.j_damp <= st.j_damp_admm * (1 + 1e-6)
    print(f"n={n} p={p} b={bits} g={g}: admm {st.j_damp_admm:.5g}/{ref.j_damp_admm:.5g} final {st.j_damp:.5g}/{ref.j_damp:.5g}"
          f" rtn {st.j_damp_rtn:.5g} code mismatch {np.mean(k != ref.codes):.4f}")


@pytest.mark.parametrize("form", ["tridiag", "band"])
def test_layer_is_deterministic(ctx, monkeypatch, form):
    import paper_2605_11222_amd as admmq
    monkeypatch.setenv("ADMMQ_FACTOR", form)
    X, W0 = correlated_problem(256, 64, 700, 9)
    H = to_dev(orc.hessian([X.astype(np.float64)]).astype(np.float32))
    sched = admmq.Schedule(T=60, ls_rounds=2, ls_pairs=16, seed=4)
    a = ctx.quantize_layer(H, to_dev(W0), 3, 64, sched)[0].cpu().numpy()
    b = ctx.quantize_layer(H, to_dev(W0), 3, 64, sched)[0].cpu().numpy()
    assert np.array_equal(a, b)


def test_statistics_without_objectives_give_the_same_codes(ctx):
    """The objective values in the statistics are reports (each a product of the Hessian with the error matrix),
    no step of Alg. 1: asked to leave them out, a call returns the same codes and grid, zeros for the objectives,
    and still the timings, iteration count and moves."""
    import paper_2605_11222_amd as admmq
    X, W0 = correlated_problem(256, 96, 700, 12)
    H = to_dev(orc.hessian([X.astype(np.float64)]).astype(np.float32))
    sched = admmq.Schedule(T=40, ls_rounds=2, ls_pairs=16, seed=3)
    ca, sa, za, st_a = ctx.quantize_layer(H, to_dev(W0), 3, 64, sched)
    cb, sb, zb, st_b = ctx.quantize_layer(H, to_dev(W0), 3, 64, sched, objectives=False)
    assert np.array_equal(ca.cpu().numpy(), cb.cpu().numpy())
    assert np.array_equal(sa.cpu().numpy(), sb.cpu().numpy()) and np.array_equal(za.cpu().numpy(), zb.cpu().numpy())
    assert st_a.j_damp > 0 and st_a.j_damp_rtn > 0 and st_a.j_damp_admm > 0 and st_a.j_recon > 0
    assert st_b.j_damp == 0 and st_b.j_damp_rtn == 0 and st_b.j_damp_admm == 0 and st_b.j_recon == 0
    assert st_b.iters_done == st_a.iters_done == 40 and st_b.ls_moves == st_a.ls_moves
    assert st_b.ms_total > 0 and st_b.ms_admm > 0


@pytest.mark.parametrize("n,p,bits,g,T,refresh", [
    (1024, 2048, 3, 128, 12, -1),     # 128 x 128 tiles of the product
    (2048, 6400, 4, 0, 8, -1),        # 256 x 256 tiles, one group per column
    (4096, 5120, 2, 64, 6, 3),        # 4096 columns in 256 x 256 tiles, the rest in 128 x 128; two groups within a
                                      # wave's rows; a grid-refresh attempt (a stand-alone pass) between fused ones
])
def test_projection_in_the_products_epilogue_equals_the_stand_alone_pass(ctx, monkeypatch, n, p, bits, g, T, refresh):
    """Eqs. 8-10 run as the epilogue of eq. 7's second product where the product's shape allows (W stays in
    registers).  The result must not depend on that: same codes, grid and objective as with the projection pass as
    a launch of its own in every iteration, and the same primal residuals up to the order of their sum."""
    import paper_2605_11222_amd as admmq
    gen = torch.Generator(device="cuda").manual_seed(1234 + n)
    X = torch.randn((2 * n, n), generator=gen, device="cuda", dtype=torch.float32)
    X = X + 0.5 * torch.roll(X, 1, dims=1)
    X = X * torch.exp(0.5 * torch.randn((n,), generator=gen, device="cuda"))[None, :]
    H = torch.zeros((n, n), dtype=torch.float32, device="cuda")
    ctx.accumulate_hessian(H, X)
    W0 = 0.02 * torch.randn((n, p), generator=gen, device="cuda", dtype=torch.float32)
    sched = admmq.Schedule(T=T, ls_rounds=0, refresh_iter=refresh)
    runs = {}
    for fused in ("1", "0"):
        monkeypatch.setenv("ADMMQ_FUSE_PROJECTION", fused)
        codes, scales, zeros, st = ctx.quantize_layer(H, W0, bits, g, sched, want_history=True, want_flips=False,
                                                      profile=True)
        torch.cuda.synchronize()
        runs[fused] = (codes.cpu().numpy(), scales.cpu().numpy(), zeros.cpu().numpy(), st)
    a, b = runs["1"], runs["0"]
    # the fused run launched the stand-alone pass only where it has to: iteration 0, the refresh attempt, the last
    assert b[3].n_project == T
    assert a[3].n_project == (3 if refresh >= 0 else 2)
    assert np.array_equal(a[0], b[0])
    assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    assert a[3].j_damp == pytest.approx(b[3].j_damp, rel=1e-12)     # (the objective's sum has no fixed order)
    assert a[3].refresh_accepted == b[3].refresh_accepted
    assert np.allclose(a[3].primal_res, b[3].primal_res, rtol=1e-5)


# ---------------------------------------------------------------------------------------------
# local search
# ---------------------------------------------------------------------------------------------
def ls_problem(n, p, bits, g, seed):
    X, W0 = correlated_problem(n, p, 4 * n, seed, sigma_w=1.0)
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    Hd, lam = orc.damp_hessian(H32.astype(np.float64), 0.01)
    return H32, Hd, lam, W0


def test_eq11_batch_totals_match_oracle(ctx):
    n, p, bits, g = 96, 1500, 3, 32
    H32, Hd, lam, W0 = ls_problem(n, p, bits, g, 5)
    W0d = to_dev(W0)
    scales, zeros = ctx.grid_init(W0d, bits, g)
    grid = orc.Grid(scales.cpu().numpy().astype(np.float64), zeros.cpu().numpy().astype(np.float64), bits,
                    scales.cpu().numpy() == 0)
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 2 ** bits, size=(n, p)).astype(np.uint8)
    G64 = Hd @ (W0.astype(np.float64) - grid.dequant(codes.astype(np.int64)))
    pairs = np.array(orc.sample_batch(11, 0, 0, 64, n), dtype=np.int32)
    tot = ctx.ls_evaluate(to_dev(H32), lam, to_dev(G64.astype(np.float32)), to_dev(codes), bits, g, scales,
                          to_dev(pairs)).cpu().numpy()
    want = []
    for i1, i2 in pairs:
        dL, _, _ = orc.pair_gains(Hd, G64, codes.astype(np.int64), grid, int(i1), int(i2))
        want.append(orc.column_moves(dL)[1].sum())
    assert np.allclose(tot, want, rtol=2e-4, atol=1e-4 * max(want))


@pytest.mark.parametrize("n,p,bits,g,seed,pairs", [(64, 40, 3, 16, 1, 16), (128, 300, 2, 0, 2, 16), (48, 1100, 4, 24, 3, 16),
                                                   (96, 512, 3, 0, 4, 64),      # move bytes staged 16 at a time
                                                   (80, 272, 3, 16, 5, 64),     # the last column chunk is ragged
                                                   (72, 130, 2, 0, 6, 96),      # more candidates than are prefetched
                                                   (40, 48, 3, 8, 7, 3)])
def test_local_search_against_oracle(ctx, n, p, bits, g, seed, pairs):
    H32, Hd, lam, W0 = ls_problem(n, p, bits, g, seed)
    W0d, Hdv = to_dev(W0), to_dev(H32)
    scales, zeros = ctx.grid_init(W0d, bits, g)
    sc, zr = scales.cpu().numpy(), zeros.cpu().numpy()
    grid = orc.Grid(sc.astype(np.float64), zr.astype(np.float64), bits, sc == 0)
    k0, _ = orc.rtn(W0.astype(np.float64), grid)
    codes = to_dev(k0.astype(np.uint8))
    j0 = ctx.objective(Hdv, W0d, g, scales, zeros, codes)
    assert j0 == pytest.approx(orc.objective(Hd, W0.astype(np.float64), grid.dequant(k0)), rel=1e-4)
    moves, drop = ctx.local_search(Hdv, W0d, bits, g, scales, zeros, codes, rounds=3, pairs_per_batch=pairs, seed=seed)
    ref = orc.local_search(Hd, W0.astype(np.float64), k0, grid, rounds=3, pairs_per_batch=pairs, seed=seed)
    k = codes.cpu().numpy().astype(np.int64)
    assert 0 <= k.min() and k.max() <= 2 ** bits - 1
    j1 = orc.objective(Hd, W0.astype(np.float64), grid.dequant(k))
    jr = orc.objective(Hd, W0.astype(np.float64), grid.dequant(ref.codes))
    assert moves > 0 and j1 < j0
    assert j0 - j1 == pytest.approx(drop, rel=2e-3)              # the reported decrease is the true one
    assert abs(j1 - jr) <= OBJ_TOL * jr
    assert ctx.objective(Hdv, W0d, g, scales, zeros, codes) == pytest.approx(j1, rel=1e-4)
    print(f"n={n} p={p}: J {j0:.5g} -> gpu {j1:.5g} / oracle {jr:.5g}; moves {moves} vs {ref.moves}; "
          f"identical codes: {np.array_equal(k, ref.codes)}")


@pytest.mark.parametrize("n,p,bits,g,seed,pairs,batches", [
    (64, 40, 3, 16, 1, 16, 0),        # one 256-column chunk, four blocks of 4 pairs, 32 batches: two full groups
    (128, 300, 2, 0, 2, 64, 37),      # two chunks (the second ragged), groups of 16 + 16 + 5 batches
    (96, 1100, 4, 24, 3, 64, 20),     # five chunks, 80 blocks
    (80, 272, 3, 16, 5, 33, 9),       # a candidate count that is not a multiple of 4, one short group
    (40, 4160, 3, 8, 7, 64, 16),      # 17 chunks: more blocks than compute units at one pair per thread
    (40, 8200, 2, 0, 8, 64, 5)])      # 33 chunks: too wide for the grouped form, runs batch by batch
def test_local_search_grouped_launches_equal_one_launch_per_batch(ctx, monkeypatch, n, p, bits, g, seed, pairs, batches):
    """The search as one launch per group of 16 batches (blocks hand their partial sums to one another through
    memory) against one launch per batch: same winners, so codes, move count and summed gain must be identical,
    bit for bit.  Third run: every wait is made to give up at once (forced from the host through the wait bound),
    so every kernel exits normally, no group is committed, and the host redoes everything batch by batch."""
    H32, Hd, lam, W0 = ls_problem(n, p, bits, g, seed)
    W0d, Hdv = to_dev(W0), to_dev(H32)
    scales, zeros = ctx.grid_init(W0d, bits, g)
    sc, zr = scales.cpu().numpy(), zeros.cpu().numpy()
    grid = orc.Grid(sc.astype(np.float64), zr.astype(np.float64), bits, sc == 0)
    k0, _ = orc.rtn(W0.astype(np.float64), grid)
    out = {}
    for mode, env in (("grouped", {}), ("stepwise", {"ADMMQ_LS_PERSISTENT": "0"}), ("gave_up", {"ADMMQ_LS_SPIN_TICKS": "-1"})):
        monkeypatch.delenv("ADMMQ_LS_PERSISTENT", raising=False)
        monkeypatch.delenv("ADMMQ_LS_SPIN_TICKS", raising=False)
        for k_, v_ in env.items():
            monkeypatch.setenv(k_, v_)
        codes = to_dev(k0.astype(np.uint8))
        moves, drop = ctx.local_search(Hdv, W0d, bits, g, scales, zeros, codes, rounds=3, batches_per_round=batches,
                                       pairs_per_batch=pairs, seed=seed)
        out[mode] = (codes.cpu().numpy(), moves, drop, ctx.ls_fallback_count())
        print(f"{mode}: moves {moves} drop {drop:.6g} groups redone {out[mode][3]}", flush=True)
    assert out["grouped"][3] == 0 and out["stepwise"][3] == 0 and (out["gave_up"][3] > 0 or p > 8192)
    assert out["grouped"][1] > 0
    for mode in ("stepwise", "gave_up"):
        assert np.array_equal(out[mode][0], out["grouped"][0])
        assert out[mode][1] == out["grouped"][1] and out[mode][2] == out["grouped"][2]
    ref = orc.local_search(Hd, W0.astype(np.float64), k0, grid, rounds=3, batches_per_round=batches or None,
                           pairs_per_batch=pairs, seed=seed)
    j1 = orc.objective(Hd, W0.astype(np.float64), grid.dequant(out["grouped"][0].astype(np.int64)))
    jr = orc.objective(Hd, W0.astype(np.float64), grid.dequant(ref.codes))
    assert abs(j1 - jr) <= OBJ_TOL * jr


def test_local_search_tiny_exhaustive_matches_oracle_moves(ctx):
    """n = 6, 2-bit, every ordered pair in every batch: gains are well separated, so the GPU must
    apply the same moves as the oracle, whose result the CPU suite checks against enumeration."""
    n, p, bits = 6, 3, 2
    rng = np.random.default_rng(2)
    X = rng.standard_normal((24, n)) * np.exp(0.7 * rng.standard_normal(n))
    X[:, 1:] += 0.6 * X[:, :-1]
    W0 = rng.standard_normal((n, p)).astype(np.float32)
    H32 = orc.hessian([X]).astype(np.float32)
    Hd, lam = orc.damp_hessian(H32.astype(np.float64), 0.01)
    W0d, Hdv = to_dev(W0), to_dev(H32)
    scales, zeros = ctx.grid_init(W0d, bits, 0)
    sc, zr = scales.cpu().numpy(), zeros.cpu().numpy()
    grid = orc.Grid(sc.astype(np.float64), zr.astype(np.float64), bits, sc == 0)
    k0, _ = orc.rtn(W0.astype(np.float64), grid)
    allp = list(itertools.permutations(range(n), 2))
    rounds = 12
    ref = orc.local_search(Hd, W0.astype(np.float64), k0, grid, rounds=rounds, batches_per_round=1,
                           pairs_fn=lambda r, m: allp)
    codes = to_dev(k0.astype(np.uint8))
    moves, drop = ctx.local_search(Hdv, W0d, bits, 0, scales, zeros, codes, rounds=rounds, batches_per_round=1,
                                   pairs_per_batch=len(allp), explicit_pairs=allp * rounds)
    assert np.array_equal(codes.cpu().numpy().astype(np.int64), ref.codes)
    assert moves == ref.moves
    G = Hd @ (W0.astype(np.float64) - grid.dequant(ref.codes))
    for i1, i2 in allp:                                              # exhausted neighbourhood
        assert np.all(orc.pair_gains(Hd, G, ref.codes, grid, i1, i2)[0] >= -1e-9)


def test_diagonal_hessian_applies_no_move(ctx):
    rng = np.random.default_rng(4)
    n, p = 32, 20
    H32 = np.diag(np.exp(rng.standard_normal(n))).astype(np.float32)
    W0 = rng.standard_normal((n, p)).astype(np.float32)
    W0d, Hdv = to_dev(W0), to_dev(H32)
    scales, zeros = ctx.grid_init(W0d, 3, 0)
    grid = orc.Grid(scales.cpu().numpy().astype(np.float64), zeros.cpu().numpy().astype(np.float64), 3,
                    scales.cpu().numpy() == 0)
    k0, _ = orc.rtn(W0.astype(np.float64), grid)
    t = (W0.astype(np.float64) - grid.z0) / grid.delta
    assert np.all(np.abs(t - np.floor(t) - 0.5) > 1e-3)             # no element sits on a midpoint
    codes = to_dev(k0.astype(np.uint8))
    moves, drop = ctx.local_search(Hdv, W0d, 3, 0, scales, zeros, codes, rounds=2, pairs_per_batch=32, seed=1)
    assert moves == 0 and drop == 0.0 and np.array_equal(codes.cpu().numpy(), k0.astype(np.uint8))


# ---------------------------------------------------------------------------------------------
# error paths that need the device
# ---------------------------------------------------------------------------------------------
def test_device_side_input_checks_leave_outputs_untouched(ctx):
    import paper_2605_11222_amd as admmq
    X, W0 = correlated_problem(64, 16, 200, 0)
    H = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    bad = H.copy()
    bad[3, 5] = np.nan
    with pytest.raises(admmq.AdmmqError) as e:
        ctx.quantize_layer(to_dev(bad), to_dev(W0), 4, 0, admmq.Schedule(T=5, ls_rounds=0))
    assert e.value.code == 4
    Wbad = W0.copy()
    Wbad[0, 0] = np.inf
    with pytest.raises(admmq.AdmmqError) as e:
        ctx.quantize_layer(to_dev(H), to_dev(Wbad), 4, 0, admmq.Schedule(T=5, ls_rounds=0))
    assert e.value.code == 4
    with pytest.raises(admmq.AdmmqError) as e:
        ctx.quantize_layer(to_dev(np.zeros_like(H)), to_dev(W0), 4, 0, admmq.Schedule(T=5, ls_rounds=0))
    assert e.value.code == 5
    # caller workspace too small
    small = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    c2 = admmq.Context(0)
    c2.set_workspace(small)
    with pytest.raises(admmq.AdmmqError) as e:
        c2.quantize_layer(to_dev(H), to_dev(W0), 4, 0, admmq.Schedule(T=5, ls_rounds=0))
    assert e.value.code == 6
    big = torch.empty(admmq.workspace_bytes(64, 16, 5), dtype=torch.uint8, device="cuda")
    c2.set_workspace(big)
    a = c2.quantize_layer(to_dev(H), to_dev(W0), 4, 0, admmq.Schedule(T=5, ls_rounds=1))[0]
    b = ctx.quantize_layer(to_dev(H), to_dev(W0), 4, 0, admmq.Schedule(T=5, ls_rounds=1))[0]
    assert torch.equal(a, b)
    # the same caller workspace serves grouped grids and the other formats
    import synth_inputs as si
    a = c2.quantize_layer(to_dev(H), to_dev(W0), 3, 8, admmq.Schedule(T=5, ls_rounds=1, refresh_iter=2))[0]
    b = ctx.quantize_layer(to_dev(H), to_dev(W0), 3, 8, admmq.Schedule(T=5, ls_rounds=1, refresh_iter=2))[0]
    assert torch.equal(a, b)
    flags = to_dev(si.outlier_mask(W0, 0.1).astype(np.uint8))
    a = c2.quantize_layer_format(to_dev(H), to_dev(W0), admmq.FORMAT_DUAL_GRID, 3, group_size=4, flags=flags,
                                 sched=admmq.Schedule(T=5, ls_rounds=0))[0]
    b = ctx.quantize_layer_format(to_dev(H), to_dev(W0), admmq.FORMAT_DUAL_GRID, 3, group_size=4, flags=flags,
                                  sched=admmq.Schedule(T=5, ls_rounds=0))[0]
    assert torch.equal(a, b)
    # several matrices in one call: the workspace of one layer with the summed width
    wide = torch.empty(admmq.workspace_bytes(64, 32, 5), dtype=torch.uint8, device="cuda")
    c2.set_workspace(wide)
    s5 = admmq.Schedule(T=5, ls_rounds=1)
    pair = c2.quantize_layers(to_dev(H), [to_dev(W0), to_dev(W0)], [4, 3], [0, 8], s5)
    assert torch.equal(pair[0][0], ctx.quantize_layer(to_dev(H), to_dev(W0), 4, 0, s5)[0])
    assert torch.equal(pair[1][0], ctx.quantize_layer(to_dev(H), to_dev(W0), 3, 8, s5)[0])
    c2.close()


# ---------------------------------------------------------------------------------------------
# switches, strides and bit-width extremes
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("precondition,gamma", [(False, 1.1), (True, 1.0), (False, 1.0)])
def test_ablation_switches_match_oracle(ctx, precondition, gamma):
    """Without the diagonal scaling (Sigma = I) and / or with a fixed penalty (gamma = 1): the paper's ablations."""
    import paper_2605_11222_amd as admmq
    X, W0 = correlated_problem(160, 48, 500, 21, outliers=2)
    H64 = orc.hessian([X.astype(np.float64)])
    H32 = H64.astype(np.float32)
    T = 60
    sched = admmq.Schedule(T=T, gamma=gamma, precondition=precondition, ls_rounds=0)
    codes, scales, zeros, st = ctx.quantize_layer(to_dev(H32), to_dev(W0), 3, 0, sched)
    grid = orc.Grid.fit(W0.astype(np.float64), 3, 0)
    Hd, lam = orc.damp_hessian(H32.astype(np.float64))
    ref = orc.admm(Hd, W0.astype(np.float64), grid, T=T, gamma=gamma, precondition=precondition)
    j_ref = orc.objective(Hd, W0.astype(np.float64), ref.Wq)
    assert abs(st.j_damp_admm - j_ref) <= OBJ_TOL * j_ref
    print(f"precondition={precondition} gamma={gamma}: J {st.j_damp_admm:.6g} / oracle {j_ref:.6g}, "
          f"code mismatch {np.mean(codes.cpu().numpy() != ref.codes):.4f}")


def test_strided_weights_and_explicit_full_group(ctx):
    """W0 with a leading dimension larger than p; group_size = n is the same grid as per-channel."""
    import paper_2605_11222_amd as admmq
    X, W0 = correlated_problem(128, 40, 400, 31)
    H = to_dev(orc.hessian([X.astype(np.float64)]).astype(np.float32))
    wide = torch.zeros((128, 64), dtype=torch.float32, device="cuda")
    wide[:, :40] = to_dev(W0)
    wide[:, 40:] = float("nan")                       # must never be read
    view = wide[:, :40]
    assert view.stride(0) == 64
    sched = admmq.Schedule(T=40, ls_rounds=1, ls_pairs=16, seed=2)
    a = ctx.quantize_layer(H, view, 4, 0, sched)
    b = ctx.quantize_layer(H, to_dev(W0), 4, 0, sched)
    c = ctx.quantize_layer(H, to_dev(W0), 4, 128, sched)
    for x, y in zip(a[:3], b[:3]):
        assert torch.equal(x, y)
    for x, y in zip(b[:3], c[:3]):
        assert torch.equal(x, y)
    assert a[3].j_damp == pytest.approx(b[3].j_damp, rel=1e-12)


@pytest.mark.parametrize("bits", [2, 8])
def test_bit_width_extremes(ctx, bits):
    import paper_2605_11222_amd as admmq
    X, W0 = correlated_problem(96, 33, 300, 40 + bits)
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    sched = admmq.Schedule(T=50, ls_rounds=1, ls_pairs=16, seed=1)
    codes, scales, zeros, st = ctx.quantize_layer(to_dev(H32), to_dev(W0), bits, 32, sched)
    ref = orc.quantize_layer(H32.astype(np.float64), W0.astype(np.float64), bits, 32, T=50, ls_rounds=1, ls_pairs=16, seed=1)
    k = codes.cpu().numpy()
    assert k.max() <= 2 ** bits - 1 and (bits < 8 or k.max() > 127)
    assert abs(st.j_damp - ref.j_damp) <= OBJ_TOL * ref.j_damp
    assert st.j_damp == pytest.approx(f64_objective(H32, st.lam, W0, k, scales.cpu().numpy(), zeros.cpu().numpy(), 32), rel=1e-4)


@pytest.mark.parametrize("form", ["tridiag", "band"])
def test_shared_hessian_reuses_the_factorisation(ctx, monkeypatch, form):
    """Two weight matrices that see the same activations: the second call skips Alg. 1 lines 1-3 and must return
    exactly what a call with its own factorisation returns; a different H is refused.  Both forms of the
    factorisation (the kept one decides how the later call solves)."""
    import paper_2605_11222_amd as admmq
    monkeypatch.setenv("ADMMQ_FACTOR", form)
    X, W0 = correlated_problem(192, 64, 600, 50)
    _, W1 = correlated_problem(192, 40, 600, 51)
    H = to_dev(orc.hessian([X.astype(np.float64)]).astype(np.float32))
    s = admmq.Schedule(T=40, ls_rounds=1, ls_pairs=16, seed=3)
    first = ctx.quantize_layer(H, to_dev(W0), 3, 64, s)
    own = ctx.quantize_layer(H, to_dev(W1), 4, 0, s)
    ctx.quantize_layer(H, to_dev(W0), 3, 64, s)                      # the context now holds H's factorisation
    s2 = admmq.Schedule(T=40, ls_rounds=1, ls_pairs=16, seed=3, reuse_factor=True)
    shared = ctx.quantize_layer(H, to_dev(W1), 4, 0, s2)
    for a, b in zip(own[:3], shared[:3]):
        assert torch.equal(a, b)
    assert shared[3].ms_factor < 0.2 * own[3].ms_factor
    other = H.clone()
    with pytest.raises(admmq.AdmmqError) as e:
        ctx.quantize_layer(other, to_dev(W1), 4, 0, s2)
    assert e.value.code == 7


@pytest.mark.parametrize("form", ["tridiag", "band"])
def test_batched_layers_on_a_shared_hessian(ctx, monkeypatch, form):
    """Three matrices of different width, bit width and group size in one call: the W-update products run over the
    concatenated columns (offsets 0, 64, 114: the last one off the 16-byte vector path), everything else per
    matrix.  Columns never interact (Sec. 3.5), so each matrix must get the grid of a call of its own, an
    objective within the tolerance of the oracle's run on that matrix alone, and codes that differ from its own
    call only where a product's rounding moved a near-midpoint value."""
    import paper_2605_11222_amd as admmq
    monkeypatch.setenv("ADMMQ_FACTOR", form)
    n, T = 192, 60
    X, Wa = correlated_problem(n, 64, 600, 60, outliers=2)
    _, Wb = correlated_problem(n, 50, 600, 61)
    _, Wc = correlated_problem(n, 37, 600, 62)
    Ws, bits, gs = [Wa, Wb, Wc], [3, 4, 2], [64, 0, 32]
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    H = to_dev(H32)
    s = admmq.Schedule(T=T, ls_rounds=1, ls_pairs=16, seed=5)
    alone = [ctx.quantize_layer(H, to_dev(W), b, g, s) for W, b, g in zip(Ws, bits, gs)]
    both = ctx.quantize_layers(H, [to_dev(W) for W in Ws], bits, gs, s, want_history=True)
    torch.cuda.synchronize()
    assert len(both) == 3
    for i, (W, b, g) in enumerate(zip(Ws, bits, gs)):
        codes, scales, zeros, st = both[i]
        a_codes, a_scales, a_zeros, a_st = alone[i]
        assert torch.equal(scales, a_scales) and torch.equal(zeros, a_zeros)
        k = codes.cpu().numpy()
        assert k.max() <= 2 ** b - 1
        mismatch = float(np.mean(k != a_codes.cpu().numpy()))
        j64 = f64_objective(H32, st.lam, W, k, scales.cpu().numpy(), zeros.cpu().numpy(), g)
        assert st.j_damp == pytest.approx(j64, rel=1e-4)
        assert st.j_damp_rtn == pytest.approx(a_st.j_damp_rtn, rel=1e-6)
        assert st.j_damp == pytest.approx(a_st.j_damp, rel=2e-3)
        assert st.j_damp <= st.j_damp_admm * (1 + 1e-6) <= st.j_damp_rtn
        ref = orc.quantize_layer(H32.astype(np.float64), W.astype(np.float64), b, g, T=T, ls_rounds=1, ls_pairs=16,
                                 seed=5)
        assert abs(st.j_damp_admm - ref.j_damp_admm) <= OBJ_TOL * ref.j_damp_admm
        assert abs(st.j_damp - ref.j_damp) <= OBJ_TOL * ref.j_damp
        assert st.primal_res[0] == pytest.approx(ref.admm.primal[0], rel=1e-4)
        assert st.iters_done == T and st.ms_factor == both[0][3].ms_factor
        print(f"matrix {i}: p={W.shape[1]} b={b} g={g}: final {st.j_damp:.6g} alone {a_st.j_damp:.6g} oracle "
              f"{ref.j_damp:.6g}; codes differing from its own call {mismatch:.2e}")
        assert mismatch < 5e-3
    # one matrix through the batched entry point is the single-layer call
    one = ctx.quantize_layers(H, [to_dev(Wa)], 3, 64, s)[0]
    assert torch.equal(one[0], alone[0][0])
    # a refresh is a per-matrix decision: refused here
    with pytest.raises(admmq.AdmmqError) as e:
        ctx.quantize_layers(H, [to_dev(Wa), to_dev(Wb)], 3, 0, admmq.Schedule(T=20, ls_rounds=0, refresh_iter=5))
    assert e.value.code == 3


def test_batched_layers_edge_cases(ctx):
    """The batched entry point at its limits: 64 one-column matrices (the maximum count; offsets off every vector
    path), strided weights, a non-finite value in a later matrix (refused before anything is written), and the
    schedule's symmetric / clipped grids passed through to every matrix."""
    import paper_2605_11222_amd as admmq
    n = 96
    X, Wbig = correlated_problem(n, 70, 400, 70, outliers=1)
    H = to_dev(orc.hessian([X.astype(np.float64)]).astype(np.float32))
    s = admmq.Schedule(T=30, ls_rounds=1, ls_pairs=8, seed=2)
    cols = [to_dev(np.ascontiguousarray(Wbig[:, i:i + 1])) for i in range(64)]
    many = ctx.quantize_layers(H, cols, 3, 0, s)
    assert len(many) == 64
    for i in (0, 17, 63):
        alone = ctx.quantize_layer(H, cols[i], 3, 0, s)
        assert torch.equal(many[i][0], alone[0]) and torch.equal(many[i][1], alone[1])
        assert many[i][3].j_damp == pytest.approx(alone[3].j_damp, rel=1e-9)
    with pytest.raises(admmq.AdmmqError) as e:
        ctx.quantize_layers(H, cols + [cols[0]], 3, 0, s)                 # 65 matrices
    assert e.value.code == 2
    # strided views: two matrices that are column ranges of one array (ldw = 70)
    Wd = to_dev(Wbig)
    views = [Wd[:, :33], Wd[:, 33:]]
    strided = ctx.quantize_layers(H, views, [4, 2], [0, 32], s)
    for v, b, g, got in zip(views, (4, 2), (0, 32), strided):
        alone = ctx.quantize_layer(H, v.contiguous(), b, g, s)
        assert torch.equal(got[0], alone[0]) and torch.equal(got[1], alone[1]) and torch.equal(got[2], alone[2])
    # a non-finite weight in the second matrix: refused, outputs of both untouched
    bad = Wbig[:, 33:].copy()
    bad[5, 2] = np.nan
    lib = admmq.load_library()
    import ctypes as C
    from paper_2605_11222_amd import binding
    outs = [(torch.full((n, 33), 7, dtype=torch.uint8, device="cuda"), torch.full((1, 33), -1.0, device="cuda"),
             torch.full((1, 33), -1.0, device="cuda")),
            (torch.full((n, 37), 7, dtype=torch.uint8, device="cuda"), torch.full((1, 37), -1.0, device="cuda"),
             torch.full((1, 37), -1.0, device="cuda"))]
    Wa, Wb = to_dev(np.ascontiguousarray(Wbig[:, :33])), to_dev(bad)
    layers = (binding._Layer * 2)(
        binding._Layer(Wa.data_ptr(), 33, 33, 3, 0, outs[0][0].data_ptr(), outs[0][1].data_ptr(), outs[0][2].data_ptr()),
        binding._Layer(Wb.data_ptr(), 37, 37, 3, 0, outs[1][0].data_ptr(), outs[1][1].data_ptr(), outs[1][2].data_ptr()))
    cs = binding._Schedule(30, 0.1, 1.1, 0.01, 1, 1, 0, 8, -1, 0, 0, 0.8, 0, 2)
    rc = lib.admmq_quantize_layers(ctx._h, C.c_void_p(H.data_ptr()), n, layers, 2, C.byref(cs), None)
    torch.cuda.synchronize()
    assert rc == 4
    for codes, sc, zr in outs:
        assert bool((codes == 7).all()) and bool((sc == -1.0).all()) and bool((zr == -1.0).all())
    # symmetric, clipped grids reach every matrix of the call
    s2 = admmq.Schedule(T=30, ls_rounds=0, symmetric=True, clip_points=20)
    both = ctx.quantize_layers(H, [Wa, to_dev(np.ascontiguousarray(Wbig[:, 33:]))], 3, 32, s2)
    for W, got in zip((Wa, to_dev(np.ascontiguousarray(Wbig[:, 33:]))), both):
        alone = ctx.quantize_layer(H, W, 3, 32, s2)
        assert torch.equal(got[0], alone[0]) and torch.equal(got[1], alone[1]) and torch.equal(got[2], alone[2])


@pytest.mark.parametrize("n,p,bits,g,seed", [(128, 64, 4, 0, 0), (256, 96, 3, 64, 1), (192, 130, 2, 32, 3)])
def test_quiet_stop_returns_the_codes_of_the_full_run(ctx, n, p, bits, g, seed):
    """The opt-in stopping rule (schedule.quiet_stop = K: stop once the codes have been unchanged for K iterations,
    Thm. 1): fewer iterations, the codes, grid and objectives of the run over all T iterations (whose flip history
    shows that nothing moved afterwards), and the iteration count the oracle's rule gives within a few iterations
    (fp32 against float64 trajectories)."""
    import paper_2605_11222_amd as admmq
    X, W0 = correlated_problem(n, p, 4 * n, 40 + seed, outliers=2)
    H32 = orc.hessian([X.astype(np.float64)]).astype(np.float32)
    Hd_, W0d = to_dev(H32), to_dev(W0)
    T, K = 160, 6
    full = ctx.quantize_layer(Hd_, W0d, bits, g, admmq.Schedule(T=T, ls_rounds=1, ls_pairs=16, seed=seed),
                              want_history=True)
    early = ctx.quantize_layer(Hd_, W0d, bits, g, admmq.Schedule(T=T, ls_rounds=1, ls_pairs=16, seed=seed, quiet_stop=K),
                               want_history=True)
    it = early[3].iters_done
    assert K + 1 <= it < T and full[3].iters_done == T
    flips = np.array(full[3].code_flips)
    assert np.all(flips[it - K:it] == 0) and flips[it - K - 1] != 0         # the window closed exactly there
    assert np.all(flips[it:] == 0)                                          # and nothing moved afterwards
    assert torch.equal(early[0], full[0]) and torch.equal(early[1], full[1]) and torch.equal(early[2], full[2])
    assert early[3].j_damp == pytest.approx(full[3].j_damp, rel=1e-9)
    assert early[3].primal_res[:it] == full[3].primal_res[:it] and all(v == 0.0 for v in early[3].primal_res[it:])
    assert early[3].code_flips[:it] == full[3].code_flips[:it]
    ref = orc.quantize_layer(H32.astype(np.float64), W0.astype(np.float64), bits, g, T=T, ls_rounds=1, ls_pairs=16,
                             seed=seed, quiet_stop=K)
    print(f"n={n} p={p}: stopped after {it} iterations (oracle {ref.admm.iters}) of {T}")
    assert abs(ref.admm.iters - it) <= 12
    assert abs(early[3].j_damp - ref.j_damp) <= OBJ_TOL * ref.j_damp
    # without the history arrays the rule works the same way
    plain = ctx.quantize_layer(Hd_, W0d, bits, g, admmq.Schedule(T=T, ls_rounds=1, ls_pairs=16, seed=seed, quiet_stop=K))
    assert plain[3].iters_done == it and torch.equal(plain[0], full[0])


def test_quiet_stop_in_the_batched_call(ctx):
    """Several matrices in one call with the stopping rule: the loop ends once no matrix has changed a code for K
    iterations, i.e. at the latest of the iterations at which each would stop alone; every matrix gets the codes of
    its own full run."""
    import paper_2605_11222_amd as admmq
    n, T, K = 192, 160, 6
    X, Wa = correlated_problem(n, 64, 800, 90, outliers=2)
    _, Wb = correlated_problem(n, 50, 800, 91)
    H = to_dev(orc.hessian([X.astype(np.float64)]).astype(np.float32))
    Ws, bits, gs = [to_dev(Wa), to_dev(Wb)], [3, 2], [64, 0]
    full = [ctx.quantize_layer(H, W, b, g, admmq.Schedule(T=T, ls_rounds=0)) for W, b, g in zip(Ws, bits, gs)]
    alone = [ctx.quantize_layer(H, W, b, g, admmq.Schedule(T=T, ls_rounds=0, quiet_stop=K)) for W, b, g in zip(Ws, bits, gs)]
    both = ctx.quantize_layers(H, Ws, bits, gs, admmq.Schedule(T=T, ls_rounds=0, quiet_stop=K))
    its = [a[3].iters_done for a in alone]
    print("stopped alone after", its, "iterations; together after", both[0][3].iters_done)
    assert both[0][3].iters_done == both[1][3].iters_done == max(its) < T
    for got, f in zip(both, full):
        assert torch.equal(got[0], f[0]) and torch.equal(got[1], f[1]) and torch.equal(got[2], f[2])
        assert got[3].j_damp == pytest.approx(f[3].j_damp, rel=1e-9)
