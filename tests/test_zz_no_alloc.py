"""The entry point for callers that cannot allocate device memory: admmq_project_dual_noalloc (reciprocals in a
fixed array inside the library's device image) against admmq_project_dual (reciprocals in the context's arena) on
the same inputs: codes, V and B bit for bit, the residual to rounding of its block sums.  Two calls in a row on the
one array, the second on a smaller input, so stale contents of the first would show."""
import gc

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _inputs(n, p, bits, g, seed):
    rng = np.random.default_rng(seed)
    d = np.exp(0.5 * rng.standard_normal(n)).astype(np.float32)
    W0 = (0.02 * rng.standard_normal((n, p))).astype(np.float32)
    Ws = W0 * d[:, None]
    a = np.float32(np.abs(Ws).mean())
    W = Ws + np.float32(0.3) * a * rng.standard_normal((n, p), dtype=np.float32)
    V = np.float32(0.1) * a * rng.standard_normal((n, p), dtype=np.float32)
    return W0, W, V, d


def test_project_dual_noalloc_matches_project_dual_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2605_11222_amd as admmq
    ctx = admmq.Context(0)
    dev = torch.device("cuda:0")
    rho, rho_next = 2.5, 2.75
    try:
        # first call: groups of 64, 16-byte vector path;
        # second call: fewer rows and columns, one grid per column, ragged column count (scalar path)
        for (n, p, bits, g, seed) in [(1536, 1032, 3, 64, 1), (640, 257, 4, 0, 2)]:
            W0, W, V, d = _inputs(n, p, bits, g, seed)
            W0d, Wd, dd = (torch.from_numpy(x).to(dev) for x in (W0, W, d))
            scales, zeros = ctx.grid_init(W0d, bits, g)
            V_ref = torch.from_numpy(V).to(dev)
            codes_ref, B_ref, rs_ref = ctx.project_dual(Wd, V_ref, dd, bits, g, scales, zeros, rho, rho_next)
            V_new = torch.from_numpy(V).to(dev)
            codes = torch.full((n, p), 255, dtype=torch.uint8, device=dev)
            B = torch.full((n, p), float("nan"), dtype=torch.float32, device=dev)
            res = torch.full((1,), float("nan"), dtype=torch.float64, device=dev)
            # (tensors that earlier tests left in reference cycles are freed now, not somewhere inside the call;
            # a collection during the call can still only lower the figure, an allocation would raise it)
            gc.collect()
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            ctx.project_dual_noalloc(Wd, V_new, dd, bits, g, scales, zeros, rho, rho_next, codes, B, res)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() <= before
            assert torch.equal(codes, codes_ref)
            assert torch.equal(V_new, V_ref)
            assert torch.equal(B, B_ref)
            assert float(res[0]) == pytest.approx(rs_ref, rel=1e-12)
            assert int(codes.max()) == 2 ** bits - 1
            print(f"{n} x {p}, {bits} bits, group {g or n}: identical to the arena-backed call")
        # a shape whose reciprocals do not fit the fixed array is refused before any device work
        n, p, g = 4096, 4096, 4
        assert 4 * (n + (n // g) * p) > admmq.NOALLOC_SCRATCH_BYTES
        W = torch.zeros((n, p), dtype=torch.float32, device=dev)
        V = torch.zeros_like(W)
        B = torch.full_like(W, 7.0)
        sc = torch.ones((n // g, p), dtype=torch.float32, device=dev)
        with pytest.raises(admmq.AdmmqError) as e:
            ctx.project_dual_noalloc(W, V, torch.ones(n, device=dev), 3, g, sc, sc, rho, rho_next, None, B, None)
        assert e.value.code == 6          # ADMMQ_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert bool((B == 7.0).all())
    finally:
        ctx.close()
