"""The arithmetic of the band form of the factorisation, emulated in NumPy on the CPU (no GPU, no library call).

The library reduces the scaled Hessian of a large layer to a band matrix of half-bandwidth 16 and applies the
middle factor of eq. 7 by 16 x 16 block elimination.  The GPU tests compare the result with eq. 7 as printed; these
tests pin the identities the kernels are built on, each against a dense textbook routine, so that a wrong sign,
index or transposition in the scheme itself (not in its HIP transcription) fails here:
  * the panel factorisation: two rounds of Cholesky-QR, then the Householder form I - Y T Y^T of the orthonormal
    factor from an LU factorisation of its top block with signs chosen against the pivots;
  * the two-sided update A - Y W^T - W Y^T with W = X T - 1/2 Y (T^T K T), X = A Y, K = Y^T X;
  * the block elimination S = (M + rho I)^-1 M Y = Y - rho (M + rho I)^-1 Y with the three matrices per block row,
    including what keeping r = yh - y in fp32 between the sweeps costs as rho grows."""
import numpy as np
import pytest

B = 16


def cholesky_qr2(P):
    """Q with orthonormal columns and upper R, P = Q R, by two rounds of Cholesky-QR."""
    R1 = np.linalg.cholesky(P.T @ P).T
    Q1 = P @ np.linalg.inv(R1)
    R2 = np.linalg.cholesky(Q1.T @ Q1).T
    return Q1 @ np.linalg.inv(R2), R2 @ R1


def householder_form(Q):
    """Y (unit lower trapezoidal), T (upper triangular), signs S with (I - Y T Y^T) [S; 0] = Q: LU without pivoting
    of Q - [S; 0], every sign chosen against the pivot it meets."""
    m, b = Q.shape
    L = Q.copy()
    S = np.zeros(b)
    for k in range(b):
        S[k] = -1.0 if L[k, k] >= 0 else 1.0
        L[k, k] -= S[k]
        L[k + 1:, k] /= L[k, k]
        L[k + 1:, k + 1:] -= np.outer(L[k + 1:, k], L[k, k + 1:])
    U = np.triu(L[:b])
    Y = np.tril(L, -1)
    Y[np.arange(b), np.arange(b)] = 1.0
    T = -(U * S[None, :]) @ np.linalg.inv(Y[:b].T)
    return Y, T, S


@pytest.mark.parametrize("m,seed,cond", [(64, 0, 1.0), (300, 1, 1e3), (1000, 2, 1e5)])
def test_householder_form_from_cholesky_qr(m, seed, cond):
    rng = np.random.default_rng(seed)
    P = rng.standard_normal((m, B)) @ np.diag(np.logspace(0, -np.log10(cond), B)) @ rng.standard_normal((B, B))
    Q, R = cholesky_qr2(P)
    assert np.abs(Q.T @ Q - np.eye(B)).max() < 1e-12
    Y, T, S = householder_form(Q)
    assert np.all(np.abs(np.diag(np.triu(householder_lu_pivots(Q)))) >= 1.0 - 1e-12)
    H = np.eye(m) - Y @ T @ Y.T
    assert np.abs(H.T @ H - np.eye(m)).max() < 1e-11                      # orthogonal
    assert np.allclose(np.triu(T), T) and np.allclose(np.tril(Y[:B], -1) + np.eye(B), Y[:B])
    # the reflectors are genuine Householder reflectors: tau_c = T[c][c] = 2 / |y_c|^2 (what the accumulation of Q
    # rebuilds its own T from)
    assert np.allclose(np.diag(T), 2.0 / np.sum(Y * Y, axis=0), rtol=1e-10)
    # applied to the panel it leaves the signed triangle on top and nothing below: the new block below the band
    HtP = H.T @ P
    scale = np.abs(P).max()
    assert np.abs(HtP[B:]).max() < 1e-10 * scale * cond
    assert np.allclose(HtP[:B], S[:, None] * R, atol=1e-10 * scale * cond)


def householder_lu_pivots(Q):
    L = Q.copy()
    b = Q.shape[1]
    piv = np.zeros((b, b))
    for k in range(b):
        s = -1.0 if L[k, k] >= 0 else 1.0
        L[k, k] -= s
        piv[k, k] = L[k, k]
        L[k + 1:, k] /= L[k, k]
        L[k + 1:, k + 1:] -= np.outer(L[k + 1:, k], L[k, k + 1:])
    return piv


def test_two_sided_update_by_one_product_and_one_rank_2b_update():
    rng = np.random.default_rng(3)
    m = 200
    A = rng.standard_normal((m, m))
    A = A + A.T
    Q, _ = cholesky_qr2(rng.standard_normal((m, B)))
    Y, T, _ = householder_form(Q)
    H = np.eye(m) - Y @ T @ Y.T
    X = A @ Y
    K = Y.T @ X
    W = X @ T - 0.5 * Y @ (T.T @ K @ T)
    assert np.allclose(A - Y @ W.T - W @ Y.T, H.T @ A @ H, atol=1e-10)


def random_band_spd(n, rng, lo=0.02):
    """Symmetric positive definite with half-bandwidth 16 and a smallest eigenvalue near lo."""
    M = np.zeros((n, n))
    for t in range(B + 1):
        v = rng.standard_normal(n - t) * (0.5 ** (t > 0))
        M += np.diag(v, -t)
    M = M + M.T
    w = np.linalg.eigvalsh(M)
    return M + (lo - w[0]) * np.eye(n)


def block_factors(M, rho):
    """F_I, rho Delta_I^-1, G_I of M + rho I, M block tridiagonal in 16 x 16 blocks."""
    nb = M.shape[0] // B
    F, Dr, G = [], [], []
    inv_prev = np.zeros((B, B))
    E_prev = np.zeros((B, B))
    for I in range(nb):
        D = M[I * B:(I + 1) * B, I * B:(I + 1) * B]
        E = M[(I + 1) * B:(I + 2) * B, I * B:(I + 1) * B] if I + 1 < nb else np.zeros((B, B))
        f = E_prev @ inv_prev
        delta = D + rho * np.eye(B) - f @ E_prev.T
        inv = np.linalg.inv(delta)
        F.append(f)
        Dr.append(rho * inv)
        G.append(inv @ E.T)
        inv_prev, E_prev = inv, E
    return F, Dr, G


def block_solve(F, Dr, G, Y, r_dtype=np.float64):
    """S = Y - u with u = rho (M + rho I)^-1 Y; between the sweeps only r = yh - y survives, in r_dtype."""
    nb = len(F)
    Yb = Y.reshape(nb, B, -1)
    r = np.zeros_like(Yb, dtype=r_dtype)
    yh = np.zeros_like(Yb[0])
    for I in range(nb):
        r[I] = (-(F[I] @ yh)).astype(r_dtype)
        yh = Yb[I] + r[I].astype(np.float64)
    S = np.zeros_like(Yb)
    u = np.zeros_like(Yb[0])
    for I in range(nb - 1, -1, -1):
        yh = Yb[I] + r[I].astype(np.float64)
        u = Dr[I] @ yh - G[I] @ u
        S[I] = Yb[I] - u
    return S.reshape(Y.shape)


@pytest.mark.parametrize("rho", [0.1, 1.0, 37.0, 1.7e7])
def test_block_elimination_is_the_middle_factor_of_eq7(rho):
    rng = np.random.default_rng(4)
    n, p = 5 * B, 7
    M = random_band_spd(n, rng)
    assert np.abs(np.tril(M, -B - 1)).max() == 0.0
    E0 = M[B:2 * B, :B]
    assert np.allclose(E0, np.triu(E0))                       # the blocks below the diagonal are upper triangular
    Y = rng.standard_normal((n, p))
    want = np.linalg.solve(M + rho * np.eye(n), M @ Y)
    got = block_solve(*block_factors(M, rho), Y)
    assert np.allclose(got, want, rtol=0, atol=1e-12 * np.abs(Y).max() * max(1.0, 1.0 / rho) * 1e3)


def test_keeping_r_in_fp32_costs_relative_to_the_result_not_to_y():
    """At a large penalty S is of the size |M Y| / rho.  With r = yh - y kept in fp32 the error of S stays a few
    units of 2^-24 of S itself; had yh been kept in fp32 instead, the error would be 2^-24 of |Y|, many orders of
    magnitude above S, and the dual update multiplies it by rho."""
    rng = np.random.default_rng(5)
    n, p, rho = 8 * B, 5, 1.0e7
    M = random_band_spd(n, rng)
    Y = rng.standard_normal((n, p)).astype(np.float32).astype(np.float64)
    want = np.linalg.solve(M + rho * np.eye(n), M @ Y)
    fac = block_factors(M, rho)
    got = block_solve(*fac, Y, r_dtype=np.float32)
    size = np.abs(want).max()
    assert size < 1e-5 * np.abs(Y).max()
    assert np.abs(got - want).max() < 2.0 ** -20 * size
    # the alternative, for contrast: yh rounded to fp32 between the sweeps
    nb = n // B
    Yb = Y.reshape(nb, B, -1)
    F, Dr, G = fac
    yhs = []
    yh = np.zeros_like(Yb[0])
    for I in range(nb):
        yh = Yb[I] - F[I] @ yh
        yhs.append(yh.astype(np.float32).astype(np.float64))
    u = np.zeros_like(Yb[0])
    worse = np.zeros_like(Yb)
    for I in range(nb - 1, -1, -1):
        u = Dr[I] @ yhs[I] - G[I] @ u
        worse[I] = Yb[I] - u
    assert np.abs(worse.reshape(Y.shape) - want).max() > 100 * np.abs(got - want).max()
