"""Float64 CPU oracle for the ADMM-Q layer solver.  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may import this file.  The
HIP library and its Python binding never do, and nothing here imports them.

The solver is a heuristic iteration for an NP-hard problem, so there is no closed-form result to write
down: the oracle takes the algorithm's steps in the paper's order and notation (Alg. 1, eqs. 7-10,
Sec. 3.5), in NumPy float64, with the W-update in the literal form of eq. 7 through the
eigendecomposition of Sec. 3.3.  No blocking, fusion or algebraic rearrangement.

Notation: X [N][n] activations, W0 = dense weights [n][p] (n input channels, p output channels),
H = X^T X, H' = H + lambda I, Sigma = Diag(H')^{-1/2} with d_i = sqrt(H'_ii) = 1/Sigma_ii,
scaled problem Hs = Sigma H' Sigma, Ws = Sigma^{-1} W0, split variable D, unscaled dual V.

Where the paper leaves a choice open the reading taken is stated at the function that takes it.

Pins (tests/test_oracle_*.py): Hessian against a triple loop; unit diagonal of Hs; the W-update
against numpy.linalg.solve; projection against brute force over the 2^b levels; first iterate equals
round-to-nearest of W0; key inequality of App. C each iteration; rho_t * residual bounded; eq. 11
against recomputed objectives; maintained gradient against a recomputed one; n <= 6, 2-bit exhaustive
enumeration for the local search; the dual-grid and codebook projections against the uniform grid they
reduce to, brute force over the levels, and the key inequality.  The absolute objective values of the five workloads are
"parity unpinned": the paper prints no worked numeric example of the solver.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

# ----------------------------------------------------------------------------------------------
# Problem set-up
# ----------------------------------------------------------------------------------------------


def hessian(chunks) -> np.ndarray:
    """H = X^T X accumulated over row chunks (Sec. 3.1, text after eq. 1), un-normalised sum."""
    H = None
    for xc in chunks:
        xc = np.asarray(xc, dtype=np.float64)
        H = xc.T @ xc if H is None else H + xc.T @ xc
    return H


def damp_hessian(H: np.ndarray, damp: float = 0.01):
    """H' = H + lambda I (App. D, implementation details).

    Reading: the printed constant multiplies Tr(X^T X); taken literally at n in the thousands this
    would make H' nearly a multiple of I.  The sentence says it follows GPTQ, whose convention is a
    fraction of the MEAN diagonal, so lambda = damp * Tr(H) / n.  The literal reading is damp*n.
    """
    H = np.asarray(H, dtype=np.float64)
    n = H.shape[0]
    lam = damp * np.trace(H) / n
    return H + lam * np.eye(n), lam


def scale_problem(Hd: np.ndarray, W0: np.ndarray, precondition: bool = True):
    """Alg. 1 lines 1-2 (eqs. 3-4): d_i = sqrt(H'_ii); Hs = Sigma H' Sigma; Ws = Sigma^{-1} W0.
    With ``precondition`` off (the paper's ablation) Sigma = I."""
    Hd = np.asarray(Hd, dtype=np.float64)
    n = Hd.shape[0]
    diag = np.diag(Hd)
    if np.any(diag <= 0) or not np.all(np.isfinite(diag)):
        raise ValueError("non-positive diagonal entry in the damped Hessian (dead input channel)")
    d = np.sqrt(diag) if precondition else np.ones(n)
    Hs = Hd / d[:, None] / d[None, :]
    Ws = np.asarray(W0, dtype=np.float64) * d[:, None]
    return d, Hs, Ws


def grid_init(W0: np.ndarray, bits: int, group_size: int = 0):
    """Min/max grid of the dense weights, no clipping (Sec. 3.4 "Clipping heuristics"; Sec. 3.3 grid
    refresh paragraph: initialised by round-to-nearest on the dense weights).

    Reading: a group is ``group_size`` consecutive INPUT channels (rows) inside one output column;
    group_size = 0 means one grid per output column.  delta = (max-min)/(2^b-1), z0 = min (the
    real-valued offset of eq. 10).  A group with max == min gets delta = 0 by that formula; it is
    degenerate: all its codes stay 0 and it dequantizes to z0.  Returns delta, z0 with shape [n/g][p].
    """
    W0 = np.asarray(W0, dtype=np.float64)
    n, p = W0.shape
    g = n if group_size in (0, None) else int(group_size)
    if n % g != 0:
        raise ValueError("group_size must divide n")
    Wg = W0.reshape(n // g, g, p)
    mn = Wg.min(axis=1)
    mx = Wg.max(axis=1)
    delta = (mx - mn) / float(2 ** bits - 1)
    return delta, mn


def grid_fit_options(W0: np.ndarray, bits: int, group_size: int = 0, symmetric: bool = False,
                     clip_points: int = 0, clip_shrink: float = 0.8):
    """Grid fit with the two options the paper's experiments use besides the plain min/max fit.

    symmetric (Table 1 is "symmetric per-channel"; the paper gives no formula).  Reading: the printed formula
    delta = (max-min)/(2^b-1) applied to the symmetrised range [-a, a], a = max(|min|, |max|): z0 = -a,
    delta = 2a/(2^b-1); the levels are symmetric about 0.

    clip_points > 0 (Sec. 3.4 "Clipping heuristics", App. D: MSE grid search, 100 points, maximum shrink 0.8).
    Reading: candidate i = 0 .. floor(clip_shrink*clip_points)-1 shrinks the range towards 0 by the ratio
    r_i = 1 - i/clip_points, i.e. (r_i*min, r_i*max); each candidate's grid quantizes the group's dense weights
    and the candidate with the smallest squared error wins (the first one on ties, i.e. the widest).
    Returns delta, z0 [n/g][p]."""
    W0 = np.asarray(W0, dtype=np.float64)
    n, p = W0.shape
    g = n if group_size in (0, None) else int(group_size)
    if n % g != 0:
        raise ValueError("group_size must divide n")
    L = float(2 ** bits - 1)
    Wg = W0.reshape(n // g, g, p)
    mn = Wg.min(axis=1)
    mx = Wg.max(axis=1)
    if symmetric:
        a = np.maximum(np.abs(mn), np.abs(mx))
        mn, mx = -a, a
    best_delta = (mx - mn) / L
    best_z0 = mn.copy()
    if clip_points <= 0:
        return best_delta, best_z0
    best_err = None
    for i in range(int(clip_shrink * clip_points)):
        r = 1.0 - i / float(clip_points)
        z0 = r * mn
        delta = r * (mx - mn) / L
        step = np.where(delta == 0.0, 1.0, delta)
        k = np.clip(np.rint((Wg - z0[:, None, :]) / step[:, None, :]), 0, L)
        k = np.where((delta == 0.0)[:, None, :], 0.0, k)
        err = np.sum((z0[:, None, :] + k * delta[:, None, :] - Wg) ** 2, axis=1)
        if best_err is None:
            best_err = err
        else:
            better = err < best_err
            best_err = np.where(better, err, best_err)
            best_delta = np.where(better, delta, best_delta)
            best_z0 = np.where(better, z0, best_z0)
    return best_delta, best_z0


def _expand(a: np.ndarray, n: int) -> np.ndarray:
    """[n/g][p] -> [n][p] by repeating each group row g times."""
    g = n // a.shape[0]
    return np.repeat(a, g, axis=0)


@dataclass
class Grid:
    """Quantization grid theta = (delta, z0) per group, plus the degenerate-group flag.

    ``codes`` is eq. 10 on unscaled values x [n][p]: k = clamp(Round((x - z0)/delta), 0, 2^b-1).
    Round is round-half-to-even; the clamp keeps k inside the finite grid of Sec. 3.5 "Setup"."""
    delta: np.ndarray      # [n/g][p]
    z0: np.ndarray         # [n/g][p]
    bits: int
    degenerate: np.ndarray  # [n/g][p] bool

    @staticmethod
    def fit(W0, bits, group_size=0, symmetric=False, clip_points=0, clip_shrink=0.8) -> "Grid":
        W0 = np.asarray(W0, dtype=np.float64)
        if symmetric or clip_points > 0:
            delta, z0 = grid_fit_options(W0, bits, group_size, symmetric, clip_points, clip_shrink)
        else:
            delta, z0 = grid_init(W0, bits, group_size)
        return Grid(delta, z0, bits, delta == 0.0)

    def codes(self, x: np.ndarray) -> np.ndarray:
        n = x.shape[0]
        dead = _expand(self.degenerate, n)
        step = np.where(dead, 1.0, _expand(self.delta, n))
        k = np.clip(np.rint((x - _expand(self.z0, n)) / step), 0, 2 ** self.bits - 1)
        k = np.where(dead, 0.0, k)
        return k.astype(np.int64)

    def dequant(self, k: np.ndarray) -> np.ndarray:
        n = k.shape[0]
        return _expand(self.z0, n) + k.astype(np.float64) * _expand(self.delta, n)


def rtn(W0: np.ndarray, grid: Grid):
    """Round-to-nearest of the dense weights on the grid (the data-free baseline of Sec. 3.1)."""
    k = grid.codes(np.asarray(W0, dtype=np.float64))
    return k, grid.dequant(k)


def objective(Hm: np.ndarray, W0: np.ndarray, Wq: np.ndarray) -> float:
    """Tr((Wq-W0)^T Hm (Wq-W0)) : eq. 2 without the 1/2, as the column sum of Sec. 3.5 writes it."""
    E = np.asarray(Wq, dtype=np.float64) - np.asarray(W0, dtype=np.float64)
    return float(np.sum(E * (np.asarray(Hm, dtype=np.float64) @ E)))


# ----------------------------------------------------------------------------------------------
# ADMM loop (Alg. 1 lines 3-10)
# ----------------------------------------------------------------------------------------------


def w_update(U, lam, HWs, D, V, rho):
    """Eq. 7 through the eigendecomposition of Sec. 3.3:
    W = U (Lambda + rho I)^{-1} U^T (Hs Ws + rho D - V)."""
    rhs = HWs + rho * D - V
    return U @ ((U.T @ rhs) / (lam + rho)[:, None])


def project_unscaled(grid, x: np.ndarray):
    """Projection of unscaled values x onto the admissible set, as (codes, projected values).  A uniform
    ``Grid`` rounds by eq. 10; the other formats of Sec. 4.3 bring their own ``project``."""
    if hasattr(grid, "project"):
        return grid.project(x)
    k = grid.codes(x)
    return k, grid.dequant(k)


def d_update(W, V, rho, d, grid):
    """Eqs. 8 and 10: target Wt = W + V/rho; Sigma Wt is projected on the format's set; D = Sigma^{-1}(...)."""
    Wt = W + V / rho
    x = Wt / d[:, None]
    k, xq = project_unscaled(grid, x)
    Dn = d[:, None] * xq
    return k, Dn, Wt


@dataclass
class AdmmResult:
    codes: np.ndarray
    Wq: np.ndarray
    primal: list = field(default_factory=list)     # ||W^{t+1} - D^{t+1}||_F
    dual: list = field(default_factory=list)       # ||D^{t+1} - D^{t}||_F
    rho: list = field(default_factory=list)
    key_lhs: list = field(default_factory=list)    # ||D^{t+1} - Wt||^2
    key_rhs: list = field(default_factory=list)    # ||D^{t}   - Wt||^2
    first_codes: np.ndarray | None = None
    d: np.ndarray | None = None
    lam_eig: np.ndarray | None = None
    grid: "Grid | None" = None                      # the grid in force at exit (refreshed or not)
    refresh_tried: int = 0
    refresh_accepted_at: int = -1
    refresh_err_old: float = float("nan")           # ||D_old - Wt||_F^2 at the attempt
    refresh_err_new: float = float("nan")           # ||D_new - Wt||_F^2 at the attempt
    iters: int = 0                                  # iterations run (T unless quiet_stop ended the loop)


def refit_grid(x: np.ndarray, grid: Grid) -> Grid:
    """The fitting routine of the initialisation (min/max per group, no clipping) applied to the current
    continuous point x = Sigma Wt in the unscaled space (App. B "Refreshed grid")."""
    n = x.shape[0]
    g = n // grid.delta.shape[0]
    return Grid.fit(x, grid.bits, 0 if g == n else g)


def admm(Hd, W0, grid: Grid, T=300, rho0=0.1, gamma=1.1, precondition=True, refresh_iter=-1,
         quiet_stop=0) -> AdmmResult:
    """Alg. 1 lines 1-10 on the damped Hessian Hd.  rho_t = rho0 * gamma^t (Sec. 3.6), exactly T
    iterations (no early stop) unless ``quiet_stop`` is set.  Tiny negative eigenvalues from round-off are
    clamped at 0.

    quiet_stop = K > 0 (not in Alg. 1, which runs T iterations): stop after the first iteration t >= 1 at which the
    codes have been equal to those of the iteration before for K iterations in a row.  Thm. 1 (Sec. 3.6) has the
    discrete iterates D^(t) converge; on a finite grid a convergent sequence is constant from some iteration on,
    and the read-out (line 10) only needs D.  ``iters`` records the iterations run.

    Grid refresh (Sec. 3.3 "Grid refresh", App. B).  Reading: the paper does not say when a refresh is tried
    nor which continuous weights are refitted; here one attempt is made at iteration ``refresh_iter`` (-1 = never),
    the grid is refitted on the projection target Sigma Wt of that iteration, the refreshed projection is accepted
    iff eq. 12 holds (Frobenius norms over the whole layer, in the scaled variables), the discrete point is replaced
    and the dual corrected by V += rho_t (D_old - D_new), as the appendix prints it.  At most one accepted refresh."""
    W0 = np.asarray(W0, dtype=np.float64)
    d, Hs, Ws = scale_problem(Hd, W0, precondition)
    lam, U = np.linalg.eigh(Hs)
    lam = np.maximum(lam, 0.0)
    HWs = Hs @ Ws
    D = Ws.copy()
    V = np.zeros_like(Ws)
    rho = float(rho0)
    res = AdmmResult(codes=None, Wq=None, d=d, lam_eig=lam)
    k = None
    quiet = 0
    for t in range(T):
        k_before = k
        W = w_update(U, lam, HWs, D, V, rho)
        k, Dn, Wt = d_update(W, V, rho, d, grid)
        V_next = V + rho * (W - Dn)                                  # eq. 9 with the current grid
        if t == refresh_iter and res.refresh_accepted_at < 0:
            res.refresh_tried += 1
            new_grid = refit_grid(Wt / d[:, None], grid)
            k_new, D_new, _ = d_update(W, V, rho, d, new_grid)
            res.refresh_err_old = float(np.sum((Dn - Wt) ** 2))
            res.refresh_err_new = float(np.sum((D_new - Wt) ** 2))
            if res.refresh_err_new <= res.refresh_err_old:            # eq. 12
                V_next = V_next + rho * (Dn - D_new)                  # dual consistency (App. B)
                grid, k, Dn = new_grid, k_new, D_new
                res.refresh_accepted_at = t
        res.key_lhs.append(float(np.sum((Dn - Wt) ** 2)))
        res.key_rhs.append(float(np.sum((D - Wt) ** 2)))
        V = V_next
        res.primal.append(float(np.linalg.norm(W - Dn)))
        res.dual.append(float(np.linalg.norm(Dn - D)))
        res.rho.append(rho)
        if t == 0:
            res.first_codes = k.copy()
        D = Dn
        rho = rho * gamma
        res.iters = t + 1
        if quiet_stop > 0 and t >= 1:
            quiet = quiet + 1 if np.array_equal(k, k_before) else 0
            if quiet >= quiet_stop:
                break
    res.codes = k
    res.grid = grid
    if hasattr(grid, "project"):
        res.Wq = D / d[:, None]     # Sigma D^(T); entries a format leaves free have no code to decode
    else:
        res.Wq = grid.dequant(k)    # = Sigma D^(T)  (Alg. 1 line 10)
    return res


# ----------------------------------------------------------------------------------------------
# Other formats (Sec. 4.3): only the projection changes, the W- and V-updates stay as they are.
# The paper names the two formats and gives no formulas; the readings are stated at each class.
# ----------------------------------------------------------------------------------------------


@dataclass
class DualGridProjection:
    """Inliers and outliers of every group on separate uniform grids (Sec. 4.3, the ICQuant format).

    Reading: the outlier set is an input, a fixed boolean mask [n][p]; within each group of each output channel
    the entries flagged as outliers share one grid and the rest another, both with the same number of bits;
    each grid is fitted by min/max over its own subset of W0 (an empty subset gives a degenerate grid); every
    entry is rounded by eq. 10 on the grid of its own subset."""
    inlier: Grid
    outlier: Grid
    mask: np.ndarray       # [n][p] bool, True = outlier

    @staticmethod
    def fit(W0, bits, mask, group_size=0) -> "DualGridProjection":
        W0 = np.asarray(W0, dtype=np.float64)
        mask = np.asarray(mask, dtype=bool)
        n, p = W0.shape
        g = group_size if group_size > 0 else n
        levels = 2 ** bits - 1
        out = []
        for sel in (~mask, mask):
            lo = np.where(sel, W0, np.inf).reshape(n // g, g, p).min(axis=1)
            hi = np.where(sel, W0, -np.inf).reshape(n // g, g, p).max(axis=1)
            empty = hi < lo
            lo = np.where(empty, 0.0, lo)
            hi = np.where(empty, 0.0, hi)
            delta = (hi - lo) / levels
            out.append(Grid(delta, lo, bits, delta == 0.0))
        return DualGridProjection(out[0], out[1], mask)

    def project(self, x: np.ndarray):
        k_in, k_out = self.inlier.codes(x), self.outlier.codes(x)
        k = np.where(self.mask, k_out, k_in)
        xq = np.where(self.mask, self.outlier.dequant(k_out), self.inlier.dequant(k_in))
        return k, xq


@dataclass
class CodebookProjection:
    """A non-uniform codebook per output channel, optionally with entries kept dense (Sec. 4.3, the
    SqueezeLLM format).

    Reading: codebook [L][p], strictly ascending in each column, and the optional mask of kept entries are
    inputs.  A constrained entry goes to the nearest level of its column (the lower one when two are equally
    near); a kept entry is unconstrained, so its projection is the entry itself (code 0 by convention)."""
    codebook: np.ndarray               # [L][p]
    free: np.ndarray | None = None     # [n][p] bool, True = kept dense

    def project(self, x: np.ndarray):
        dist = np.abs(x[None, :, :] - self.codebook[:, None, :])       # [L][n][p]
        k = np.argmin(dist, axis=0)                                    # first minimum = lowest level on ties
        xq = np.take_along_axis(self.codebook, k, axis=0)
        if self.free is not None:
            k = np.where(self.free, 0, k)
            xq = np.where(self.free, x, xq)
        return k.astype(np.int64), xq


def quantize_layer_format(H, W0, fmt, T=300, rho0=0.1, gamma=1.1, damp=0.01, precondition=True):
    """Alg. 1 lines 1-10 with the projection of another format (no local search: its unit moves of one grid step
    are defined for uniform grids only).  Returns (AdmmResult, J of the result, J of the plain projection of W0),
    both objectives on the damped Hessian."""
    H = np.asarray(H, dtype=np.float64)
    W0 = np.asarray(W0, dtype=np.float64)
    Hd, _ = damp_hessian(H, damp)
    a = admm(Hd, W0, fmt, T, rho0, gamma, precondition)
    _, W_near = project_unscaled(fmt, W0)
    return a, objective(Hd, W0, a.Wq), objective(Hd, W0, W_near)


def project_dual_step_format_f32(W, V, rho, rho_next, d, fmt):
    """fp32 mirror of one projection + dual pass for the formats above (the uniform grid has its own below).
    Same operation order as there up to the unscaled target x; then
      dual grid : eq. 10 with the (delta, 1/delta, z0) of the entry's own subset;
      codebook  : code = number of midpoints m_l = fl(fl(c_l + c_{l+1}) / 2) strictly below x; a kept entry
                  takes D = Wt itself and a zero dual.
    Returns codes (uint8), V_new, B_new, the projected unscaled values, and the float64 sum of (W - D_new)^2."""
    f = np.float32
    W = np.asarray(W, dtype=f)
    V = np.asarray(V, dtype=f)
    n = W.shape[0]
    rho = f(rho)
    inv_rho = f(1.0) / rho
    inv_rho_next = f(1.0) / f(rho_next)
    d = np.asarray(d, dtype=f)
    inv_d = (f(1.0) / d)[:, None]
    q = V * inv_rho
    wt = W + q
    x = wt * inv_d
    free = None
    if isinstance(fmt, DualGridProjection):
        parts = []
        for gr in (fmt.inlier, fmt.outlier):
            dl = np.asarray(gr.delta, dtype=f)
            with np.errstate(divide="ignore"):
                inv_dl = np.where(dl == f(0.0), f(0.0), f(1.0) / dl).astype(f)
            parts.append((_expand(dl, n), _expand(inv_dl, n), _expand(np.asarray(gr.z0, dtype=f), n)))
        dl_e, inv_dl_e, z_e = (np.where(fmt.mask, parts[1][i], parts[0][i]) for i in range(3))
        t = (x - z_e) * inv_dl_e
        k = np.minimum(np.maximum(np.rint(t), f(0.0)), f(2 ** fmt.inlier.bits - 1))
        xq = k * dl_e + z_e
    else:
        cb = np.asarray(fmt.codebook, dtype=f)
        mid = (cb[:-1] + cb[1:]) * f(0.5)
        k = np.zeros(W.shape, dtype=np.int64)
        for l in range(mid.shape[0]):
            k += (x > mid[l][None, :])
        xq = np.take_along_axis(cb, k, axis=0)
        free = fmt.free
    Dn = d[:, None] * xq
    if free is not None:
        Dn = np.where(free, wt, Dn)
        xq = np.where(free, x, xq)
        k = np.where(free, 0, k)
    r = W - Dn
    Vn = V + rho * r
    if free is not None:
        Vn = np.where(free, f(0.0), Vn)
    Bn = Dn - Vn * inv_rho_next
    ss = float(np.sum(r.astype(np.float64) ** 2))
    return k.astype(np.uint8), Vn.astype(f), Bn.astype(f), xq.astype(f), ss


# ----------------------------------------------------------------------------------------------
# fp32 mirror of one projection + dual step, for bit-exact comparison of integer codes.
# Where floating point decides an integer both sides must decide in the same precision; the HIP
# kernel works in fp32 with this exact operation order (every operation rounded once, no fused
# multiply-add), and with reciprocals of rho, d_i and delta formed once in fp32.
# ----------------------------------------------------------------------------------------------


def project_dual_step_f32(W, V, rho, rho_next, d, delta, z0, degenerate, bits):
    """One pass of eqs. 8-10 in fp32.  Returns codes (uint8), V_new, B_new = D_new - V_new/rho_next,
    and the float64 sum of squares of (W - D_new) over the fp32 differences."""
    f = np.float32
    W = np.asarray(W, dtype=f)
    V = np.asarray(V, dtype=f)
    n = W.shape[0]
    rho = f(rho)
    inv_rho = f(1.0) / rho
    inv_rho_next = f(1.0) / f(rho_next)
    d = np.asarray(d, dtype=f)
    inv_d = (f(1.0) / d)[:, None]
    dl = np.asarray(delta, dtype=f)
    with np.errstate(divide="ignore"):
        inv_dl = np.where(dl == f(0.0), f(0.0), f(1.0) / dl).astype(f)
    dl_e = _expand(dl, n)
    inv_dl_e = _expand(inv_dl, n)
    z_e = _expand(np.asarray(z0, dtype=f), n)
    q = V * inv_rho
    wt = W + q
    x = wt * inv_d
    y = x - z_e
    t = y * inv_dl_e
    k = np.minimum(np.maximum(np.rint(t), f(0.0)), f(2 ** bits - 1))
    xq = k * dl_e + z_e          # two roundings: product, then sum
    Dn = d[:, None] * xq
    r = W - Dn
    Vn = V + rho * r
    Bn = Dn - Vn * inv_rho_next
    ss = float(np.sum(r.astype(np.float64) ** 2))
    return k.astype(np.uint8), Vn.astype(f), Bn.astype(f), ss


# ----------------------------------------------------------------------------------------------
# Pair-swap local search (Sec. 3.5)
# ----------------------------------------------------------------------------------------------

_M64 = (1 << 64) - 1


def _mix64(x: int) -> int:
    """The SplitMix64 output function (Steele, Lea, Flood 2014) applied to x + golden-ratio gamma."""
    x = (x + 0x9E3779B97F4A7C15) & _M64
    z = x
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    return z ^ (z >> 31)


def sample_pair(seed: int, rnd: int, batch: int, slot: int, n: int):
    """Counter-based draw of an ordered row pair i1 != i2 for (round, batch, slot).
    key = round*2^48 + batch*2^16 + slot; c = mix(seed xor mix(key));
    i1 = low32(c) mod n; i2 = (i1 + 1 + high32(c) mod (n-1)) mod n."""
    key = ((rnd << 48) ^ (batch << 16) ^ slot) & _M64
    c = _mix64((seed & _M64) ^ _mix64(key))
    i1 = (c & 0xFFFFFFFF) % n
    i2 = (i1 + 1 + ((c >> 32) % (n - 1))) % n
    return int(i1), int(i2)


def sample_batch(seed, rnd, batch, B, n):
    return [sample_pair(seed, rnd, batch, s, n) for s in range(B)]


_SIGNS = ((1, 1), (1, -1), (-1, 1), (-1, -1))   # fixed evaluation order of the four combinations


def pair_gains(Hd, G, codes, grid: Grid, i1: int, i2: int):
    """Eq. 11 for one row pair, all columns, all four sign combinations.
    Returns dL [4][p] with +inf where a combination leaves the grid bounds (or the group is
    degenerate), and the per-row step sizes (delta of that row's group: per-group extension of the
    per-channel delta_j of the paper)."""
    n, p = codes.shape
    g = n // grid.delta.shape[0]
    L = 2 ** grid.bits - 1
    d1 = grid.delta[i1 // g]
    d2 = grid.delta[i2 // g]
    dead = grid.degenerate[i1 // g] | grid.degenerate[i2 // g]
    k1 = codes[i1]
    k2 = codes[i2]
    dL = np.empty((4, p))
    for c, (s1, s2) in enumerate(_SIGNS):
        a = s1 * d1
        b = s2 * d2
        val = (-2.0 * a * G[i1] + a * a * Hd[i1, i1] - 2.0 * b * G[i2] + b * b * Hd[i2, i2]
               + 2.0 * a * b * Hd[i1, i2])
        ok = (k1 + s1 >= 0) & (k1 + s1 <= L) & (k2 + s2 >= 0) & (k2 + s2 <= L) & (~dead)
        dL[c] = np.where(ok, val, np.inf)
    return dL, d1, d2


def column_moves(dL):
    """Per column: index of the feasible combination with the smallest dL (first in the fixed order
    on ties), the move is taken only if that dL < 0.  Returns (combo index or -1, gain = -dL or 0)."""
    best = np.argmin(dL, axis=0)                  # argmin returns the first minimiser
    val = dL[best, np.arange(dL.shape[1])]
    take = val < 0.0
    return np.where(take, best, -1), np.where(take, -val, 0.0)


@dataclass
class LocalSearchResult:
    codes: np.ndarray
    moves: int                 # number of applied pairs
    entries_changed: int       # number of (row, column) code changes
    applied: list              # (round, batch, slot, i1, i2, total gain)
    objective_drop: float      # sum of the applied totals (= J_before - J_after)
    G: np.ndarray | None = None  # maintained gradient H'(W0 - Wq) at exit


def local_search(Hd, W0, codes, grid: Grid, rounds=5, batches_per_round=None, pairs_per_batch=64,
                 seed=0, pairs_fn=None, G=None) -> LocalSearchResult:
    """Pair-swap refinement in the UNSCALED space on the damped Hessian (objective of eq. 2).

    Reading of Sec. 3.5 (its list of steps skips one number and leaves sizes open): G = H'(W0 - Wq).
    Each round runs ``batches_per_round`` batches (default ceil(n/2), about one visit per row); a
    batch draws ``pairs_per_batch`` ordered pairs with the counter-based generator above; for every
    pair each column picks its best feasible sign combination by eq. 11 and moves only if that
    lowers the loss; the pair's total is the sum of the columns' gains; the pair with the largest
    total (lowest slot on ties) is applied if its total is positive, and G gets the rank-2
    correction.  A round that applies nothing ends the search.  ``pairs_fn(round, batch)`` may
    replace the generator (the exhaustive variant of the brute-force tests passes all pairs).
    """
    Hd = np.asarray(Hd, dtype=np.float64)
    W0 = np.asarray(W0, dtype=np.float64)
    codes = np.array(codes, dtype=np.int64, copy=True)
    n, p = codes.shape
    M = (n + 1) // 2 if batches_per_round is None else int(batches_per_round)
    if G is None:
        G = Hd @ (W0 - grid.dequant(codes))
    else:
        G = np.array(G, dtype=np.float64, copy=True)
    out = LocalSearchResult(codes, 0, 0, [], 0.0)
    for r in range(rounds):
        applied_this_round = 0
        for m in range(M):
            pairs = pairs_fn(r, m) if pairs_fn is not None else sample_batch(seed, r, m, pairs_per_batch, n)
            best_total, best_slot, best_plan = 0.0, -1, None
            for slot, (i1, i2) in enumerate(pairs):
                dL, d1, d2 = pair_gains(Hd, G, codes, grid, i1, i2)
                combo, gain = column_moves(dL)
                total = float(np.sum(gain))
                if total > best_total:
                    best_total, best_slot, best_plan = total, slot, (i1, i2, combo, d1, d2)
            if best_slot < 0:
                continue
            i1, i2, combo, d1, d2 = best_plan
            s1 = np.array([_SIGNS[c][0] if c >= 0 else 0 for c in combo], dtype=np.int64)
            s2 = np.array([_SIGNS[c][1] if c >= 0 else 0 for c in combo], dtype=np.int64)
            codes[i1] += s1
            codes[i2] += s2
            G -= np.outer(Hd[:, i1], s1 * d1) + np.outer(Hd[:, i2], s2 * d2)
            out.moves += 1
            out.entries_changed += int(np.count_nonzero(s1) + np.count_nonzero(s2))
            out.applied.append((r, m, best_slot, i1, i2, best_total))
            out.objective_drop += best_total
            applied_this_round += 1
        if applied_this_round == 0:
            break
    out.codes = codes
    out.G = G
    return out


# ----------------------------------------------------------------------------------------------
# Whole layer (Alg. 1)
# ----------------------------------------------------------------------------------------------


@dataclass
class LayerResult:
    codes: np.ndarray
    scales: np.ndarray
    zeros: np.ndarray
    Wq: np.ndarray
    j_damp: float          # objective on H' after ADMM + local search
    j_damp_admm: float     # after ADMM, before local search
    j_damp_rtn: float      # round-to-nearest on the same grid
    j_recon: float         # ||X (Wq - W0)||_F^2  (objective on the undamped H)
    admm: AdmmResult
    ls: LocalSearchResult | None
    lam: float


def quantize_layer(H, W0, bits, group_size=0, T=300, rho0=0.1, gamma=1.1, damp=0.01, precondition=True,
                   ls_rounds=5, ls_batches=None, ls_pairs=64, seed=0, refresh_iter=-1, symmetric=False,
                   clip_points=0, clip_shrink=0.8, quiet_stop=0) -> LayerResult:
    """Alg. 1 end to end from the raw (undamped) Hessian H = X^T X."""
    H = np.asarray(H, dtype=np.float64)
    W0 = np.asarray(W0, dtype=np.float64)
    Hd, lam = damp_hessian(H, damp)
    grid = Grid.fit(W0, bits, group_size, symmetric, clip_points, clip_shrink)
    k_rtn, W_rtn = rtn(W0, grid)
    a = admm(Hd, W0, grid, T, rho0, gamma, precondition, refresh_iter, quiet_stop)
    j_admm = objective(Hd, W0, a.Wq)
    j_rtn = objective(Hd, W0, W_rtn)                # on the initial grid
    grid = a.grid                                    # the local search moves on the grid in force
    codes, ls = a.codes, None
    if ls_rounds > 0:
        ls = local_search(Hd, W0, a.codes, grid, ls_rounds, ls_batches, ls_pairs, seed)
        codes = ls.codes
    Wq = grid.dequant(codes)
    return LayerResult(codes, grid.delta, grid.z0, Wq, objective(Hd, W0, Wq), j_admm, j_rtn,
                       objective(H, W0, Wq), a, ls, lam)
