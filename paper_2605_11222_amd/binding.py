"""ctypes binding with the same names as include/admmq.h (argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None

EXPORTED_SYMBOLS = [
    "admmq_create", "admmq_destroy", "admmq_status_string", "admmq_workspace_bytes", "admmq_set_workspace",
    "admmq_accumulate_hessian", "admmq_quantize_layer", "admmq_local_search", "admmq_sample_pair",
    "admmq_grid_init", "admmq_factorize", "admmq_w_update", "admmq_project_dual", "admmq_objective",
    "admmq_ls_evaluate", "admmq_grid_refresh", "admmq_grid_fit", "admmq_grid_init_dual",
    "admmq_project_dual_format", "admmq_quantize_layer_format", "admmq_quantize_layers",
    "admmq_set_fast_products", "admmq_fast_products_bytes", "admmq_project_dual_noalloc", "admmq_stream_copy", "admmq_ls_fallback_count",
]

NOALLOC_SCRATCH_BYTES = 8 << 20

FORMAT_DUAL_GRID, FORMAT_CODEBOOK = 1, 2

ADMMQ_F32, ADMMQ_BF16 = 0, 1


class AdmmqError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"admmq: {what} (status {code})")
        self.code = code


class _Schedule(C.Structure):
    _fields_ = [("T", C.c_int32), ("rho0", C.c_double), ("gamma", C.c_double), ("damp", C.c_double),
                ("precondition", C.c_int32), ("ls_rounds", C.c_int32), ("ls_batches", C.c_int32),
                ("ls_pairs", C.c_int32), ("refresh_iter", C.c_int32), ("symmetric", C.c_int32),
                ("clip_points", C.c_int32), ("clip_shrink", C.c_double), ("reuse_factor", C.c_int32),
                ("seed", C.c_uint64), ("quiet_stop", C.c_int32)]


class _Stats(C.Structure):
    _fields_ = [("ms_total", C.c_float), ("ms_setup", C.c_float), ("ms_factor", C.c_float),
                ("ms_admm", C.c_float), ("ms_local_search", C.c_float),
                ("j_damp", C.c_double), ("j_damp_admm", C.c_double), ("j_damp_rtn", C.c_double),
                ("lambda_", C.c_double), ("iters_done", C.c_int32), ("ls_moves", C.c_int32),
                ("primal_res", C.POINTER(C.c_float)), ("code_flips", C.POINTER(C.c_int64)),
                ("profile", C.c_int32), ("n_gemm", C.c_int32), ("n_tridiag", C.c_int32), ("n_project", C.c_int32),
                ("n_ls_apply", C.c_int32), ("ms_gemm", C.c_float), ("ms_tridiag", C.c_float),
                ("ms_project", C.c_float), ("ms_ls_apply", C.c_float), ("refresh_accepted", C.c_int32),
                ("refresh_err_old", C.c_double), ("refresh_err_new", C.c_double), ("j_recon", C.c_double),
                ("n_gemm_project", C.c_int32), ("ms_gemm_project", C.c_float), ("skip_objectives", C.c_int32)]


class _Format(C.Structure):
    _fields_ = [("kind", C.c_int32), ("bits", C.c_int32), ("group_size", C.c_int32), ("flags", C.c_void_p),
                ("codebook", C.c_void_p), ("scales", C.c_void_p), ("zeros", C.c_void_p)]


class _Layer(C.Structure):
    _fields_ = [("W0", C.c_void_p), ("p", C.c_int64), ("ldw", C.c_int64), ("bits", C.c_int32),
                ("group_size", C.c_int32), ("codes", C.c_void_p), ("scales", C.c_void_p), ("zeros", C.c_void_p)]


class _LsParams(C.Structure):
    _fields_ = [("rounds", C.c_int32), ("batches_per_round", C.c_int32), ("pairs_per_batch", C.c_int32),
                ("damp", C.c_double), ("seed", C.c_uint64)]


def library_path() -> str:
    return os.path.join(_HERE, "libadmmq.so")


def load_library():
    """Loads libadmmq.so (built in-tree by paper_2605_11222_amd/csrc/build.sh).  No fallback."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise AdmmqError(-1, f"{path} is missing: run paper_2605_11222_amd/csrc/build.sh (there is no CPU fallback)")
    lib = C.CDLL(path)
    vp, i64, i32, dbl = C.c_void_p, C.c_int64, C.c_int32, C.c_double
    lib.admmq_create.argtypes = [C.POINTER(vp), C.c_int, vp]
    lib.admmq_destroy.argtypes = [vp]
    lib.admmq_destroy.restype = None
    lib.admmq_status_string.argtypes = [C.c_int]
    lib.admmq_status_string.restype = C.c_char_p
    lib.admmq_workspace_bytes.argtypes = [i64, i64, i32]
    lib.admmq_workspace_bytes.restype = C.c_size_t
    lib.admmq_set_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.admmq_set_fast_products.argtypes = [vp, i32]
    lib.admmq_fast_products_bytes.argtypes = [i64, i64]
    lib.admmq_fast_products_bytes.restype = C.c_size_t
    lib.admmq_accumulate_hessian.argtypes = [vp, vp, i64, vp, C.c_int, i64, i64, C.POINTER(C.c_uint64)]
    lib.admmq_quantize_layer.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, C.POINTER(_Schedule), vp, vp, vp,
                                         C.POINTER(_Stats)]
    lib.admmq_local_search.argtypes = [vp, vp, vp, i64, i64, i64, i32, i32, vp, vp, vp, C.POINTER(_LsParams),
                                       C.POINTER(i32), C.POINTER(i32), C.POINTER(dbl)]
    lib.admmq_sample_pair.argtypes = [C.c_uint64, i32, i32, i32, i64, C.POINTER(i32), C.POINTER(i32)]
    lib.admmq_sample_pair.restype = None
    lib.admmq_grid_init.argtypes = [vp, vp, i64, i64, i64, i32, i32, vp, vp]
    lib.admmq_grid_fit.argtypes = [vp, vp, i64, i64, i64, i32, i32, i32, i32, dbl, vp, vp]
    lib.admmq_factorize.argtypes = [vp, vp, i64, dbl, i32, vp, C.POINTER(dbl)]
    lib.admmq_w_update.argtypes = [vp, vp, vp, vp, i64, i64, dbl, vp]
    lib.admmq_project_dual.argtypes = [vp, vp, vp, i64, i64, vp, i32, i32, vp, vp, dbl, dbl, vp, vp,
                                       C.POINTER(dbl)]
    lib.admmq_project_dual_noalloc.argtypes = [vp, vp, vp, i64, i64, vp, i32, i32, vp, vp, dbl, dbl, vp, vp, vp]
    lib.admmq_stream_copy.argtypes = [vp, vp, vp, C.c_size_t]
    lib.admmq_ls_fallback_count.argtypes = [vp]
    lib.admmq_objective.argtypes = [vp, vp, vp, i64, i64, i64, i32, vp, vp, vp, dbl, C.POINTER(dbl)]
    lib.admmq_ls_evaluate.argtypes = [vp, vp, dbl, vp, vp, i64, i64, i32, i32, vp, vp, i32, vp]
    lib.admmq_grid_init_dual.argtypes = [vp, vp, i64, i64, i64, C.POINTER(_Format)]
    lib.admmq_project_dual_format.argtypes = [vp, vp, vp, i64, i64, vp, C.POINTER(_Format), dbl, dbl, vp, vp, vp,
                                              C.POINTER(dbl)]
    lib.admmq_quantize_layer_format.argtypes = [vp, vp, vp, i64, i64, i64, C.POINTER(_Format),
                                                C.POINTER(_Schedule), vp, vp, C.POINTER(_Stats)]
    lib.admmq_quantize_layers.argtypes = [vp, vp, i64, C.POINTER(_Layer), i32, C.POINTER(_Schedule),
                                          C.POINTER(_Stats)]
    lib.admmq_grid_refresh.argtypes = [vp, vp, vp, i64, i64, vp, i32, i32, dbl, vp, vp, C.POINTER(i32),
                                       C.POINTER(dbl), C.POINTER(dbl)]
    for name in EXPORTED_SYMBOLS:
        fn = getattr(lib, name)
        if name not in ("admmq_destroy", "admmq_status_string", "admmq_workspace_bytes", "admmq_sample_pair",
                        "admmq_fast_products_bytes"):
            fn.restype = C.c_int
    _LIB = lib
    return lib


def _check(code: int):
    if code != 0:
        raise AdmmqError(code, load_library().admmq_status_string(code).decode())


def workspace_bytes(n: int, p: int, T: int) -> int:
    return int(load_library().admmq_workspace_bytes(n, p, T))


def fast_products_bytes(n: int, p: int) -> int:
    return int(load_library().admmq_fast_products_bytes(n, p))


def sample_pair(seed: int, rnd: int, batch: int, slot: int, n: int):
    a, b = C.c_int32(), C.c_int32()
    load_library().admmq_sample_pair(seed, rnd, batch, slot, n, C.byref(a), C.byref(b))
    return a.value, b.value


@dataclass
class Schedule:
    T: int = 300
    rho0: float = 0.1
    gamma: float = 1.1
    damp: float = 0.01
    precondition: bool = True
    ls_rounds: int = 5
    ls_batches: int = 0
    ls_pairs: int = 0
    refresh_iter: int = -1
    symmetric: bool = False
    clip_points: int = 0
    clip_shrink: float = 0.8
    reuse_factor: bool = False
    seed: int = 0
    quiet_stop: int = 0


@dataclass
class LayerStats:
    ms_total: float = 0.0
    ms_setup: float = 0.0
    ms_factor: float = 0.0
    ms_admm: float = 0.0
    ms_local_search: float = 0.0
    j_damp: float = 0.0
    j_damp_admm: float = 0.0
    j_damp_rtn: float = 0.0
    lam: float = 0.0
    iters_done: int = 0
    ls_moves: int = 0
    primal_res: list = field(default_factory=list)
    code_flips: list = field(default_factory=list)
    n_gemm: int = 0
    n_tridiag: int = 0
    n_project: int = 0
    n_ls_apply: int = 0
    ms_gemm: float = 0.0
    ms_tridiag: float = 0.0
    ms_project: float = 0.0
    ms_ls_apply: float = 0.0
    refresh_accepted: bool = False
    refresh_err_old: float = 0.0
    refresh_err_new: float = 0.0
    j_recon: float = 0.0
    n_gemm_project: int = 0
    ms_gemm_project: float = 0.0


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


class Context:
    """admmq_ctx bound to a torch device and to torch's current stream on it."""

    def __init__(self, device: int = 0, stream=None):
        import torch
        self._lib = load_library()
        self._torch = torch
        self.device = int(device)
        if stream is None:
            stream = torch.cuda.current_stream(self.device)
        self.stream = stream
        h = C.c_void_p()
        _check(self._lib.admmq_create(C.byref(h), self.device, C.c_void_p(stream.cuda_stream)))
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            self._lib.admmq_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    # -- entry points (names follow include/admmq.h without the prefix) ------------------------
    def set_fast_products(self, on: bool):
        _check(self._lib.admmq_set_fast_products(self._h, 1 if on else 0))

    def set_workspace(self, buf):
        _check(self._lib.admmq_set_workspace(self._h, _ptr(buf), buf.numel() * buf.element_size()))
        self._ws = buf

    def stream_copy(self, dst, src):
        """dst <- src by the library's plain copy kernel (measurement aid); same byte size, a multiple of 16."""
        nbytes = src.numel() * src.element_size()
        assert nbytes == dst.numel() * dst.element_size()
        _check(self._lib.admmq_stream_copy(self._h, _ptr(dst), _ptr(src), nbytes))

    def ls_fallback_count(self):
        """Groups of the last local search that were redone with one launch per batch (0 normally)."""
        return int(self._lib.admmq_ls_fallback_count(self._h))

    def accumulate_hessian(self, H, X):
        """H fp32 [n][n] += X^T X for a chunk X [rows][n] (float32 or bfloat16 tensor)."""
        torch = self._torch
        n = H.shape[0]
        dt = ADMMQ_BF16 if X.dtype == torch.bfloat16 else ADMMQ_F32
        cnt = C.c_uint64(0)
        _check(self._lib.admmq_accumulate_hessian(self._h, _ptr(H), n, _ptr(X), dt, X.shape[0], X.stride(0),
                                                  C.byref(cnt)))
        return cnt.value

    def quantize_layer(self, H, W0, bits, group_size=0, sched: Schedule | None = None, want_stats=True,
                       want_history=False, profile=False, want_flips=None, objectives=True):
        """want_history: the primal residual of every iteration and, unless want_flips=False, the number of codes
        each iteration changed (asking for those makes every iteration write its codes).  objectives=False: the
        statistics without the objective values (each costs a product of the Hessian with the error matrix)."""
        torch = self._torch
        if want_flips is None:
            want_flips = want_history
        sched = sched or Schedule()
        n, p = W0.shape
        g = group_size if group_size else n
        codes = torch.empty((n, p), dtype=torch.uint8, device=W0.device)
        scales = torch.empty((n // g, p), dtype=torch.float32, device=W0.device)
        zeros = torch.empty((n // g, p), dtype=torch.float32, device=W0.device)
        cs = _Schedule(sched.T, sched.rho0, sched.gamma, sched.damp, int(sched.precondition), sched.ls_rounds,
                       sched.ls_batches, sched.ls_pairs, sched.refresh_iter, int(sched.symmetric), sched.clip_points,
                       sched.clip_shrink, int(sched.reuse_factor), sched.seed, sched.quiet_stop)
        st = _Stats()
        st.profile = int(bool(profile))
        st.skip_objectives = 0 if objectives else 1
        res = (C.c_float * sched.T)() if want_history else None
        flips = (C.c_int64 * sched.T)() if want_history and want_flips else None
        if want_history:
            st.primal_res = C.cast(res, C.POINTER(C.c_float))
        if flips is not None:
            st.code_flips = C.cast(flips, C.POINTER(C.c_int64))
        _check(self._lib.admmq_quantize_layer(self._h, _ptr(H), _ptr(W0), n, p, W0.stride(0), bits, group_size,
                                              C.byref(cs), _ptr(codes), _ptr(scales), _ptr(zeros),
                                              C.byref(st) if want_stats else None))
        out = None
        if want_stats:
            out = LayerStats(st.ms_total, st.ms_setup, st.ms_factor, st.ms_admm, st.ms_local_search, st.j_damp,
                             st.j_damp_admm, st.j_damp_rtn, st.lambda_, st.iters_done, st.ls_moves,
                             list(res) if want_history else [], list(flips) if flips is not None else [],
                             st.n_gemm, st.n_tridiag, st.n_project, st.n_ls_apply, st.ms_gemm, st.ms_tridiag,
                             st.ms_project, st.ms_ls_apply, bool(st.refresh_accepted), st.refresh_err_old,
                             st.refresh_err_new, st.j_recon, st.n_gemm_project, st.ms_gemm_project)
        return codes, scales, zeros, out

    def local_search(self, H, W0, bits, group_size, scales, zeros, codes, rounds=5, batches_per_round=0,
                     pairs_per_batch=0, damp=0.01, seed=0, explicit_pairs=None):
        n, p = W0.shape
        prm = _LsParams(rounds, batches_per_round, pairs_per_batch, damp, seed)
        moves, drop = C.c_int32(0), C.c_double(0.0)
        ep = None
        if explicit_pairs is not None:
            flat = [int(v) for pr in explicit_pairs for v in pr]
            ep = (C.c_int32 * len(flat))(*flat)
        _check(self._lib.admmq_local_search(self._h, _ptr(H), _ptr(W0), n, p, W0.stride(0), bits, group_size,
                                            _ptr(scales), _ptr(zeros), _ptr(codes), C.byref(prm), ep,
                                            C.byref(moves), C.byref(drop)))
        return moves.value, drop.value

    def grid_init(self, W0, bits, group_size=0):
        torch = self._torch
        n, p = W0.shape
        g = group_size if group_size else n
        scales = torch.empty((n // g, p), dtype=torch.float32, device=W0.device)
        zeros = torch.empty((n // g, p), dtype=torch.float32, device=W0.device)
        _check(self._lib.admmq_grid_init(self._h, _ptr(W0), n, p, W0.stride(0), bits, group_size, _ptr(scales),
                                         _ptr(zeros)))
        return scales, zeros

    def grid_fit(self, W0, bits, group_size=0, symmetric=False, clip_points=0, clip_shrink=0.8):
        torch = self._torch
        n, p = W0.shape
        g = group_size if group_size else n
        scales = torch.empty((n // g, p), dtype=torch.float32, device=W0.device)
        zeros = torch.empty((n // g, p), dtype=torch.float32, device=W0.device)
        _check(self._lib.admmq_grid_fit(self._h, _ptr(W0), n, p, W0.stride(0), bits, group_size, int(symmetric),
                                        clip_points, float(clip_shrink), _ptr(scales), _ptr(zeros)))
        return scales, zeros

    def factorize(self, H, damp=0.01, precondition=True):
        torch = self._torch
        n = H.shape[0]
        d = torch.empty((n,), dtype=torch.float32, device=H.device)
        lam = C.c_double(0.0)
        _check(self._lib.admmq_factorize(self._h, _ptr(H), n, damp, int(precondition), _ptr(d), C.byref(lam)))
        return d, lam.value

    def w_update(self, Ws, D, V, rho):
        torch = self._torch
        n, p = Ws.shape
        W = torch.empty_like(Ws)
        _check(self._lib.admmq_w_update(self._h, _ptr(Ws), _ptr(D), _ptr(V), n, p, float(rho), _ptr(W)))
        return W

    def project_dual(self, W, V, d, bits, group_size, scales, zeros, rho, rho_next, want_codes=True):
        """V is updated in place; returns codes, B, ||W-D||_F^2."""
        torch = self._torch
        n, p = W.shape
        codes = torch.empty((n, p), dtype=torch.uint8, device=W.device) if want_codes else None
        B = torch.empty_like(W)
        rs = C.c_double(0.0)
        _check(self._lib.admmq_project_dual(self._h, _ptr(W), _ptr(V), n, p, _ptr(d), bits, group_size,
                                            _ptr(scales), _ptr(zeros), float(rho), float(rho_next), _ptr(codes),
                                            _ptr(B), C.byref(rs)))
        return codes, B, rs.value

    def project_dual_noalloc(self, W, V, d, bits, group_size, scales, zeros, rho, rho_next, codes, B, res_sq):
        """The same pass for callers that cannot allocate: every output is the caller's (codes u8 [n][p] or None,
        B fp32 [n][p], res_sq a float64 device tensor of one element or None); V is updated in place.  Nothing is
        allocated here or in the library, and nothing is synchronised."""
        n, p = W.shape
        _check(self._lib.admmq_project_dual_noalloc(self._h, _ptr(W), _ptr(V), n, p, _ptr(d), bits, group_size,
                                                    _ptr(scales), _ptr(zeros), float(rho), float(rho_next),
                                                    _ptr(codes), _ptr(B), _ptr(res_sq)))

    # ---- other formats (Sec. 4.3) -------------------------------------------------------------------------
    def _format(self, kind, bits, group_size, n, p, device, flags=None, codebook=None, scales=None, zeros=None):
        """Marshals an admmq_format; a dual grid without scales / zeros gets fresh [2][n/g][p] arrays."""
        torch = self._torch
        if kind == FORMAT_DUAL_GRID and scales is None:
            g = group_size if group_size else n
            scales = torch.empty((2, n // g, p), dtype=torch.float32, device=device)
            zeros = torch.empty((2, n // g, p), dtype=torch.float32, device=device)
        fmt = _Format(kind, bits, group_size, _ptr(flags), _ptr(codebook), _ptr(scales), _ptr(zeros))
        return fmt, scales, zeros

    def grid_init_dual(self, W0, bits, flags, group_size=0):
        n, p = W0.shape
        fmt, scales, zeros = self._format(FORMAT_DUAL_GRID, bits, group_size, n, p, W0.device, flags=flags)
        _check(self._lib.admmq_grid_init_dual(self._h, _ptr(W0), n, p, W0.stride(0), C.byref(fmt)))
        return scales, zeros

    def project_dual_format(self, W, V, d, kind, bits, rho, rho_next, group_size=0, flags=None, codebook=None,
                            scales=None, zeros=None):
        """V is updated in place; returns codes, B, Xq (projected unscaled values), ||W-D||_F^2."""
        torch = self._torch
        n, p = W.shape
        fmt, _, _ = self._format(kind, bits, group_size, n, p, W.device, flags, codebook, scales, zeros)
        codes = torch.empty((n, p), dtype=torch.uint8, device=W.device)
        B = torch.empty_like(W)
        Xq = torch.empty_like(W)
        rs = C.c_double(0.0)
        _check(self._lib.admmq_project_dual_format(self._h, _ptr(W), _ptr(V), n, p, _ptr(d), C.byref(fmt),
                                                   float(rho), float(rho_next), _ptr(codes), _ptr(B), _ptr(Xq),
                                                   C.byref(rs)))
        return codes, B, Xq, rs.value

    def quantize_layer_format(self, H, W0, kind, bits, group_size=0, flags=None, codebook=None,
                              sched: Schedule | None = None, want_history=False, profile=False):
        """Alg. 1 with the projection of another format.  Returns codes, Wq, (scales, zeros) of a dual grid
        (else None), stats."""
        torch = self._torch
        sched = sched or Schedule(ls_rounds=0)
        n, p = W0.shape
        fmt, scales, zeros = self._format(kind, bits, group_size, n, p, W0.device, flags, codebook)
        codes = torch.empty((n, p), dtype=torch.uint8, device=W0.device)
        Wq = torch.empty((n, p), dtype=torch.float32, device=W0.device)
        cs = _Schedule(sched.T, sched.rho0, sched.gamma, sched.damp, int(sched.precondition), sched.ls_rounds,
                       sched.ls_batches, sched.ls_pairs, sched.refresh_iter, int(sched.symmetric), sched.clip_points,
                       sched.clip_shrink, int(sched.reuse_factor), sched.seed, sched.quiet_stop)
        st = _Stats()
        st.profile = int(bool(profile))
        res = (C.c_float * sched.T)() if want_history else None
        if want_history:
            st.primal_res = C.cast(res, C.POINTER(C.c_float))
        _check(self._lib.admmq_quantize_layer_format(self._h, _ptr(H), _ptr(W0), n, p, W0.stride(0), C.byref(fmt),
                                                     C.byref(cs), _ptr(codes), _ptr(Wq), C.byref(st)))
        out = LayerStats(st.ms_total, st.ms_setup, st.ms_factor, st.ms_admm, st.ms_local_search, st.j_damp,
                         st.j_damp_admm, st.j_damp_rtn, st.lambda_, st.iters_done, st.ls_moves,
                         list(res) if want_history else [], [], st.n_gemm, st.n_tridiag, st.n_project,
                         st.n_ls_apply, st.ms_gemm, st.ms_tridiag, st.ms_project, st.ms_ls_apply, False, 0.0, 0.0,
                         st.j_recon)
        return codes, Wq, (scales, zeros) if kind == FORMAT_DUAL_GRID else None, out

    def quantize_layers(self, H, W0s, bits, group_sizes=0, sched: Schedule | None = None, want_history=False,
                        profile=False):
        """Alg. 1 for several matrices that share H, in one call.  bits / group_sizes: one value or one per
        matrix.  Returns a list of (codes, scales, zeros, stats), one per matrix."""
        torch = self._torch
        sched = sched or Schedule()
        count = len(W0s)
        n = H.shape[0]
        bits = list(bits) if isinstance(bits, (list, tuple)) else [bits] * count
        gs = list(group_sizes) if isinstance(group_sizes, (list, tuple)) else [group_sizes] * count
        layers = (_Layer * max(count, 1))()
        stats = (_Stats * max(count, 1))()
        outs, keep = [], []
        for i, W0 in enumerate(W0s):
            p = W0.shape[1]
            g = gs[i] if gs[i] else n
            codes = torch.empty((n, p), dtype=torch.uint8, device=W0.device)
            scales = torch.empty((max(n // g, 1), p), dtype=torch.float32, device=W0.device)
            zeros = torch.empty((max(n // g, 1), p), dtype=torch.float32, device=W0.device)
            layers[i] = _Layer(_ptr(W0), p, W0.stride(0), bits[i], gs[i], _ptr(codes), _ptr(scales), _ptr(zeros))
            outs.append((codes, scales, zeros))
            if want_history:
                res = (C.c_float * sched.T)()
                stats[i].primal_res = C.cast(res, C.POINTER(C.c_float))
                keep.append(res)
        stats[0].profile = int(bool(profile))
        cs = _Schedule(sched.T, sched.rho0, sched.gamma, sched.damp, int(sched.precondition), sched.ls_rounds,
                       sched.ls_batches, sched.ls_pairs, sched.refresh_iter, int(sched.symmetric), sched.clip_points,
                       sched.clip_shrink, int(sched.reuse_factor), sched.seed, sched.quiet_stop)
        _check(self._lib.admmq_quantize_layers(self._h, _ptr(H), n, layers, count, C.byref(cs), stats))
        result = []
        for i in range(count):
            st = stats[i]
            ls = LayerStats(st.ms_total, st.ms_setup, st.ms_factor, st.ms_admm, st.ms_local_search, st.j_damp,
                            st.j_damp_admm, st.j_damp_rtn, st.lambda_, st.iters_done, st.ls_moves,
                            list(keep[i]) if want_history else [], [], st.n_gemm, st.n_tridiag, st.n_project,
                            st.n_ls_apply, st.ms_gemm, st.ms_tridiag, st.ms_project, st.ms_ls_apply, False, 0.0, 0.0,
                            st.j_recon)
            result.append(outs[i] + (ls,))
        return result

    def grid_refresh(self, W, V, d, bits, group_size, rho, scales, zeros):
        """scales/zeros are overwritten when the refit is accepted; returns (accepted, err_old, err_new)."""
        n, p = W.shape
        acc, eo, en = C.c_int32(0), C.c_double(0.0), C.c_double(0.0)
        _check(self._lib.admmq_grid_refresh(self._h, _ptr(W), _ptr(V), n, p, _ptr(d), bits, group_size, float(rho),
                                            _ptr(scales), _ptr(zeros), C.byref(acc), C.byref(eo), C.byref(en)))
        return bool(acc.value), eo.value, en.value

    def objective(self, H, W0, group_size, scales, zeros, codes, damp=0.01):
        n, p = W0.shape
        j = C.c_double(0.0)
        _check(self._lib.admmq_objective(self._h, _ptr(H), _ptr(W0), n, p, W0.stride(0), group_size, _ptr(scales),
                                         _ptr(zeros), _ptr(codes), damp, C.byref(j)))
        return j.value

    def ls_evaluate(self, H, lam, G, codes, bits, group_size, scales, pairs):
        torch = self._torch
        n, p = G.shape
        totals = torch.empty((pairs.shape[0],), dtype=torch.float32, device=G.device)
        _check(self._lib.admmq_ls_evaluate(self._h, _ptr(H), float(lam), _ptr(G), _ptr(codes), n, p, bits,
                                           group_size, _ptr(scales), _ptr(pairs), pairs.shape[0], _ptr(totals)))
        return totals
