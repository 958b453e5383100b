"""Writes tests/golden/<cfg>_slice_oracle.json: what the float64 oracle returns for a column slice of the two
large workloads (12288 x 4096, 2 bits, groups of 64; 25600 x 5120, 3 bits, groups of 128), run as a problem of
its own at the workload's own schedule: Alg. 1 with T = 300, rho_0 = 0.1, gamma = 1.1, then five rounds of the
pair-swap search of Sec. 3.5 with ceil(n/2) batches of 64 pairs.

Alg. 1 acts on every output column by itself up to the local search (eqs. 7-10 are column-wise; Sec. 3.5 writes the
objective as a sum over columns), so a slice of columns with the full Hessian is the same computation the full layer
performs on those columns.  The Hessian is formed in float64 from the first H_TOKENS seeded tokens (more tokens than
input channels, so it has full rank before the damping).

Imports only the oracle and the seeded input generators.  CPU only; the eigendecomposition of the 25600-row
Hessian takes the better part of an hour on 8 cores and about 40 GB of memory.

    python tests/golden/make_large_layer_goldens.py cfg4 cfg5
"""
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import synth_inputs as si                      # noqa: E402
from oracle import admmq_oracle as orc         # noqa: E402

H_TOKENS = 32768
SLICE = 32
LS_ROUNDS = 5
LS_PAIRS = 64

_seconds = {}


def _timed(name, fn):
    def wrapper(*a, **kw):
        t0 = time.perf_counter()
        out = fn(*a, **kw)
        _seconds[name] = _seconds.get(name, 0.0) + time.perf_counter() - t0
        print(f"  {name}: {_seconds[name]:.1f} s", flush=True)
        return out
    return wrapper


def run(name):
    cfg = si.CONFIGS[name]
    n = cfg.n
    _seconds.clear()
    t0 = time.perf_counter()
    H = np.zeros((n, n))
    for c, xc in si.iter_x_chunks(cfg, H_TOKENS):
        H += orc.hessian([si.chunk_as_f64(cfg, xc)])
        print(f"{name}: Hessian chunk {c} ({time.perf_counter() - t0:.0f} s)", flush=True)
    _seconds["hessian"] = time.perf_counter() - t0
    W0 = np.ascontiguousarray(si.layer_weights(cfg)[:, :SLICE]).astype(np.float64)
    res = orc.quantize_layer(H, W0, cfg.bits, cfg.group_size, T=cfg.T, ls_rounds=LS_ROUNDS, ls_pairs=LS_PAIRS,
                             seed=cfg.seed)
    gg = n if cfg.group_size == 0 else cfg.group_size
    E = res.Wq - W0
    E_admm = res.admm.Wq - W0
    col_final = np.sum(E * (H @ E), axis=0) + res.lam * np.sum(E * E, axis=0)
    col_admm = np.sum(E_admm * (H @ E_admm), axis=0) + res.lam * np.sum(E_admm * E_admm, axis=0)
    out = {
        "what": "float64 oracle, column slice run as its own problem (Alg. 1 + Sec. 3.5 local search)",
        "config": name, "n": n, "slice_columns": SLICE, "hessian_tokens": H_TOKENS, "bits": cfg.bits,
        "group_size": cfg.group_size, "T": cfg.T, "rho0": 0.1, "gamma": 1.1, "damp": 0.01,
        "ls_rounds": LS_ROUNDS, "ls_batches": (n + 1) // 2, "ls_pairs": LS_PAIRS, "seed": cfg.seed,
        "lambda": res.lam,
        "trace_H": float(np.trace(H)),
        "j_damp_rtn": res.j_damp_rtn, "j_damp_admm": res.j_damp_admm, "j_damp": res.j_damp, "j_recon": res.j_recon,
        "j_damp_admm_per_column": [float(v) for v in col_admm],
        "j_damp_per_column": [float(v) for v in col_final],
        "ls_moves": res.ls.moves, "ls_entries_changed": res.ls.entries_changed,
        "ls_objective_drop": res.ls.objective_drop,
        "primal_residual": {str(t): res.admm.primal[t] for t in (0, 1, 2, 5, 10, 20, 50, 100, 150, 200, 250, 299)
                            if t < cfg.T},
        "rtn_code_histogram": np.bincount(res.admm.first_codes.ravel(), minlength=2 ** cfg.bits).tolist(),
        "final_code_histogram": np.bincount(res.codes.ravel(), minlength=2 ** cfg.bits).tolist(),
        "scales_sum": float(np.sum(res.scales)), "zeros_sum": float(np.sum(res.zeros)),
        "eig_min": float(res.admm.lam_eig.min()), "eig_max": float(res.admm.lam_eig.max()),
        "oracle_seconds": {k: round(v, 1) for k, v in _seconds.items()},
        "oracle_threads": os.cpu_count(),
    }
    assert abs(float(np.sum(col_final)) - res.j_damp) <= 1e-9 * res.j_damp
    assert gg * res.scales.shape[0] == n
    path = os.path.join(HERE, f"{name}_slice_oracle.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print(f"{name}: wrote {path}: rtn {res.j_damp_rtn:.6g} admm {res.j_damp_admm:.6g} final {res.j_damp:.6g} "
          f"moves {res.ls.moves}; seconds {out['oracle_seconds']}", flush=True)


if __name__ == "__main__":
    np.linalg.eigh = _timed("eigh", np.linalg.eigh)
    orc.admm = _timed("admm_incl_eigh", orc.admm)
    orc.local_search = _timed("local_search", orc.local_search)
    for name in sys.argv[1:] or ["cfg4", "cfg5"]:
        run(name)
