"""Seeded synthetic inputs for the ADMM-Q layer solver: calibration activations X and dense weights W0.

This module only draws random numbers and formats them (fp32 / bf16 bit patterns).  It holds none of
the method's arithmetic, so both the CPU oracle's tests and the HIP path's tests may import it.

The inputs stand in for the linear layers and calibration activations of the language models the
paper quantizes (Sec. 4.1), which are not available here.  Shapes follow those models; the per-channel
log-normal scales and the few 20x channels imitate the "channel outlier" structure the paper cites as
the reason for its diagonal scaling (Sec. 3.2).

Recipe (NumPy ``Generator(PCG64(SeedSequence([seed, stream])))``):
  stream 0          channel scales  s_c = exp(zeta_c), zeta ~ N(0,1); optionally ``n_outliers`` distinct
                    channels (drawn without replacement, after the zetas) are multiplied by 20
  stream 1          W0 ~ N(0, sigma_w^2), fp32, shape [n][p]  (n = input channels, p = output channels)
  stream 2 + chunk  X rows [chunk*chunk_rows, (chunk+1)*chunk_rows): law "gauss": z * s_c, z ~ N(0,1);
                    law "silu": SiLU(a) * b * s_c with a, b ~ N(0,1) (a drawn first, full chunk, then b)
X is fp32 for the tiny config and bf16 (round-to-nearest-even of the fp32 value, done once here) for
the others; the same bits feed the GPU and the oracle.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    seed: int
    n: int            # input channels  (rows of W0)
    p: int            # output channels (columns of W0)
    tokens: int       # N, calibration rows of X
    x_dtype: str      # "f32" | "bf16"
    x_law: str        # "gauss" | "silu"
    n_outliers: int
    sigma_w: float
    bits: int
    group_size: int   # 0 = one grid per output channel
    T: int            # ADMM iterations
    chunk_rows: int = 2048


# The five workloads (weights in [n = d_in][p = d_out] orientation).
CONFIGS = {
    "cfg1": LayerConfig("cfg1", 0, 128, 64, 512, "f32", "gauss", 0, 0.02, 4, 0, 50, chunk_rows=512),
    "cfg2": LayerConfig("cfg2", 2, 4096, 4096, 262144, "bf16", "gauss", 8, 0.02, 3, 0, 200),
    "cfg3": LayerConfig("cfg3", 2, 4096, 1024, 262144, "bf16", "gauss", 8, 0.02, 4, 128, 200),
    "cfg4": LayerConfig("cfg4", 4, 12288, 4096, 262144, "bf16", "silu", 0, 0.01, 2, 64, 300),
    "cfg5": LayerConfig("cfg5", 5, 25600, 5120, 262144, "bf16", "silu", 0, 0.01, 3, 128, 300),
}
# cfg3 shares cfg2's activations (same seed, same X streams); its W0 uses its own stream key below.


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(seed), int(stream)])))


def channel_scales(seed: int, n: int, n_outliers: int = 0) -> np.ndarray:
    """Per-input-channel activation scales, float64 [n]."""
    g = _rng(seed, 0)
    s = np.exp(g.standard_normal(n))
    if n_outliers > 0:
        idx = g.choice(n, size=n_outliers, replace=False)
        s[idx] *= 20.0
    return s


def weights(seed: int, n: int, p: int, sigma_w: float, stream: int = 1) -> np.ndarray:
    """Dense weights W0, fp32 [n][p]."""
    g = _rng(seed, stream)
    return (g.standard_normal((n, p), dtype=np.float32) * np.float32(sigma_w)).astype(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def x_chunk(seed: int, chunk: int, rows: int, n: int, law: str, scales: np.ndarray) -> np.ndarray:
    """One chunk of activations as fp32 [rows][n] (not yet rounded to bf16)."""
    g = _rng(seed, 2 + chunk)
    s = scales.astype(np.float32)
    if law == "gauss":
        z = g.standard_normal((rows, n), dtype=np.float32)
        return z * s
    if law == "silu":
        a = g.standard_normal((rows, n), dtype=np.float32)
        b = g.standard_normal((rows, n), dtype=np.float32)
        silu = a / (np.float32(1.0) + np.exp(-a))
        return silu * b * s
    raise ValueError(f"unknown law {law!r}")


def layer_weights(cfg: LayerConfig, p_slice: int | None = None) -> np.ndarray:
    """W0 of a config; ``p_slice`` keeps only the first columns (the draw is always the full matrix
    for small layers; for the big ones the slice is drawn row-block by row-block to bound memory)."""
    stream = 1 if cfg.name != "cfg3" else 1001   # cfg3 shares cfg2's X but has its own weights
    w = weights(cfg.seed, cfg.n, cfg.p, cfg.sigma_w, stream=stream)
    if p_slice is not None:
        w = np.ascontiguousarray(w[:, :p_slice])
    return w


def iter_x_chunks(cfg: LayerConfig, tokens: int | None = None):
    """Yield (chunk_index, X_chunk) where X_chunk is fp32 [rows][n] for "f32" configs and uint16
    bf16 bit patterns for "bf16" configs.  ``tokens`` truncates the stream (a prefix of the chunks)."""
    total = cfg.tokens if tokens is None else int(tokens)
    s = channel_scales(cfg.seed, cfg.n, cfg.n_outliers)
    done = 0
    c = 0
    while done < total:
        rows = min(cfg.chunk_rows, total - done)
        x = x_chunk(cfg.seed, c, cfg.chunk_rows, cfg.n, cfg.x_law, s)[:rows]
        if cfg.x_dtype == "bf16":
            yield c, f32_to_bf16_bits(x)
        else:
            yield c, np.ascontiguousarray(x, dtype=np.float32)
        done += rows
        c += 1


def chunk_as_f64(cfg: LayerConfig, xc: np.ndarray) -> np.ndarray:
    """The exact real values of a chunk as float64 (bf16 bits are widened, never re-rounded)."""
    if cfg.x_dtype == "bf16":
        return bf16_bits_to_f32(xc).astype(np.float64)
    return xc.astype(np.float64)


# ---- inputs of the other formats (Sec. 4.3): the paper takes them from other methods' artefacts, which are not
# ---- here; these stand in for them ---------------------------------------------------------------------------


def outlier_mask(W0: np.ndarray, frac: float = 0.05) -> np.ndarray:
    """[n][p] bool: in every column, the ceil(frac * n) entries of largest magnitude (ties: lowest row first)."""
    n, p = W0.shape
    k = int(np.ceil(frac * n))
    order = np.argsort(-np.abs(W0), axis=0, kind="stable")[:k]
    mask = np.zeros((n, p), dtype=bool)
    np.put_along_axis(mask, order, True, axis=0)
    return mask


def column_codebook(W0: np.ndarray, bits: int) -> np.ndarray:
    """[2^bits][p] float32, strictly ascending per column: the (l + 1/2)/L quantiles of the column, pushed apart
    by one float32 step wherever two of them coincide."""
    L = 1 << bits
    qs = (np.arange(L) + 0.5) / L
    cb = np.quantile(W0.astype(np.float64), qs, axis=0).astype(np.float32)
    for l in range(1, L):
        bump = np.nextafter(cb[l - 1], np.float32(np.inf))
        cb[l] = np.where(cb[l] <= cb[l - 1], bump, cb[l])
    return cb
