"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module only draws random numbers and casts them.  It holds none of the
method's arithmetic (no clustering, no allocation, no packing, no loss), so it
can feed both the CPU oracle and the HIP path without coupling them.

The matrices stand in for LLaMA linear-layer weights and their diagonal-Fisher
sensitivities (the paper's W and "Gradient Square" G, Alg. 3 inputs): a narrow
Gaussian core with a small fraction of wide outliers, and heavy-tailed squared
gradients.  Real model weights and calibration data are not available here.

Recipe (draw order is part of the recipe; all draws are float64, cast to
float32 last):
    rng  = numpy.random.default_rng(SeedSequence([config_index, matrix_index]))
    base = rng.standard_normal((n, m)) * core_sigma
    mask = rng.random((n, m)) < outlier_frac
    outl = rng.standard_normal((n, m)) * outlier_sigma
    g    = rng.standard_normal((n, m))            (config 0)
           rng.standard_t(3, (n, m))              (all other configs)
    W = where(mask, outl, base);  S = g * g
"""
from __future__ import annotations

import numpy as np

# (config index) -> list of (n, m) matrices, weight core sigma, outlier sigma, S distribution
CONFIGS = {
    0: dict(shapes=[(512, 512)], core=0.02, outl=0.2, sdist="normal"),
    1: dict(shapes=[(4096, 4096)], core=0.02, outl=0.2, sdist="t3"),
    2: dict(shapes=[(11008, 4096), (11008, 4096), (4096, 11008)], core=0.02, outl=0.2, sdist="t3"),
    3: dict(shapes=[(4096, 4096)], core=0.02, outl=0.2, sdist="t3"),
    4: dict(shapes=[(22016, 8192), (8192, 22016)], core=0.015, outl=0.15, sdist="t3"),
}
OUTLIER_FRAC = 0.005


def make_ws(config: int, matrix: int = 0, n: int | None = None, m: int | None = None,
            rows: int | None = None):
    """Return (W, S) float32 C-contiguous arrays for one matrix of a config.

    n, m override the config's shape (same distributions, same seed path) for
    reduced-size parity cases.  rows keeps only the first `rows` rows of the
    full draw (the full matrix is still drawn so that row i is the same row i).
    """
    cfg = CONFIGS[config]
    if n is None or m is None:
        n, m = cfg["shapes"][matrix]
    rng = np.random.default_rng(np.random.SeedSequence([config, matrix]))
    base = rng.standard_normal((n, m)) * cfg["core"]
    mask = rng.random((n, m)) < OUTLIER_FRAC
    outl = rng.standard_normal((n, m)) * cfg["outl"]
    if cfg["sdist"] == "normal":
        g = rng.standard_normal((n, m))
    else:
        g = rng.standard_t(3, (n, m))
    W = np.where(mask, outl, base).astype(np.float32)
    S = (g * g).astype(np.float32)
    if rows is not None:
        W = np.ascontiguousarray(W[:rows])
        S = np.ascontiguousarray(S[:rows])
    return W, S


def make_ws_small(seed: int, n: int, m: int, sdist: str = "t3", core: float = 0.02,
                  outl: float = 0.2, dup_frac: float = 0.0, zero_s_frac: float = 0.0):
    """Small free-form cases for edge-case tests: same mixture, optional
    duplicated weight values and zero sensitivities."""
    rng = np.random.default_rng(np.random.SeedSequence([1000, seed]))
    base = rng.standard_normal((n, m)) * core
    mask = rng.random((n, m)) < OUTLIER_FRAC
    o = rng.standard_normal((n, m)) * outl
    g = rng.standard_normal((n, m)) if sdist == "normal" else rng.standard_t(3, (n, m))
    W = np.where(mask, o, base).astype(np.float32)
    S = (g * g).astype(np.float32)
    if dup_frac > 0:
        # overwrite a fraction of entries with a value copied from another column of the same row
        src = rng.integers(0, m, size=(n, m))
        dup = rng.random((n, m)) < dup_frac
        W = np.where(dup, np.take_along_axis(W, src, axis=1), W)
    if zero_s_frac > 0:
        S = np.where(rng.random((n, m)) < zero_s_frac, np.float32(0), S).astype(np.float32)
    return np.ascontiguousarray(W), np.ascontiguousarray(S)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) & np.uint32(0xFFFF0000)).view(np.float32)


def make_x(config: int, N: int, m: int, chunk: int = 8192):
    """Yield bf16-rounded calibration activations X (N x m) in row chunks.

    X ~ N(0,1); 1 % of the columns (feature channels), chosen once, are scaled
    by 20 (outlier channels).  Each chunk is float32 holding bf16 values."""
    rng = np.random.default_rng(np.random.SeedSequence([config, 77]))
    ncol = max(1, int(round(0.01 * m)))
    cols = rng.choice(m, size=ncol, replace=False)
    scale = np.ones(m, dtype=np.float32)
    scale[cols] = 20.0
    done = 0
    while done < N:
        c = min(chunk, N - done)
        x = rng.standard_normal((c, m), dtype=np.float32) * scale
        yield bf16_round(x)
        done += c


def make_h_host(config: int, N: int, m: int) -> np.ndarray:
    """H = X^T X / N in float64 accumulation, returned float32 (small shapes only)."""
    acc = np.zeros((m, m), dtype=np.float64)
    for x in make_x(config, N, m):
        xd = x.astype(np.float64)
        acc += xd.T @ xd
    return (acc / N).astype(np.float32)


def make_alpha(seed: int, m: int, spread: float = 0.1) -> np.ndarray:
    """A positive scaling vector near one (for tests of the scaled path)."""
    rng = np.random.default_rng(np.random.SeedSequence([2000, seed]))
    return np.exp(rng.standard_normal(m) * spread).astype(np.float32)
