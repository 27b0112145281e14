"""Seeded synthetic inputs for the f16 GEMM hot path.

This module holds no GEMM arithmetic: it only draws the A, B and C0 matrices
(numpy, on the host) that both the HIP path and the CPU oracle are fed with,
and names the workloads.  The paper measures on no dataset (Evaluation
section: square problems, 1024 to 16384); every matrix here comes from
`numpy.random.default_rng(seed)`, drawn in float64 and rounded to float16.
"""
from __future__ import annotations

import numpy as np

# name -> (M, N, K, distribution of A and B, distribution of C0, modes)
WORKLOADS = {
    "sq256_uniform":    (256, 256, 256, "uniform", "zeros", ("f32",)),
    "sq256_int":        (256, 256, 256, "int2", "zeros", ("f32", "f16")),
    "sq1024_uniform":   (1024, 1024, 1024, "uniform", "uniform", ("f32", "f16")),
    "sq8192_normal":    (8192, 8192, 8192, "normal_rsqrtk", "zeros", ("f32", "f16")),
    "ffn_up":           (16384, 3072, 768, "normal_0p02", "zeros", ("f32",)),
    "ffn_down":         (16384, 768, 3072, "normal_0p02", "zeros", ("f32",)),
    "qkv":              (16384, 2304, 768, "normal_0p02", "zeros", ("f32",)),
    "ragged4000":       (4000, 4000, 4000, "normal_0p02", "zeros", ("f32",)),
    # skinny: a few rows against a large weight matrix (bound by streaming B)
    "skinny16":         (16, 8192, 8192, "normal_0p02", "zeros", ("f32", "f16")),
    "skinny256":        (256, 4096, 16384, "normal_0p02", "zeros", ("f32", "f16")),
}
SQUARE_SWEEP = tuple(range(1024, 16384 + 1, 1024))  # uniform A, B; C0 zero; both modes


def draw(rng: np.random.Generator, shape, dist: str, K: int) -> np.ndarray:
    """float64 values of the named distribution (the recipe of every operand here; bench.py's
    MFMA-only and loop-budget legs draw their register operands from the workload's own)."""
    if dist == "uniform":
        x = rng.uniform(-1.0, 1.0, size=shape)
    elif dist == "int2":
        x = rng.integers(-2, 3, size=shape).astype(np.float64)
    elif dist == "int1":
        x = rng.integers(-1, 2, size=shape).astype(np.float64)
    elif dist == "normal_rsqrtk":
        x = rng.standard_normal(size=shape) / np.sqrt(float(max(K, 1)))
    elif dist == "normal_0p02":
        x = rng.standard_normal(size=shape) * 0.02
    elif dist == "zeros":
        x = np.zeros(shape, dtype=np.float64)
    else:
        raise ValueError(f"unknown distribution {dist!r}")
    return x


def make_inputs(M: int, N: int, K: int, dist_ab: str, dist_c: str, seed: int = 0,
                c_dtype=np.float32, lda: int | None = None, ldb: int | None = None,
                ldc: int | None = None):
    """Return (A, B, C0): float16 M x K, float16 K x N, `c_dtype` M x N.

    With a leading dimension larger than the row length the returned array is
    a view of the first columns of a wider buffer whose padding holds NaN, so
    that reading the padding shows up in the result.
    """
    rng = np.random.default_rng(seed)

    def padded(shape, dist, dtype, ld):
        rows, cols = shape
        vals = draw(rng, shape, dist, K).astype(dtype)
        if ld is None or ld == cols:
            return np.ascontiguousarray(vals)
        if ld < cols:
            raise ValueError("leading dimension below row length")
        buf = np.full((rows, ld), np.nan, dtype=dtype)
        buf[:, :cols] = vals
        return buf[:, :cols]

    A = padded((M, K), dist_ab, np.float16, lda)
    B = padded((K, N), dist_ab, np.float16, ldb)
    C0 = padded((M, N), dist_c, c_dtype, ldc)
    return A, B, C0


def workload_inputs(name: str, mode: str = "f32", seed: int = 0):
    """Inputs of a named workload; mode "f32" gives float32 C0, "f16" float16."""
    M, N, K, dab, dc, modes = WORKLOADS[name]
    if mode not in modes:
        raise ValueError(f"workload {name} is not run in mode {mode}")
    return make_inputs(M, N, K, dab, dc, seed, np.float32 if mode == "f32" else np.float16)


def sample_rows(M: int, nrows: int, tile: int, seed: int = 0) -> np.ndarray:
    """A sorted sample of row indices: first, last, both sides of some tile
    boundaries, and the rest uniform at random without repetition."""
    rng = np.random.default_rng(seed + 977)
    picked = {0, M - 1}
    bounds = np.arange(tile, M, tile)
    if bounds.size:
        for b in rng.choice(bounds, size=min(bounds.size, max(1, nrows // 4)), replace=False):
            picked.update((int(b) - 1, int(b)))
    while len(picked) < min(nrows, M):
        picked.add(int(rng.integers(0, M)))
    return np.array(sorted(picked), dtype=np.int64)
