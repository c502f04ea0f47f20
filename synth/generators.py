"""Seeded generators (numpy ``default_rng``) for the LCD linear-layer inputs.

Recipe (stand-ins for clustered LLaMA-2 weights and real activations):

* centroids: ``sigma * Phi^-1(p)`` at the mid-percentiles of ``2**bits`` equal-mass bins
  (12.5/37.5/62.5/87.5 % for 2 bits), sigma = 0.02 (a standard deviation), rounded to
  fp16 and sorted;
* per-row codebook: variant "A" repeats that set on every row; variant "B" gives row n
  its own sigma_n = 0.02*(1 + 0.25*u_n), u_n ~ U(-1, 1), so rows differ;
* indices: draw w ~ N(0, 0.02^2) i.i.d. and take the nearest centroid of the *base* set
  (so the inner centroids are more likely than the outer ones);
* activations: fp16 N(0,1), a seeded 1 % of the channels multiplied by 50;
* smoothing: s_k = sqrt(max_rows |x_cal[:, k]|) over a 64-row calibration batch drawn
  like the activations (same outlier channels, its own seed), fp32, floored at 1e-5.

Nothing here dequantises, divides by s, or multiplies: that is the method, not the input.
"""
from __future__ import annotations

from statistics import NormalDist
from typing import Dict, Optional

import numpy as np

BASE_SEED = 20250612
SIGMA_W = 0.02
STREAMS = {"codebook": 0, "idx": 1, "outliers": 2, "x": 3, "calib": 4}


def seed_for(config: int, matrix_id: int, stream: str) -> int:
    return BASE_SEED + 1000 * config + 10 * matrix_id + STREAMS[stream]


def centroid_set(bits: int, sigma: float = SIGMA_W) -> np.ndarray:
    """Sorted fp16 centroids at the mid-percentiles of 2**bits equal-mass Gaussian bins."""
    n = 1 << bits
    nd = NormalDist()
    vals = [sigma * nd.inv_cdf((2 * i + 1) / (2 * n)) for i in range(n)]
    return np.sort(np.asarray(vals, dtype=np.float64).astype(np.float16))


def make_codebook(N: int, bits: int, rng: np.random.Generator, variant: str = "B") -> np.ndarray:
    """fp16 [N, 2**bits] per-output-row codebook."""
    n = 1 << bits
    if variant == "A":
        return np.tile(centroid_set(bits)[None, :], (N, 1))
    if variant != "B":
        raise ValueError("variant must be 'A' or 'B'")
    u = rng.uniform(-1.0, 1.0, size=N)
    sig = SIGMA_W * (1.0 + 0.25 * u)
    nd = NormalDist()
    z = np.asarray([nd.inv_cdf((2 * i + 1) / (2 * n)) for i in range(n)], dtype=np.float64)
    return (sig[:, None] * z[None, :]).astype(np.float16)


def make_indices(N: int, K: int, bits: int, rng: np.random.Generator) -> np.ndarray:
    """uint8 [N, K] indices: nearest base centroid of an i.i.d. N(0, 0.02^2) draw."""
    cent = centroid_set(bits).astype(np.float32)
    mid = (cent[1:] + cent[:-1]) * 0.5
    out = np.empty((N, K), dtype=np.uint8)
    rows_per_chunk = max(1, (1 << 24) // K)
    for r0 in range(0, N, rows_per_chunk):
        r1 = min(N, r0 + rows_per_chunk)
        w = rng.standard_normal(size=(r1 - r0, K), dtype=np.float32) * np.float32(SIGMA_W)
        out[r0:r1] = np.searchsorted(mid, w).astype(np.uint8)
    return out


def outlier_channels(K: int, rng: np.random.Generator) -> np.ndarray:
    """A seeded choice of round(0.01*K) outlier input channels."""
    return np.sort(rng.choice(K, size=int(round(0.01 * K)), replace=False))


def make_activations(M: int, K: int, rng: np.random.Generator, outliers: np.ndarray) -> np.ndarray:
    """fp16 [M, K]: N(0,1) with the outlier channels multiplied by 50."""
    x = rng.standard_normal(size=(M, K), dtype=np.float32)
    x[:, outliers] *= np.float32(50.0)
    return x.astype(np.float16)


def make_smoothing(K: int, rng: np.random.Generator, outliers: np.ndarray, rows: int = 64) -> np.ndarray:
    """fp32 [K]: sqrt of the per-channel max |x| over a calibration batch, floored at 1e-5."""
    cal = make_activations(rows, K, rng, outliers).astype(np.float32)
    s = np.sqrt(np.max(np.abs(cal), axis=0)).astype(np.float32)
    return np.maximum(s, np.float32(1e-5))


def make_layer(config: int, matrix_id: int, N: int, K: int, bits: int, M: int,
               variant: str = "B", seed_offset: int = 0) -> Dict[str, np.ndarray]:
    """All inputs of one linear layer: codebook, idx, x, s (+ the outlier channel list)."""
    def rng(stream: str) -> np.random.Generator:
        return np.random.default_rng(seed_for(config, matrix_id, stream) + seed_offset)

    out_ch = outlier_channels(K, rng("outliers"))
    return {
        "codebook": make_codebook(N, bits, rng("codebook"), variant),
        "idx": make_indices(N, K, bits, rng("idx")),
        "x": make_activations(M, K, rng("x"), out_ch),
        "s": make_smoothing(K, rng("calib"), out_ch),
        "outliers": out_ch,
    }


def make_layer_uniform(N: int, K: int, bits: int, M: int, seed: int) -> Dict[str, np.ndarray]:
    """A cheap layer for large structural tests: indices uniform over the 2^bits codes (one integer
    draw per weight instead of a normal draw and a search), everything else as in make_layer."""
    def rng(stream: int) -> np.random.Generator:
        return np.random.default_rng([seed, stream, N, K, bits])

    out_ch = outlier_channels(K, rng(0))
    return {
        "codebook": make_codebook(N, bits, rng(1), "B"),
        "idx": rng(2).integers(0, 1 << bits, size=(N, K), dtype=np.uint8),
        "x": make_activations(M, K, rng(3), out_ch),
        "s": make_smoothing(K, rng(4), out_ch),
        "outliers": out_ch,
    }

