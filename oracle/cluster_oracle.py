"""CPU oracle for the clustering-side steps that need no calibration data.  TEST INFRASTRUCTURE ONLY.

Plain numpy in fp64 (every fp16 input converts exactly), no blocking, no shortcuts:

* nearest-centroid assignment -- a weight belongs to the cluster whose centroid is closest.  This is
  the state the reclassification rule of Sec. 3.2 (Eq. 6) preserves: a weight changes cluster once
  it crosses half the distance to a neighbouring centroid, i.e. once that neighbour is the nearer
  one.  A weight exactly half way between two centroids has crossed nothing and stays with the lower.
* cluster sizes n_i (the "number of points in each cluster" of Sec. 3.3).
* merge of the two closest centroids into their count-weighted mean (Sec. 3.3, Eq. 8).  The printed
  formula pairs each centroid with the OTHER cluster's count; the sentence above it defines the new
  centroid as the average weighted by the clusters' own sizes, which is also the only choice that
  keeps sum_i n_i C_i (the clustered weights' total) unchanged.  That reading is taken here.

Codebooks are per output row, [N, 2**bits], of which the first `ncent` entries are in use and
strictly ascending.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def assign_nearest(w: np.ndarray, codebook: np.ndarray, ncent: int) -> np.ndarray:
    """idx[n, k] = argmin_i |w[n, k] - C[n, i]| over i < ncent; equal distances go to the lower index."""
    w64 = np.asarray(w, dtype=np.float16).astype(np.float64)
    c64 = np.asarray(codebook, dtype=np.float16).astype(np.float64)[:, :ncent]
    dist = np.abs(w64[:, :, None] - c64[:, None, :])          # [N, K, ncent], exact in fp64
    return np.argmin(dist, axis=2).astype(np.uint8)             # first minimum = lowest index


def cluster_counts(idx: np.ndarray, nslots: int) -> np.ndarray:
    """counts[n, i] = number of k with idx[n, k] == i, for i < nslots."""
    idx = np.asarray(idx)
    return np.stack([np.bincount(row, minlength=nslots)[:nslots] for row in idx]).astype(np.uint32)


def merge_closest(codebook: np.ndarray, counts: np.ndarray, idx: np.ndarray, ncent: int):
    """Per row: the adjacent pair (a, a+1) with the smallest gap (lowest a on equal gaps) becomes one
    centroid, the mean of the two weighted by their cluster sizes (the plain mean if both are empty).
    Returns (new codebook fp64 [N, 2**bits] with ncent-1 entries in use and zeros behind them,
    merged position a [N], re-numbered indices)."""
    c64 = np.asarray(codebook, dtype=np.float16).astype(np.float64)
    cnt = np.asarray(counts).astype(np.float64)
    N, slots = c64.shape
    out = np.zeros_like(c64)
    merged = np.zeros(N, dtype=np.uint8)
    for n in range(N):
        gaps = c64[n, 1:ncent] - c64[n, :ncent - 1]
        a = int(np.argmin(gaps))
        na, nb = cnt[n, a], cnt[n, a + 1]
        new = (na * c64[n, a] + nb * c64[n, a + 1]) / (na + nb) if na + nb > 0 else 0.5 * (c64[n, a] + c64[n, a + 1])
        row = np.concatenate([c64[n, :a], [new], c64[n, a + 2:ncent]])
        out[n, :ncent - 1] = row
        merged[n] = a
    idx = np.asarray(idx, dtype=np.uint8)
    new_idx = idx - (idx > merged[:, None]).astype(np.uint8)
    return out, merged, new_idx


def round_to_half(v: Fraction) -> np.float16:
    """The fp16 number nearest to the rational v, ties to the even mantissa (IEEE 754 roundTiesToEven),
    straight from the format: normal numbers are m * 2^(e-10) with 1024 <= m < 2048 and -14 <= e <= 15,
    subnormal ones m * 2^-24 with m < 1024.  |v| must be at most the largest finite fp16 number."""
    v = Fraction(v)
    sign, a = (-1 if v < 0 else 1), abs(v)
    if a > 65504:
        raise ValueError("beyond the fp16 range")
    e = -14
    while e < 15 and a >= Fraction(2) ** (e + 1):
        e += 1
    ulp = Fraction(2) ** (e - 10)                  # spacing of fp16 numbers in [2^e, 2^(e+1)); 2^-24 below 2^-14
    m, rem = divmod(a, ulp)
    m = int(m)
    if 2 * rem > ulp or (2 * rem == ulp and m % 2 == 1):
        m += 1
    if m == 0:
        return np.float16(-0.0 if sign < 0 else 0.0)      # a negative value that rounds to zero keeps its sign; 0 itself is +0
    return np.float16(float(sign * m * ulp))       # m * ulp is an fp16 number: both conversions are exact


def merge_closest_stored(codebook: np.ndarray, counts: np.ndarray, idx: np.ndarray, ncent: int):
    """merge_closest with the new centroid as it is stored: the weighted mean of Eq. 8 evaluated in exact
    rational arithmetic and rounded ONCE to fp16, ties to even.  Returns (codebook fp16 [N, 2**bits],
    merged position [N], re-numbered indices)."""
    cb = np.asarray(codebook, dtype=np.float16)
    _, merged, new_idx = merge_closest(cb, counts, idx, ncent)
    cnt = np.asarray(counts)
    out = np.zeros_like(cb)
    for n in range(cb.shape[0]):
        a = int(merged[n])
        ca, cb_ = Fraction(float(cb[n, a])), Fraction(float(cb[n, a + 1]))
        na, nb = int(cnt[n, a]), int(cnt[n, a + 1])
        new = (na * ca + nb * cb_) / (na + nb) if na + nb > 0 else (ca + cb_) / 2
        out[n, :a] = cb[n, :a]
        out[n, a] = round_to_half(new)
        out[n, a + 1:ncent - 1] = cb[n, a + 2:ncent]
    return out, merged, new_idx
