"""CPU oracle for the clustering-side steps that need no calibration data.  TEST INFRASTRUCTURE ONLY.

Plain numpy in fp64 (every fp16 input converts exactly), no blocking, no shortcuts:

* nearest-centroid assignment -- a weight belongs to the cluster whose centroid is closest.  This is
  the state the reclassification rule of Sec. 3.3 (Eq. 6) preserves: a weight changes cluster once
  it crosses half the distance to a neighbouring centroid, i.e. once that neighbour is the nearer
  one.  A weight exactly half way between two centroids has crossed nothing and stays with the lower.
* cluster sizes n_i (the "number of points in each cluster" of Sec. 3.5).
* merge of the two closest centroids into their count-weighted mean (Sec. 3.5, Eq. 8).  The printed
  formula pairs each centroid with the OTHER cluster's count; the sentence above it defines the new
  centroid as the average weighted by the clusters' own sizes, which is also the only choice that
  keeps sum_i n_i C_i (the clustered weights' total) unchanged.  That reading is taken here.

Codebooks are per output row, [N, 2**bits], of which the first `ncent` entries are in use and
strictly ascending.
"""
from __future__ import annotations

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
