"""Reference packer written from the layout definition alone.  TEST INFRASTRUCTURE ONLY.

Element-wise restatement of the packed-index layout (revision 1): for every (n, k) it
computes the byte and bit the index lands in.  It shares nothing with the library's packers
(which walk tiles and build lane words).

Layout: tiles of 16 rows x 256 columns; tile (t = n // 16, c = k // 256) starts at byte
(t * (K // 256) + c) * T, T = 1024 (2 bits), 1536 (3 bits) or 2048 (4 bits).  In a tile, lane
l = 16 * ((k % 256) // 64) + n % 16; w = k % 64.
  * low two bits of the index: bits [2w+1 : 2w] of the 128-bit little-endian word at
    tile byte 16 * l;
  * third bit (3-bit only): with w = 16 d + 8 a + e, bit
    8 * ((e >> 2) + 2 * (e & 1)) + 2 d + ((e & 3) >> 1) of the 32-bit little-endian word at
    tile byte 1024 + 8 * l + 4 * a;
  * third and fourth bit (4-bit only): bits [2w+1 : 2w] of the 128-bit little-endian word at
    tile byte 1024 + 16 * l (the arrangement of the low field, once more).
"""
from __future__ import annotations

import numpy as np


def _positions(N: int, K: int, bits: int):
    n = np.arange(N, dtype=np.int64)[:, None]
    k = np.arange(K, dtype=np.int64)[None, :]
    T = {2: 1024, 3: 1536, 4: 2048}[bits]
    tile0 = ((n // 16) * (K // 256) + (k // 256)) * T
    lane = 16 * ((k % 256) // 64) + (n % 16)
    w = k % 64
    lo_bit = (tile0 + 16 * lane) * 8 + 2 * w          # absolute bit offset of the low field
    d, a, e = w // 16, (w // 8) % 2, w % 8
    if bits == 4:
        hi_bit = (tile0 + 1024 + 16 * lane) * 8 + 2 * w
    else:
        hi_bit = (tile0 + 1024 + 8 * lane + 4 * a) * 8 + 8 * ((e >> 2) + 2 * (e & 1)) + 2 * d + ((e & 3) >> 1)
    return np.broadcast_to(lo_bit, (N, K)), np.broadcast_to(hi_bit, (N, K))


def pack_ref(idx: np.ndarray, bits: int) -> np.ndarray:
    idx = np.asarray(idx, dtype=np.uint8)
    N, K = idx.shape
    assert bits in (2, 3, 4) and N % 16 == 0 and K % 256 == 0 and int(idx.max(initial=0)) < (1 << bits)
    nbytes = N * K * bits // 8
    bitmap = np.zeros(nbytes * 8, dtype=np.uint8)      # one entry per bit, little-endian in a byte
    lo_bit, hi_bit = _positions(N, K, bits)
    bitmap[lo_bit.ravel()] = (idx & 1).ravel()
    bitmap[lo_bit.ravel() + 1] = ((idx >> 1) & 1).ravel()
    if bits >= 3:
        bitmap[hi_bit.ravel()] = ((idx >> 2) & 1).ravel()
    if bits == 4:
        bitmap[hi_bit.ravel() + 1] = ((idx >> 3) & 1).ravel()
    return np.packbits(bitmap, bitorder="little")


def unpack_ref(packed: np.ndarray, N: int, K: int, bits: int) -> np.ndarray:
    bitmap = np.unpackbits(np.asarray(packed, dtype=np.uint8), bitorder="little")
    lo_bit, hi_bit = _positions(N, K, bits)
    idx = bitmap[lo_bit] | (bitmap[lo_bit + 1] << 1)
    if bits >= 3:
        idx = idx | (bitmap[hi_bit] << 2)
    if bits == 4:
        idx = idx | (bitmap[hi_bit + 1] << 3)
    return idx.astype(np.uint8)
