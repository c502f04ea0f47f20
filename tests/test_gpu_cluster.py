"""GPU: clustering-side kernels (nearest-centroid assignment, cluster sizes, Eq. 8 merge) against the
numpy oracle.  Everything is compared bit for bit: indices, sizes, merged position, and the merged
centroid (the exact weighted mean rounded once to fp16, ties to even)."""
import numpy as np
import pytest

import oracle
import synth
import paper_2506_12038_amd as lcd
from gpu_common import to_dev

pytestmark = pytest.mark.gpu


def _row_codebooks(N, ncent, bits, seed, scale=0.03):
    """Strictly ascending distinct fp16 centroids per row, zeros in the unused slots."""
    rng = np.random.default_rng(seed)
    cb = np.zeros((N, 1 << bits), dtype=np.float16)
    for n in range(N):
        vals = np.unique((rng.standard_normal(6 * ncent) * scale).astype(np.float16))
        cb[n, :ncent] = np.sort(rng.choice(vals, size=ncent, replace=False))
    return cb


def _weights(N, K, cb, ncent, seed, scale=0.04):
    """Gaussian weights with planted hard cases: exact centroids, exact midpoints where representable,
    their fp16 neighbours, zeros of both signs, huge values, a NaN."""
    rng = np.random.default_rng(seed)
    w = (rng.standard_normal((N, K)) * scale).astype(np.float16)
    c64 = cb.astype(np.float64)
    for n in range(N):
        k = 0
        for i in range(ncent):
            w[n, k] = cb[n, i]; k += 1
        for i in range(ncent - 1):
            m = np.float16((c64[n, i] + c64[n, i + 1]) / 2)
            for v in (m, np.nextafter(m, np.float16(np.inf)), np.nextafter(m, np.float16(-np.inf))):
                w[n, k] = v; k += 1
        w[n, k:k + 5] = np.array([0.0, -0.0, 65504.0, -65504.0, 6e-8], dtype=np.float16)
    w[0, K - 1] = np.float16(np.nan)
    return w


@pytest.mark.parametrize("bits,ncent", [(2, 4), (2, 3), (3, 8), (3, 5), (4, 16), (4, 10), (3, 1)])
@pytest.mark.parametrize("shape", [(16, 256), (48, 2304), (32, 4352)])
def test_assign_indices_is_the_nearest_centroid(bits, ncent, shape):
    N, K = shape
    cb = _row_codebooks(N, ncent, bits, 7 * bits + ncent + N)
    w = _weights(N, K, cb, ncent, K + ncent)
    got = lcd.lcd_assign_indices(to_dev(w), to_dev(cb), ncent, bits).cpu().numpy()
    expect = oracle.assign_nearest(w, cb, ncent)
    expect[0, K - 1] = 0                      # NaN: no comparison holds, the kernel stays at centroid 0
    assert np.array_equal(got, expect)


def test_assign_then_pack_then_product_reproduces_the_clustered_weights():
    # dense weights -> indices on the GPU -> the decode path; equals the oracle product on the
    # oracle's own assignment of the same weights
    bits, N, K = 3, 64, 1024
    layer = synth.make_layer(1, 0, N, K, bits, 1, seed_offset=77)
    cb = _row_codebooks(N, 8, bits, 5)
    w = (np.random.default_rng(3).standard_normal((N, K)) * 0.04).astype(np.float16)
    idx_dev = lcd.lcd_assign_indices(to_dev(w), to_dev(cb), 8, bits)
    idx = oracle.assign_nearest(w, cb, 8)
    assert np.array_equal(idx_dev.cpu().numpy(), idx)
    packed = lcd.lcd_pack_indices(idx_dev, bits)
    lut = lcd.lcd_build_lut(to_dev(cb), bits)
    y = lcd.lcd_lut_gemv(packed, lut, to_dev(layer["x"]), to_dev(layer["s"]), N, bits).cpu().numpy()
    Y = oracle.lut_matmul(cb, idx, layer["x"], layer["s"], bits)
    assert oracle.parity_errors(y, Y)["max_rel_floored"] <= 2e-3


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("shape", [(16, 256), (48, 2304), (64, 11008)])
def test_cluster_counts_are_exact(bits, shape):
    N, K = shape
    rng = np.random.default_rng(N + K + bits)
    idx = rng.integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    idx[1, :] = (1 << bits) - 1               # one cluster holds a whole row
    got = lcd.lcd_cluster_counts(to_dev(idx), bits).cpu().numpy().view(np.uint32)
    assert np.array_equal(got, oracle.cluster_counts(idx, 1 << bits))


@pytest.mark.parametrize("bits,ncent", [(2, 4), (2, 2), (3, 8), (3, 6), (4, 16), (4, 11)])
def test_merge_closest_matches_the_oracle(bits, ncent):
    N, K = 48, 1280
    cb = _row_codebooks(N, ncent, bits, 31 * bits + ncent)
    if ncent >= 4:
        cb[3, :ncent] = np.arange(ncent, dtype=np.float16) * 0.25 - 1      # all gaps equal: the lowest pair
    w = _weights(N, K, cb, ncent, 11)
    w[0, K - 1] = 0
    idx = oracle.assign_nearest(w, cb, ncent)
    idx[5, :] = np.where(idx[5] <= 1, 2 % ncent, idx[5])                   # clusters 0 and 1 of row 5 empty
    counts = oracle.cluster_counts(idx, 1 << bits)
    cb_ref, merged_ref, idx_ref = oracle.merge_closest_stored(cb, counts, idx, ncent)
    counts_dev = lcd.lcd_cluster_counts(to_dev(idx), bits)
    cb_out, idx_out, merged = lcd.lcd_merge_closest(to_dev(cb), counts_dev, to_dev(idx), ncent, bits)
    assert np.array_equal(merged.cpu().numpy(), merged_ref)
    assert np.array_equal(idx_out.cpu().numpy(), idx_ref)
    # bit for bit: untouched centroids copied, the merged one the exact weighted mean rounded once to fp16
    assert np.array_equal(cb_out.cpu().numpy().view(np.uint16), cb_ref.view(np.uint16))
    # in place re-numbering gives the same indices
    idx_dev = to_dev(idx)
    lcd.lcd_merge_closest(to_dev(cb), counts_dev, idx_dev, ncent, bits, idx_out=idx_dev)
    assert np.array_equal(idx_dev.cpu().numpy(), idx_ref)


def test_full_size_layer_assign_counts_merge_sampled():
    # LLaMA-7B gate/up shape, 3-bit container: the oracle evaluates a seeded sample of rows
    import torch
    bits, ncent, N, K = 3, 8, 11008, 4096
    cb = _row_codebooks(N, ncent, bits, 99)
    g = torch.Generator(device="cuda"); g.manual_seed(5)
    w_dev = (torch.randn((N, K), device="cuda", generator=g) * 0.04).to(torch.float16)
    idx_dev = lcd.lcd_assign_indices(w_dev, to_dev(cb), ncent, bits)
    counts_dev = lcd.lcd_cluster_counts(idx_dev, bits)
    cb_out, idx_out, merged = lcd.lcd_merge_closest(to_dev(cb), counts_dev, idx_dev, ncent, bits)
    torch.cuda.synchronize()
    rs = np.sort(np.random.default_rng(1).choice(N, size=96, replace=False)); rs[0] = 0; rs[-1] = N - 1
    w = w_dev[torch.from_numpy(rs).cuda()].cpu().numpy()
    idx = oracle.assign_nearest(w, cb[rs], ncent)
    assert np.array_equal(idx_dev.cpu().numpy()[rs], idx)
    counts = oracle.cluster_counts(idx, 1 << bits)
    assert np.array_equal(counts_dev.cpu().numpy().view(np.uint32)[rs], counts)
    assert int(counts_dev.sum().item()) == N * K
    cb_ref, merged_ref, idx_ref = oracle.merge_closest_stored(cb[rs], counts, idx, ncent)
    assert np.array_equal(merged.cpu().numpy()[rs], merged_ref)
    assert np.array_equal(idx_out.cpu().numpy()[rs], idx_ref)
    assert np.array_equal(cb_out.cpu().numpy()[rs].view(np.uint16), cb_ref.view(np.uint16))


def test_merged_centroid_is_correctly_rounded_on_hard_cases():
    # one (pair of centroids, pair of cluster sizes) per row, two centroids in a 2-bit container: exact
    # ties between neighbouring fp16 numbers, means a hair above or below a tie (where rounding through
    # binary32 first goes the wrong way), subnormal and mixed-sign pairs, sizes up to 2^32 - 1, empty clusters
    rng = np.random.default_rng(23)
    N, K = 4096, 256
    bitsA = rng.integers(0, 0x7bff, size=N).astype(np.uint16)
    kind = rng.integers(0, 4, size=N)
    step = np.where(kind == 0, 1, rng.integers(1, 0x2000, size=N)).astype(np.int64)         # kind 0: adjacent numbers
    bitsB = np.minimum(bitsA.astype(np.int64) + step, 0x7bff).astype(np.uint16)
    lo = bitsA.view(np.float16).astype(np.float64); hi = bitsB.view(np.float16).astype(np.float64)
    sign = rng.integers(0, 3, size=N)                                                      # both positive / both negative / mixed
    lo, hi = np.where(sign == 1, -hi, np.where(sign == 2, -lo, lo)), np.where(sign == 1, -lo, hi)
    keep = hi > lo
    lo, hi = np.where(keep, lo, 0.0), np.where(keep, hi, 1.0)
    cb = np.zeros((N, 4), dtype=np.float16); cb[:, 0] = lo; cb[:, 1] = hi
    big = rng.integers(1, 2 ** 32 - 1, size=N, dtype=np.uint64)
    na = np.where(kind == 3, rng.integers(0, 5, size=N).astype(np.uint64), big)
    delta = rng.integers(-2, 3, size=N)
    nb = np.where(kind <= 1, np.clip(na.astype(np.int64) + delta, 0, 2 ** 32 - 1).astype(np.uint64),   # nearly equal sizes: near the midpoint
                  rng.integers(0, 2 ** 32 - 1, size=N, dtype=np.uint64))
    counts = np.zeros((N, 4), dtype=np.uint32); counts[:, 0] = na; counts[:, 1] = nb
    counts[:8, :2] = 0                                                                      # both clusters empty
    idx = rng.integers(0, 2, size=(N, K), dtype=np.uint8)
    cb_ref, merged_ref, idx_ref = oracle.merge_closest_stored(cb, counts, idx, 2)
    cb_out, idx_out, merged = lcd.lcd_merge_closest(to_dev(cb), to_dev(counts.view(np.int32)), to_dev(idx), 2, 2)
    got = cb_out.cpu().numpy()
    assert np.array_equal(got.view(np.uint16), cb_ref.view(np.uint16))
    assert np.array_equal(merged.cpu().numpy(), merged_ref) and np.array_equal(idx_out.cpu().numpy(), idx_ref)
    # the cases bite: rounding the fp64 mean through binary32 gives another fp16 number on some of them
    mean64 = np.where((na + nb) > 0, (na * lo + nb * hi) / np.maximum(na + nb, 1).astype(np.float64), 0.5 * (lo + hi))
    twice = mean64.astype(np.float32).astype(np.float16)
    assert np.count_nonzero(twice.view(np.uint16)[8:] != cb_ref[8:, 0].view(np.uint16)) >= 5
