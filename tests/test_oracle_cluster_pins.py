"""Pins for the clustering-side oracle (nearest-centroid assignment, cluster sizes, Eq. 8 merge):
hand-worked values, exact rational brute force, the half-gap rule of Eq. 6 written out, and the
invariants a plausible mistake would break."""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _case(N, K, ncent, slots, seed):
    rng = np.random.default_rng(seed)
    cb = np.zeros((N, slots), dtype=np.float16)
    for n in range(N):
        vals = np.unique((rng.standard_normal(4 * ncent) * 0.05).astype(np.float16))
        cb[n, :ncent] = np.sort(rng.choice(vals, size=ncent, replace=False))
    w = (rng.standard_normal((N, K)) * 0.06).astype(np.float16)
    return w, cb


def test_hand_worked_assignment():
    # centroids -1, 0, 0.25, 2: boundaries at -0.5, 0.125, 1.125; a weight ON a boundary stays low
    C = np.array([[-1, 0, 0.25, 2]], dtype=np.float16)
    w = np.array([[-3, -0.6, -0.5, -0.499, 0.1, 0.125, 0.13, 1.125, 1.2, 5]], dtype=np.float16)
    assert oracle.assign_nearest(w, C, 4).tolist() == [[0, 0, 0, 1, 1, 1, 2, 2, 3, 3]]
    # only the first ncent entries are in use
    assert oracle.assign_nearest(w, C, 2).tolist() == [[0, 0, 0, 1, 1, 1, 1, 1, 1, 1]]


@pytest.mark.parametrize("ncent,slots", [(4, 4), (5, 8), (8, 8), (10, 16), (16, 16)])
def test_assignment_exact_rational_brute_force(ncent, slots):
    w, cb = _case(3, 40, ncent, slots, 50 + ncent)
    got = oracle.assign_nearest(w, cb, ncent)
    for n in range(3):
        cs = [Fraction(float(c)) for c in cb[n, :ncent]]
        for k in range(40):
            x = Fraction(float(w[n, k]))
            d = [abs(x - c) for c in cs]
            assert got[n, k] == d.index(min(d))       # list.index: the first (lowest) minimum


def test_centroids_map_to_themselves_and_midpoints_stay_low():
    _, cb = _case(4, 8, 6, 8, 3)
    assert np.array_equal(oracle.assign_nearest(cb[:, :6], cb, 6), np.tile(np.arange(6, dtype=np.uint8), (4, 1)))
    # exact midpoints, representable because both ends are small multiples of 2^-10
    C = np.array([[-0.5, -0.25, 0.125, 0.375, 1.0]], dtype=np.float16)
    mid = ((C[:, :-1].astype(np.float64) + C[:, 1:].astype(np.float64)) / 2).astype(np.float16)
    assert np.array_equal(mid.astype(np.float64) * 2, C[:, :-1].astype(np.float64) + C[:, 1:].astype(np.float64))
    assert oracle.assign_nearest(mid, C, 5).tolist() == [[0, 1, 2, 3]]
    up = np.nextafter(mid, np.float16(np.inf))
    assert oracle.assign_nearest(up, C, 5).tolist() == [[1, 2, 3, 4]]


def test_assignment_is_monotone_and_minimises_the_clustering_error():
    w, cb = _case(5, 300, 7, 8, 9)
    idx = oracle.assign_nearest(w, cb, 7)
    order = np.argsort(w.astype(np.float64), axis=1, kind="stable")
    assert np.all(np.diff(np.take_along_axis(idx, order, axis=1).astype(int), axis=1) >= 0)
    c64, w64 = cb.astype(np.float64), w.astype(np.float64)
    err = (w64 - np.take_along_axis(c64, idx.astype(np.int64), axis=1)) ** 2
    for shift in (-1, 1):
        other = np.clip(idx.astype(int) + shift, 0, 6)
        assert np.all(err <= (w64 - np.take_along_axis(c64, other, axis=1)) ** 2)


def test_half_gap_rule_of_eq6_reaches_the_same_clusters():
    # weights sitting on their centroids receive an update dw; Eq. 6: leave the cluster to the left
    # when the move exceeds half the gap to the left neighbour, to the right likewise (edge
    # centroids have one neighbour).  While a move crosses at most one boundary this is the
    # nearest-centroid assignment of the moved weight.
    rng = np.random.default_rng(4)
    C = np.array([[-0.75, -0.25, 0.0, 0.5, 1.0, 1.25]], dtype=np.float16)
    c = C[0].astype(np.float64)
    start = rng.integers(0, 6, size=400)
    # odd multiples of 2^-7: never exactly half a gap (those are multiples of 2^-3), and c + dw is
    # exact in fp16.  (On an exact boundary the two rules differ by construction: Eq. 6 keeps the
    # cluster the weight came from, the stateless assignment takes the lower centroid.)
    dw = ((2 * rng.integers(-13, 13, size=400) + 1) / 128.0).astype(np.float16)
    moved = (c[start] + dw.astype(np.float64)).astype(np.float16)
    assert np.array_equal(moved.astype(np.float64), c[start] + dw.astype(np.float64))   # the sum is exact here
    expect = []
    for i, d in zip(start, dw.astype(np.float64)):
        d_left = (c[i] - c[i - 1]) / 2 if i > 0 else None
        d_right = (c[i + 1] - c[i]) / 2 if i < 5 else None
        if d_left is not None and d < -d_left:
            expect.append(i - 1)
        elif d_right is not None and d > d_right:
            expect.append(i + 1)
        else:
            expect.append(i)
    assert oracle.assign_nearest(moved[None, :], C, 6)[0].tolist() == expect


def test_counts_against_a_plain_loop():
    rng = np.random.default_rng(8)
    idx = rng.integers(0, 10, size=(6, 257), dtype=np.uint8)
    got = oracle.cluster_counts(idx, 16)
    for n in range(6):
        for i in range(16):
            assert got[n, i] == sum(1 for v in idx[n] if v == i)


def test_hand_worked_merge():
    # gaps 1, 0.25, 1.75: (0, 0.25) merge; sizes 1 and 3 -> (1*0 + 3*0.25)/4 = 0.1875, nearer the larger cluster
    C = np.array([[-1, 0, 0.25, 2]], dtype=np.float16)
    counts = np.array([[3, 1, 3, 5]], dtype=np.uint32)
    idx = np.array([[0, 1, 2, 3, 2, 3]], dtype=np.uint8)
    cb, merged, new_idx = oracle.merge_closest(C, counts, idx, 4)
    assert cb.tolist() == [[-1.0, 0.1875, 2.0, 0.0]]
    assert merged.tolist() == [1]
    assert new_idx.tolist() == [[0, 1, 1, 2, 1, 2]]
    # equal gaps: the lowest pair; empty clusters: the plain mean
    C2 = np.array([[0, 1, 2, 4]], dtype=np.float16)
    cb2, merged2, _ = oracle.merge_closest(C2, np.array([[0, 0, 7, 7]]), idx, 4)
    assert merged2.tolist() == [0] and cb2.tolist() == [[0.5, 2.0, 4.0, 0.0]]


@pytest.mark.parametrize("ncent,slots", [(3, 4), (6, 8), (8, 8), (13, 16)])
def test_merge_conserves_the_clustered_weights_total(ncent, slots):
    w, cb = _case(7, 500, ncent, slots, 20 + ncent)
    idx = oracle.assign_nearest(w, cb, ncent)
    counts = oracle.cluster_counts(idx, slots)
    new_cb, merged, new_idx = oracle.merge_closest(cb, counts, idx, ncent)
    new_counts = oracle.cluster_counts(new_idx, slots)
    c64 = cb.astype(np.float64)
    assert np.array_equal(new_counts.sum(axis=1), counts.sum(axis=1))
    assert np.all(new_counts[:, ncent - 1:] == 0)
    # sum_i n_i C_i is unchanged (the printed form of Eq. 8, with the counts crossed, changes it)
    before = (counts[:, :ncent] * c64[:, :ncent]).sum(axis=1)
    after = (new_counts[:, :ncent - 1] * new_cb[:, :ncent - 1]).sum(axis=1)
    assert np.allclose(before, after, rtol=0, atol=1e-9)
    crossed = before.copy()
    for n in range(7):
        a = merged[n]; na, nb = float(counts[n, a]), float(counts[n, a + 1])
        if na + nb > 0 and na != nb:
            wrong = (nb * c64[n, a] + na * c64[n, a + 1]) / (na + nb)
            crossed[n] += (na + nb) * (wrong - new_cb[n, a])
    assert not np.allclose(before, crossed, rtol=0, atol=1e-9)
    # still strictly ascending, and the merged pair was the closest one
    assert np.all(np.diff(new_cb[:, :ncent - 1], axis=1) > 0)
    gaps = np.diff(c64[:, :ncent], axis=1)
    assert np.array_equal(merged, np.argmin(gaps, axis=1))
    # dequantised weights change only inside the merged pair
    old_vals = np.take_along_axis(c64, idx.astype(np.int64), axis=1)
    new_vals = np.take_along_axis(new_cb, new_idx.astype(np.int64), axis=1)
    untouched = (idx != merged[:, None]) & (idx != merged[:, None] + 1)
    assert np.array_equal(old_vals[untouched], new_vals[untouched])


def test_rounding_to_fp16_against_the_format_and_a_library_conversion():
    from fractions import Fraction
    # hand-worked: fp16 numbers near 1 are 2^-10 apart
    one, u = Fraction(1), Fraction(1, 1024)
    assert oracle.round_to_half(one + u / 2) == np.float16(1.0)                      # tie: mantissa 1024 is even
    assert oracle.round_to_half(one + 3 * u / 2) == np.float16(1.0 + 2.0 ** -9)      # tie: up to the even 1026
    assert oracle.round_to_half(one + u / 2 + Fraction(1, 10 ** 12)) == np.float16(1.0 + 2.0 ** -10)   # just above a tie
    assert oracle.round_to_half(-(one + u / 2 + Fraction(1, 10 ** 12))) == np.float16(-1.0 - 2.0 ** -10)
    assert oracle.round_to_half(Fraction(2) - u / 4) == np.float16(2.0)               # rounds up into the next binade
    assert oracle.round_to_half(Fraction(3, 2 ** 25)) == np.float16(2.0 ** -23)       # subnormal tie 1.5 -> 2
    assert oracle.round_to_half(Fraction(1, 2 ** 25)) == np.float16(0.0)              # subnormal tie 0.5 -> 0
    assert oracle.round_to_half(Fraction(1, 2 ** 14) - Fraction(1, 2 ** 26)) == np.float16(2.0 ** -14)   # largest subnormal + 3/4
    assert oracle.round_to_half(Fraction(65504)) == np.float16(65504.0)
    with pytest.raises(ValueError):
        oracle.round_to_half(Fraction(65505))
    # numpy's float64 -> float16 conversion rounds once, to nearest even: it must agree on every value that
    # a double holds exactly (the double is then the rational itself)
    rng = np.random.default_rng(17)
    vals = np.concatenate([rng.standard_normal(3000) * 0.05, rng.standard_normal(500) * 1e-6,
                           rng.standard_normal(500) * 100.0,
                           # exact ties and their neighbours: midpoints of adjacent fp16 numbers, +- one double ulp
                           *[[m, np.nextafter(m, np.inf), np.nextafter(m, -np.inf)]
                             for h in rng.integers(1, 0x7bff, size=300)
                             for m in [(float(np.array([h], dtype=np.uint16).view(np.float16)[0]) +
                                        float(np.array([h + 1], dtype=np.uint16).view(np.float16)[0])) / 2]]])
    for v in vals:
        assert oracle.round_to_half(Fraction(float(v))).view(np.uint16) == np.float64(v).astype(np.float16).view(np.uint16), v


def test_stored_merge_rounds_the_exact_mean_once():
    from fractions import Fraction
    # hand-worked: centroids 1 and 1 + 2^-10 (adjacent fp16 numbers), gap smallest
    a, b = 1.0, 1.0 + 2.0 ** -10
    C = np.array([[-1.0, a, b, 4.0]], dtype=np.float16)
    idx = np.array([[0, 1, 2, 3]], dtype=np.uint8)
    # equal sizes: the mean is the midpoint, a tie -> the even neighbour 1.0
    cb, merged, new_idx = oracle.merge_closest_stored(C, np.array([[1, 5, 5, 1]], dtype=np.uint32), idx, 4)
    assert merged.tolist() == [1] and cb.tolist() == [[-1.0, 1.0, 4.0, 0.0]] and new_idx.tolist() == [[0, 1, 1, 2]]
    # sizes 1000000 and 1000001: the mean is above the midpoint by 2.4e-10 -- less than half a binary32
    # step, so rounding to binary32 first would land ON the midpoint and then go to the even 1.0;
    # rounded once it is the upper neighbour
    cb, _, _ = oracle.merge_closest_stored(C, np.array([[1, 1000000, 1000001, 1]], dtype=np.uint32), idx, 4)
    assert cb[0, 1] == np.float16(b)
    assert np.float16(np.float32((1000000 * a + 1000001 * b) / 2000001)) == np.float16(a)      # what double rounding gives
    cb, _, _ = oracle.merge_closest_stored(C, np.array([[1, 1000001, 1000000, 1]], dtype=np.uint32), idx, 4)
    assert cb[0, 1] == np.float16(a)
    # both clusters empty: the plain mean; untouched centroids are copied, the tail is zero
    cb, _, _ = oracle.merge_closest_stored(np.array([[0.5, 0.75, 2.0, 4.0]], dtype=np.float16), np.array([[0, 0, 3, 3]]), idx, 4)
    assert cb.tolist() == [[0.625, 2.0, 4.0, 0.0]]
    # against merge_closest (the unrounded fp64 mean): same decisions, value within half an fp16 step
    w, cbk = _case(9, 300, 6, 8, 77)
    ix = oracle.assign_nearest(w, cbk, 6)
    counts = oracle.cluster_counts(ix, 8)
    ref, merged_ref, idx_ref = oracle.merge_closest(cbk, counts, ix, 6)
    got, merged, new_idx = oracle.merge_closest_stored(cbk, counts, ix, 6)
    assert np.array_equal(merged, merged_ref) and np.array_equal(new_idx, idx_ref) and got.dtype == np.float16
    up = np.nextafter(got, np.float16(np.inf)).astype(np.float64)
    down = np.nextafter(got, np.float16(-np.inf)).astype(np.float64)
    g64 = got.astype(np.float64)
    assert np.all(ref <= (g64 + up) / 2) and np.all(ref >= (g64 + down) / 2)
    # exact rational check of one row, written out
    n = 4
    a_ = int(merged[n]); na, nb = int(counts[n, a_]), int(counts[n, a_ + 1])
    exact = (na * Fraction(float(cbk[n, a_])) + nb * Fraction(float(cbk[n, a_ + 1]))) / (na + nb)
    assert abs(Fraction(float(got[n, a_])) - exact) <= min(Fraction(float(up[n, a_])) - Fraction(float(got[n, a_])),
                                                           Fraction(float(got[n, a_])) - Fraction(float(down[n, a_]))) / 2
