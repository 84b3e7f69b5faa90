"""Pins for the oracle of the inverted-file neighbour search (Sec. III-B, Eq. 10-11, flat second stage)."""
import numpy as np
import pytest

import oracle
from oracle import ivf
from paper_1807_11824_amd import synth


def test_all_lists_probed_is_the_exact_search():
    """tau = |C|: every point is a candidate, so Eq. (11) is the exact k-argmin (the brute-force oracle)."""
    X, _ = synth.gaussian_mixture(700, 12, 5, 4.0, 1.0, seed=2)
    C, _ = ivf.kmeans_train(X, 9, 3)
    idx, d2 = ivf.ivf_knn(X, C, 9, 15)
    eidx, ed2 = oracle.knn(X, 15)
    assert np.array_equal(idx, eidx)
    assert np.allclose(d2, ed2, rtol=1e-12, atol=0)


def test_line_example_by_hand():
    """Twenty points on a line in two groups, one centroid per group, one list probed: neighbours never
    cross to the other group; equal distances go to the lower index."""
    X = np.concatenate([np.arange(10.0), 100.0 + np.arange(10.0)]).astype(np.float32)[:, None]
    C = np.array([[4.5], [104.5]], np.float32)
    idx, d2 = ivf.ivf_knn(X, C, 1, 3)
    assert idx[0].tolist() == [1, 2, 3] and d2[0].tolist() == [1.0, 4.0, 9.0]
    assert idx[5].tolist() == [4, 6, 3] and d2[5].tolist() == [1.0, 1.0, 4.0]
    assert idx[9].tolist() == [8, 7, 6]
    assert idx[10].tolist() == [11, 12, 13]
    assert idx[19].tolist() == [18, 17, 16] and d2[19].tolist() == [1.0, 4.0, 9.0]
    # both lists probed: point 9 still has 8, 7, 6 (the other group is 91 away), with k = 9 it needs all of its group
    idx2, _ = ivf.ivf_knn(X, C, 2, 10)
    assert idx2[9].tolist() == [8, 7, 6, 5, 4, 3, 2, 1, 0, 10]
    with pytest.raises(ValueError):
        ivf.ivf_knn(X, C, 1, 10)         # nine other points in the list, ten asked for


def test_probe_order_and_ties():
    """Eq. (10) by hand: distances 1, 1, 4, 0 to four centroids -> order 3, 0, 1, 2; a copy of a centroid
    never wins against the original."""
    X = np.array([[0.0, 0.0]], np.float32)
    C = np.array([[1, 0], [0, -1], [2, 0], [0, 0]], np.float32)
    assert ivf.probes(X, C, 4)[0].tolist() == [3, 0, 1, 2]
    assert ivf.probes(X, C, 2)[0].tolist() == [3, 0]
    a, dmin = ivf.assign(np.array([[1.0, 0.1]], np.float32), np.array([[1, 0], [1, 0], [5, 5]], np.float32))
    assert a.tolist() == [0] and abs(dmin[0] - np.float64(np.float32(0.1)) ** 2) < 1e-15


def test_sq_dists_against_plain_loops():
    r = np.random.default_rng(0)
    X = r.standard_normal((7, 5)).astype(np.float32)
    C = r.standard_normal((4, 5)).astype(np.float32)
    D = ivf.sq_dists(X, C)
    for i in range(7):
        for c in range(4):
            s = 0.0
            for t in range(5):
                s += (float(X[i, t]) - float(C[c, t])) ** 2
            assert abs(D[i, c] - s) <= 1e-14 * s


def test_start_is_spread_out_by_hand():
    """Eight points on a line, three centroids, all eight in the sample: the first row, then the farthest
    from it, then the farthest from both (ties to the lower row)."""
    X = np.array([0, 1, 2, 3, 10, 11, 20, 21], np.float32)[:, None]
    assert ivf.kmeans_init(X, 3)[:, 0].tolist() == [0.0, 21.0, 10.0]     # 10 and 11 are both 10 away: the lower row
    assert ivf.kmeans_init(X, 1)[:, 0].tolist() == [0.0]
    # copies only: every distance is zero and the first sample row is taken again and again
    assert ivf.kmeans_init(np.ones((5, 2), np.float32), 3).tolist() == [[1.0, 1.0]] * 3
    # the sample: m = min(n, 8 nlist) rows floor(j n / m); with n = 100, nlist = 2 these are rows 0, 6, 12, 18, ...
    Y = np.arange(100, dtype=np.float32)[:, None]
    assert ivf.kmeans_init(Y, 2)[:, 0].tolist() == [0.0, float((15 * 100) // 16)]


def test_kmeans_separated_groups_reach_the_group_means_in_one_step():
    """Three groups far apart: the spread-out start puts one centroid into each, every point's nearest centroid
    is its own group's, and one update gives the three means."""
    r = np.random.default_rng(3)
    groups = [r.standard_normal((40, 6)) + 100.0 * g for g in range(3)]
    X = np.concatenate(groups).astype(np.float32)
    C, inertia = ivf.kmeans_train(X, 3, 2)
    want = np.stack([X[40 * g:40 * g + 40].astype(np.float64).mean(axis=0) for g in range(3)])
    order = np.argsort(C[:, 0])
    assert np.allclose(C[order], want, rtol=0, atol=1e-5)
    assert inertia[1] < inertia[0]
    # a fixed point: another pass changes nothing
    C2, _ = ivf.kmeans_train(X, 3, 5)
    assert np.array_equal(C, C2)


def test_kmeans_inertia_never_rises_and_empty_cells_stay():
    X, _ = synth.gaussian_mixture(900, 8, 4, 5.0, 1.0, seed=5)
    C, inertia = ivf.kmeans_train(X, 30, 8)
    assert all(b <= a * (1 + 1e-6) for a, b in zip(inertia, inertia[1:]))   # (centroids are rounded to float)
    # two points, each twice, four centroids: the start is (0,0,0), (1,1,1) and twice more (0,0,0); the copies
    # never win a point against the first (ties go to the lower index) and must not move
    Xd = np.concatenate([np.zeros((2, 3), np.float32), np.ones((2, 3), np.float32)])
    C, _ = ivf.kmeans_train(Xd, 4, 3)
    assert C.tolist() == [[0.0] * 3, [1.0] * 3, [0.0] * 3, [0.0] * 3]


def test_kmeans_rounds_see_only_the_sample():
    """One centroid, 1000 rows: the rounds use the 256 rows floor(i 1000 / 256); the other rows can hold anything."""
    r = np.random.default_rng(8)
    X = r.standard_normal((1000, 4)).astype(np.float32)
    rows = (np.arange(256) * 1000) // 256
    other = np.setdiff1d(np.arange(1000), rows)
    X[other] = 1e6
    C, _ = ivf.kmeans_train(X, 1, 2)
    assert np.allclose(C[0], X[rows].astype(np.float64).mean(axis=0), rtol=0, atol=1e-6)


def test_more_lists_never_hurt():
    """The candidate sets are nested in tau, so the distance to the k-th neighbour cannot grow and the recall
    cannot fall; at tau = |C| the recall is 1."""
    X, _ = synth.gaussian_mixture(1200, 10, 6, 3.0, 1.0, seed=7)
    C, _ = ivf.kmeans_train(X, 20, 5)
    eidx, _ = oracle.knn(X, 10)
    last_d, last_r = None, 0.0
    for tau in (2, 4, 8, 20):
        idx, d2 = ivf.ivf_knn(X, C, tau, 10)
        assert np.all(np.diff(d2, axis=1) >= 0)
        assert not np.any(idx == np.arange(1200)[:, None])
        if last_d is not None:
            assert np.all(d2 <= last_d)
        rec = ivf.recall(idx, eidx)
        assert rec >= last_r
        last_d, last_r = d2, rec
    assert last_r == 1.0


def test_lists_partition_the_points():
    X, _ = synth.gaussian_mixture(500, 6, 3, 3.0, 1.0, seed=1)
    C = ivf.kmeans_init(X, 11)
    lists = ivf.ivf_lists(X, C)
    allp = np.sort(np.concatenate(lists))
    assert np.array_equal(allp, np.arange(500))
    a, _ = ivf.assign(X, C)
    for c, l in enumerate(lists):
        assert np.all(a[l] == c)


# ---------------------------------------------------------------------------- product-quantised second stage
def test_pq_hand_example():
    """Eq. (8) and (11) by hand.  One list (centroid at the origin), five points in the plane, two sub-vectors of
    one coordinate each, two centroids per sub-quantiser."""
    X = np.array([[1.0, 10.0], [3.0, 10.0], [1.0, 20.0], [3.0, 20.0], [2.0, 16.0]], np.float32)
    C = np.array([[0.0, 0.0]], np.float32)
    cb = np.array([[[1.0], [3.0]], [[10.0], [20.0]]], np.float32)       # x-codebook {1, 3}, y-codebook {10, 20}
    codes, a = ivf.pq_encode(X, C, cb)
    assert a.tolist() == [0] * 5
    assert codes.tolist() == [[0, 0], [1, 0], [0, 1], [1, 1], [0, 1]]     # x = 2 is equally far from 1 and 3: lower index
    Q = ivf.pq_decode(C, cb, codes, a)
    assert Q.tolist() == [[1, 10], [3, 10], [1, 20], [3, 20], [1, 20]]
    # query 4 = (2, 16): |x - q(y)|^2 to the codes of points 0..3 = 1 + 36, 1 + 36, 1 + 16, 1 + 16
    idx, d2 = ivf.ivfpq_knn(X, C, cb, 1, 4, rows=[4])
    assert idx[0].tolist() == [2, 3, 0, 1] and d2[0].tolist() == [17.0, 17.0, 37.0, 37.0]
    # query 0 = (1, 10) sees point 4 through its code (1, 20): 100 away, behind point 1 (4) and level with point 2
    idx, d2 = ivf.ivfpq_knn(X, C, cb, 1, 4, rows=[0])
    assert idx[0].tolist() == [1, 2, 4, 3] and d2[0].tolist() == [4.0, 100.0, 100.0, 104.0]


def test_pq_with_enough_centroids_is_the_flat_search():
    """When every residual sub-vector is one of its sub-quantiser's centroids, q(y) = y and Eq. (11) compares exact
    distances: the lists are those of the flat second stage.  Lattice data (three values a coordinate), one list
    at the origin, codebooks holding all nine pairs of values."""
    X = synth.lattice(600, 6, span=3, seed=4)
    C = np.zeros((1, 6), np.float32)                       # one list at the origin: residual = the point itself
    vals = np.array([0.0, 1.0, 2.0], np.float32)
    pairs = np.array([[u, v] for u in vals for v in vals], np.float32)          # every possible sub-vector of two
    cb = np.stack([pairs, pairs, pairs])                   # m = 3 sub-vectors, 9 centroids each
    idx, d2 = ivf.ivfpq_knn(X, C, cb, 1, 12)
    fidx, fd2 = ivf.ivf_knn(X, C, 1, 12)
    assert np.array_equal(idx, fidx) and np.array_equal(d2, fd2)
    eidx, _ = oracle.knn(X, 12)
    assert np.array_equal(idx, eidx)


def test_pq_codes_are_the_nearest_reconstruction():
    """q2 takes each sub-vector to its nearest centroid, so no other code reconstructs a point better; the
    distance of Eq. (11) is the distance to the decoded point; and the trained codebooks have the stated shape."""
    X, _ = synth.gaussian_mixture(900, 8, 6, 3.0, 1.0, seed=7)
    C, _ = ivf.kmeans_train(X, 12, 4)
    cb = ivf.pq_train(X, C, 4, 16, 5)
    assert cb.shape == (4, 16, 2) and cb.dtype == np.float32
    codes, a = ivf.pq_encode(X, C, cb)
    Q = ivf.pq_decode(C, cb, codes, a)
    err = ((X.astype(np.float64) - Q) ** 2).sum(1)
    rng = np.random.default_rng(0)
    for _ in range(20):
        other = codes.copy()
        j = rng.integers(0, 4)
        other[:, j] = (other[:, j] + rng.integers(1, 16)) % 16
        worse = ((X.astype(np.float64) - ivf.pq_decode(C, cb, other, a)) ** 2).sum(1)
        assert np.all(worse >= err - 1e-12)
    # quantising the residual loses less than dropping it: the code is closer to the point than its list's centroid
    _, dcoarse = ivf.assign(X, C)
    assert err.mean() < 0.5 * dcoarse.mean()
    idx, d2 = ivf.ivfpq_knn(X, C, cb, 3, 10, rows=[5, 77, 400])
    for o, i in enumerate([5, 77, 400]):
        direct = ((X[i].astype(np.float64)[None, :] - Q[idx[o]]) ** 2).sum(1)
        assert np.allclose(d2[o], direct, rtol=1e-12, atol=1e-12)
        assert np.all(np.diff(d2[o]) >= 0) and i not in idx[o]


def test_pq_recall_grows_with_the_code():
    """A finer second stage (more centroids per sub-quantiser) finds more of the true neighbours; with tau = |C|
    the only approximation left is the code."""
    X, _ = synth.gaussian_mixture(1200, 8, 5, 4.0, 1.0, seed=9)
    C, _ = ivf.kmeans_train(X, 10, 4)
    eidx, _ = oracle.knn(X, 10)
    rows = np.arange(0, 1200, 7)
    rec = []
    for ksub in (2, 16, 128):
        cb = ivf.pq_train(X, C, 4, ksub, 6)
        idx, _ = ivf.ivfpq_knn(X, C, cb, 10, 10, rows=rows)
        rec.append(ivf.recall(idx, eidx[rows]))
    assert rec[0] < rec[1] < rec[2] and rec[2] > 0.6
