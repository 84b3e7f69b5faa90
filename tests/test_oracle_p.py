"""Pins for the oracle's affinity construction: kNN, Eq. (1) calibration, symmetrisation."""
import numpy as np
import scipy.sparse as sp
from scipy.spatial import cKDTree

import oracle
from paper_1807_11824_amd import synth


def test_knn_lattice_with_ties():
    """Integer rows: all squared distances are exact integers with many ties -> order by (d2, j)."""
    X = synth.lattice(200, 6, span=3, seed=1)
    idx, d2 = oracle.knn(X, 17)
    Xi = X.astype(np.int64)
    D = ((Xi[:, None, :] - Xi[None, :, :]) ** 2).sum(-1)
    for i in range(200):
        order = sorted((int(D[i, j]), j) for j in range(200) if j != i)[:17]
        assert [j for _, j in order] == idx[i].tolist()
        assert [float(d) for d, _ in order] == d2[i].tolist()


def test_knn_against_kdtree_low_d():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((1500, 3)).astype(np.float32)
    idx, d2 = oracle.knn(X, 12)
    dd, ii = cKDTree(X.astype(np.float64)).query(X.astype(np.float64), k=13)
    assert np.array_equal(ii[:, 1:], idx)
    assert np.allclose(dd[:, 1:] ** 2, d2, rtol=1e-12)
    # rows given explicitly
    rows = np.array([7, 0, 1499, 300], np.int32)
    i2, dd2 = oracle.knn(X, 12, rows=rows)
    assert np.array_equal(i2, idx[rows]) and np.array_equal(dd2, d2[rows])


def _entropy(p):
    p = p[p > 0]
    return float(-(p * np.log(p)).sum())


def test_rows_hit_the_perplexity():
    X, _ = synth.config1(n=600, d=50, seed=2)
    idx, d2 = oracle.knn(X, 90)
    cond, beta, bad = oracle.cond_p(d2, 30.0)
    assert bad == 0
    assert np.allclose(cond.sum(1), 1.0, rtol=0, atol=1e-14)
    H = np.array([_entropy(r) for r in cond])
    assert np.abs(H - np.log(30.0)).max() <= 1e-5
    # the row really is Eq. (1) at the returned beta: p_j proportional to exp(-beta d_j)
    r = np.exp(-beta[:, None] * (d2 - d2[:, :1]))
    assert np.allclose(cond, r / r.sum(1, keepdims=True), rtol=1e-12)
    # monotone: nearer neighbours never get less weight
    assert np.all(np.diff(cond, axis=1) <= 1e-18)


def test_two_neighbour_row_closed_form():
    """k = 2: p = (1/(1+e^{-b D}), .), D = d2 - d1; the entropy target fixes p, hence beta = ln(p/(1-p))/D."""
    d2 = np.array([[1.0, 3.5]])
    target = np.log(1.5)
    lo, hi = 0.5, 1.0 - 1e-15       # larger share p of the nearer neighbour, H(p) decreasing on (1/2, 1)
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        H = -(mid * np.log(mid) + (1 - mid) * np.log(1 - mid))
        lo, hi = (mid, hi) if H > target else (lo, mid)
    p = 0.5 * (lo + hi)
    cond, beta, bad = oracle.cond_p(d2, 1.5)
    assert bad == 0
    assert abs(cond[0, 0] - p) < 1e-9
    assert abs(beta[0] - np.log(p / (1 - p)) / 2.5) < 1e-8


def test_equal_distances_terminate_and_are_counted():
    d2 = np.full((3, 8), 2.0)
    cond, beta, bad = oracle.cond_p(d2, 4.0)
    assert bad == 3
    assert np.allclose(cond, 1.0 / 8.0)
    # but perplexity == k is met at once
    cond, beta, bad = oracle.cond_p(d2, 8.0, tol=1e-9)
    assert bad == 0


def test_symmetrised_P(small_problem):
    P = small_problem["P"]
    n, k = P["idx"].shape
    rp, col, val = P["row_ptr"], P["col"], P["val"]
    M = sp.csr_matrix((val, col, rp), shape=(n, n))
    # independent construction with scipy: (C + C^T) / 2N
    Cm = sp.csr_matrix((P["cond"].ravel(), P["idx"].ravel(), np.arange(0, n * k + 1, k)), shape=(n, n))
    want = ((Cm + Cm.T) / (2.0 * n)).tocsr()
    want.eliminate_zeros()
    want.sort_indices()
    # the structure is that of the kNN graph (Sec. III-B); scipy drops entries whose value
    # underflowed to 0, so compare on the entries that are > 0
    got = M.copy()
    got.eliminate_zeros()
    assert np.array_equal(want.indptr, got.indptr) and np.array_equal(want.indices, got.indices)
    assert np.allclose(want.data, got.data, rtol=1e-15)
    G = sp.csr_matrix((np.ones(n * k), P["idx"].ravel(), np.arange(0, n * k + 1, k)), shape=(n, n))
    S = ((G + G.T) > 0).tocsr()
    S.sort_indices()
    assert np.array_equal(S.indptr, rp) and np.array_equal(S.indices, col)
    assert abs(val.sum() - 1.0) < 1e-12
    assert (M != M.T).nnz == 0                       # bitwise symmetric
    assert n * k <= len(val) <= 2 * n * k
    assert np.all(np.diff(rp) >= k)
    for i in range(n):
        c = col[rp[i]:rp[i + 1]]
        assert np.all(np.diff(c) > 0) and i not in c
    assert np.all(val >= 0)
