"""CPU oracle for the approximate neighbour search of Sec. III-B (test infrastructure only).

Inverted-file search: the coarse quantiser q1 is the nearest of |C| centroids trained by k-means
(the paper takes |C| = sqrt(N)); a query looks at the tau lists whose centroids are nearest to it
(Eq. 10) and keeps the k nearest of the points stored there (Eq. 11).  Two second stages:
  flat      q(y) = y: list entries are compared by their exact squared distance (ivf_knn);
  product   q(y) = q1(y) + q2(y - q1(y)) (Eq. 8) with q2 a product quantiser, as Sec. III-B names it:
            the residual is cut into m sub-vectors and each is replaced by the nearest of ksub
            centroids of its own sub-quantiser, trained by k-means on residual sub-vectors; Eq. (11)
            then compares the query with the code's reconstruction (pq_train, pq_encode, ivfpq_knn).
Everything below is the definition written out in numpy, in double precision, ties broken towards
the lower index.  Nothing here is shared with the GPU code.
"""
import numpy as np

__all__ = ["kmeans_init", "sq_dists", "assign", "kmeans_train", "probes", "ivf_lists", "ivf_knn", "recall",
           "residuals", "pq_train", "pq_encode", "pq_decode", "ivfpq_knn"]


def kmeans_init(X, nlist):
    """Starting centroids, spread out: from the sample of m = min(n, 8 nlist) rows floor(j n / m) take the
    first, then nlist - 1 times the sample row farthest (squared distance in double, lowest j among equals)
    from the ones taken so far."""
    X = np.asarray(X, np.float32)
    n = X.shape[0]
    m = min(n, 8 * nlist)
    rows = (np.arange(m, dtype=np.int64) * n) // m
    S = X[rows].astype(np.float64)
    chosen = [0]
    diff = S - S[0]
    mind = np.einsum("md,md->m", diff, diff)
    for _ in range(1, nlist):
        j = int(np.argmax(mind))            # first maximum = lowest j
        chosen.append(j)
        diff = S - S[j]
        mind = np.minimum(mind, np.einsum("md,md->m", diff, diff))
    return X[rows[chosen]].copy()


def sq_dists(Xq, C):
    """|x - c|^2 for every row of Xq against every row of C, in double."""
    Xq = np.asarray(Xq, np.float64)
    C = np.asarray(C, np.float64)
    out = np.empty((Xq.shape[0], C.shape[0]), np.float64)
    step = max(1, (1 << 24) // max(1, C.shape[0] * Xq.shape[1]))
    for a in range(0, Xq.shape[0], step):
        diff = Xq[a:a + step, None, :] - C[None, :, :]
        out[a:a + step] = np.einsum("qcd,qcd->qc", diff, diff)
    return out


def assign(X, C):
    """q1: index of the nearest centroid (lowest index among equals) and the squared distance to it."""
    D = sq_dists(X, C)
    a = np.argmin(D, axis=1)            # first minimum = lowest index
    return a.astype(np.int32), D[np.arange(D.shape[0]), a]


def kmeans_train(X, nlist, iters):
    """Lloyd's algorithm from kmeans_init (which see) on the sample of min(n, 256 nlist) rows floor(i n / m):
    assign every sample point to its nearest centroid, move every centroid to the mean of its points (a
    centroid without points stays where it is).  Centroids are kept as float between the iterations.
    Returns (centroids float32, inertia of the sample before each update)."""
    X = np.asarray(X, np.float32)
    C = kmeans_init(X, nlist)
    n = X.shape[0]
    m = min(n, 256 * nlist)
    X = X[(np.arange(m, dtype=np.int64) * n) // m]
    Xd = X.astype(np.float64)
    inertia = []
    for _ in range(iters):
        a, dmin = assign(X, C)
        inertia.append(float(dmin.sum()))
        for c in range(nlist):
            members = Xd[a == c]
            if members.shape[0] > 0:
                C[c] = members.mean(axis=0).astype(np.float32)
    return C, inertia


def probes(X, C, tau):
    """Eq. (10): for every row of X the tau nearest centroids, ordered by (distance, index)."""
    D = sq_dists(X, C)
    ids = np.broadcast_to(np.arange(C.shape[0]), D.shape)
    out = np.empty((X.shape[0], tau), np.int32)
    for i in range(X.shape[0]):
        out[i] = np.lexsort((ids[i], D[i]))[:tau]
    return out


def ivf_lists(X, C):
    """The inverted file: for every centroid the indices (ascending) of the points whose q1 it is."""
    a, _ = assign(X, C)
    return [np.flatnonzero(a == c).astype(np.int32) for c in range(C.shape[0])]


def ivf_knn(X, C, tau, k, rows=None):
    """Eq. (11) with a flat second stage: the k nearest (exact squared distance in double, then index)
    among the points of the tau probed lists, the query itself left out; for the queries `rows` (all).
    Returns (idx int32 [len(rows), k], d2 float64 [len(rows), k]); raises if a query sees fewer than k points."""
    X = np.asarray(X, np.float32)
    n = X.shape[0]
    Xd = X.astype(np.float64)
    lists = ivf_lists(X, C)
    rows = np.arange(n) if rows is None else np.asarray(rows)
    pr = probes(X[rows], C, tau)
    idx = np.empty((rows.shape[0], k), np.int32)
    d2 = np.empty((rows.shape[0], k), np.float64)
    for o, i in enumerate(rows):
        cand = np.concatenate([lists[c] for c in pr[o]])
        cand = cand[cand != i]
        if cand.shape[0] < k:
            raise ValueError(f"row {i}: only {cand.shape[0]} candidates in its {tau} lists, need {k}")
        diff = Xd[cand] - Xd[i]
        dd = np.einsum("cd,cd->c", diff, diff)
        order = np.lexsort((cand, dd))[:k]
        idx[o] = cand[order]
        d2[o] = dd[order]
    return idx, d2


def recall(idx, idx_exact):
    """Fraction of the exact neighbours that the approximate lists contain (recall at k)."""
    hit = 0
    for a, b in zip(idx, idx_exact):
        hit += np.intersect1d(a, b).shape[0]
    return hit / idx_exact.size


# ---------------------------------------------------------------------------- product-quantised second stage (Eq. 8, 11)
def residuals(X, C, a=None):
    """y - q1(y) for every row, one float subtraction per coordinate (a: the rows' lists, computed if not given)."""
    X = np.asarray(X, np.float32)
    C = np.asarray(C, np.float32)
    if a is None:
        a, _ = assign(X, C)
    return (X - C[a]).astype(np.float32), np.asarray(a, np.int32)


def pq_train(X, C, m, ksub, iters):
    """Codebooks of q2: sub-quantiser j is ksub centroids trained by kmeans_train (which see: spread-out start,
    `iters` Lloyd rounds on evenly spaced rows) on the j-th sub-vectors (coordinates j D/m .. (j+1) D/m - 1) of the
    residuals of all rows.  Returns float32 [m, ksub, D/m]."""
    R, _ = residuals(X, C)
    d = R.shape[1]
    if d % m != 0:
        raise ValueError("the dimension must be a multiple of the number of sub-vectors")
    ds = d // m
    cb = np.empty((m, ksub, ds), np.float32)
    for j in range(m):
        cb[j], _ = kmeans_train(np.ascontiguousarray(R[:, j * ds:(j + 1) * ds]), ksub, iters)
    return cb


def pq_encode(X, C, cb):
    """Code of every row: for each sub-vector of its residual the index of the nearest centroid of that
    sub-quantiser (squared distance in double, lowest index among equals).  Returns (codes uint8/int32 [n, m], lists)."""
    R, a = residuals(X, C)
    m, ksub, ds = cb.shape
    codes = np.empty((R.shape[0], m), np.int32)
    for j in range(m):
        codes[:, j], _ = assign(np.ascontiguousarray(R[:, j * ds:(j + 1) * ds]), cb[j])
    return codes, a


def pq_decode(C, cb, codes, a):
    """q(y) = q1(y) + q2(y - q1(y)) of Eq. (8), in double: the list's centroid plus the sub-quantisers' centroids."""
    m, ksub, ds = cb.shape
    out = np.asarray(C, np.float64)[a].copy()
    for j in range(m):
        out[:, j * ds:(j + 1) * ds] += np.asarray(cb[j], np.float64)[codes[:, j]]
    return out


def ivfpq_knn(X, C, cb, tau, k, rows=None):
    """Eq. (11) with the product-quantised second stage: among the points of the tau probed lists (the query itself
    left out) the k smallest |x - q(y)|^2, then index.  The distance is formed as the method does it, from the
    query's residual to the candidate's list: sum over the sub-vectors j, in order, of
    sum_t ((x_t - c_t) - cb[j][code_j][t])^2, every operation in double, each inner sum accumulated coordinate by
    coordinate (a product and an addition, two roundings).  Returns (idx int32, approximate d2 float64)."""
    X = np.asarray(X, np.float32)
    n, d = X.shape
    m, ksub, ds = cb.shape
    Xd = X.astype(np.float64)
    Cd = np.asarray(C, np.float64)
    cbd = np.asarray(cb, np.float64)
    codes, a = pq_encode(X, C, cb)
    lists = [np.flatnonzero(a == c).astype(np.int32) for c in range(C.shape[0])]
    rows = np.arange(n) if rows is None else np.asarray(rows)
    pr = probes(X[rows], C, tau)
    idx = np.empty((rows.shape[0], k), np.int32)
    d2 = np.empty((rows.shape[0], k), np.float64)
    for o, i in enumerate(rows):
        cand = np.concatenate([lists[c] for c in pr[o]])
        cand = cand[cand != i]
        if cand.shape[0] < k:
            raise ValueError(f"row {i}: only {cand.shape[0]} candidates in its {tau} lists, need {k}")
        rq = Xd[i][None, :] - Cd[a[cand]]                  # the query's residual to each candidate's list
        total = np.zeros(cand.shape[0])
        for j in range(m):
            sub = np.zeros(cand.shape[0])
            rec = cbd[j][codes[cand, j]]
            for t in range(ds):
                df = rq[:, j * ds + t] - rec[:, t]
                sub = sub + df * df
            total = total + sub
        order = np.lexsort((cand, total))[:k]
        idx[o] = cand[order]
        d2[o] = total[order]
    return idx, d2
