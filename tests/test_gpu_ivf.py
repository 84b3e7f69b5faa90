"""GPU vs oracle: the inverted-file neighbour search (Sec. III-B, Eq. 10-11), its k-means and the P built on it.

Both sides take every decision on squared distances in double precision with ties towards the lower index,
so neighbour indices must agree exactly; distances differ only by the order of the summation."""
import numpy as np
import pytest

import oracle
from oracle import ivf
from paper_1807_11824_amd import synth

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _case(name):
    r = np.random.default_rng(11)
    if name == "blobs_50d":
        X, _ = synth.gaussian_mixture(3000, 50, 4, 10.0, 1.0, seed=0)
        return X, 40, 5, 30
    if name == "two_chunks_and_tail":        # d = 130: two full chunks of 64 coordinates and two left over
        X, _ = synth.gaussian_mixture(2500, 130, 6, 3.0, 1.0, seed=1)
        return X, 50, 8, 90
    if name == "all_lists":                  # tau = nlist: the exact search
        X, _ = synth.gaussian_mixture(2000, 7, 3, 2.0, 1.0, seed=2)
        return X, 10, 10, 60
    if name == "every_row_five_times":       # ties at every distance, decided by index
        base = r.standard_normal((500, 9)).astype(np.float32)
        return np.repeat(base, 5, axis=0), 12, 4, 23
    if name == "one_point_many_times":       # thousands of candidates at distance 0: selection by index alone
        X = np.concatenate([np.tile(r.standard_normal((1, 6)).astype(np.float32), (2600, 1)),
                            r.standard_normal((400, 6)).astype(np.float32)])
        return X[r.permutation(3000)], 4, 2, 20
    if name == "k_one":
        X = r.standard_normal((700, 3)).astype(np.float32)
        return X, 26, 3, 1
    if name == "one_list_all_but_self":      # a single list and k = n - 1: every candidate is a neighbour
        X = r.standard_normal((130, 3)).astype(np.float32)
        return X, 1, 1, 129
    if name == "large_k":                    # k = 1500 of 5000 candidates: the cut lets about 3000 keys pass
        X = r.standard_normal((5000, 5)).astype(np.float32)
        return X, 7, 7, 1500
    if name == "largest_k_cut_fails":        # k = 1900 of 9000: more keys pass the cut than the buffer holds
        X = r.standard_normal((9000, 4)).astype(np.float32)
        return X, 3, 3, 1900
    # rows longer than 64 coordinates: candidates from the matrix-core tiles, exact re-rank, certificate
    if name == "long_rows_ties":             # every row five times: no certificate for anybody, decided by index
        base = r.standard_normal((400, 100)).astype(np.float32)
        return np.repeat(base, 5, axis=0), 10, 3, 23
    if name == "long_rows_one_point_many_times":   # more equal distances than the tie buffer of the exact pass holds
        X = np.concatenate([np.tile(r.standard_normal((1, 70)).astype(np.float32), (5000, 1)),
                            r.standard_normal((600, 70)).astype(np.float32)])
        return X[r.permutation(5600)], 4, 2, 20
    if name == "long_rows_long_lists":       # lists of about 3000 rows: two launches per list and rank
        X, _ = synth.gaussian_mixture(9000, 80, 3, 4.0, 1.0, seed=9)
        return X, 3, 2, 50
    if name == "long_rows_all_but_self":
        X = r.standard_normal((130, 66)).astype(np.float32)
        return X, 1, 1, 129
    if name == "long_rows_far_from_origin":  # the search works on centred rows
        X, _ = synth.gaussian_mixture(3000, 96, 5, 3.0, 1.0, seed=10)
        return X + np.float32(200.0), 30, 4, 40
    if name == "long_rows_k_one":
        X = r.standard_normal((900, 65)).astype(np.float32)
        return X, 20, 3, 1
    raise KeyError(name)


@pytest.mark.parametrize("name", ["blobs_50d", "two_chunks_and_tail", "all_lists", "every_row_five_times",
                                  "one_point_many_times", "k_one", "one_list_all_but_self", "large_k",
                                  "largest_k_cut_fails", "long_rows_ties", "long_rows_one_point_many_times",
                                  "long_rows_long_lists", "long_rows_all_but_self", "long_rows_far_from_origin",
                                  "long_rows_k_one"])
def test_ivf_knn_matches_oracle(name):
    from paper_1807_11824_amd import ivf_knn
    X, nlist, tau, k = _case(name)
    print(f"case={name} n={X.shape[0]} d={X.shape[1]} nlist={nlist} tau={tau} k={k}", flush=True)
    C, _ = ivf.kmeans_train(X, nlist, 4)
    want_idx, want_d2 = ivf.ivf_knn(X, C, tau, k)
    idx, d2 = ivf_knn(_dev(X), _dev(C), tau, k)
    idx, d2 = idx.cpu().numpy(), d2.cpu().numpy()
    assert np.array_equal(idx, want_idx)
    assert np.allclose(d2, want_d2, rtol=1e-13, atol=1e-300)


def test_several_passes_and_rows_longer_than_the_lds_keys():
    """Large lists: a query sees about 30,000 candidates (more than the float keys kept in LDS) and the
    distance scratch of the minimum workspace holds a fraction of the rows, so the search runs in passes."""
    from paper_1807_11824_amd import ivf_knn
    X, _ = synth.gaussian_mixture(40_000, 4, 5, 3.0, 1.0, seed=4)
    C, _ = ivf.kmeans_train(X[::10], 4, 3)
    rows = np.random.default_rng(0).choice(40_000, 300, replace=False)
    want_idx, want_d2 = ivf.ivf_knn(X, C, 3, 40, rows=rows)
    idx, d2 = ivf_knn(_dev(X), _dev(C), 3, 40)
    assert np.array_equal(idx.cpu().numpy()[rows], want_idx)
    assert np.allclose(d2.cpu().numpy()[rows], want_d2, rtol=1e-13, atol=1e-300)


def test_long_rows_in_several_passes():
    """140,000 queries of 72 coordinates: two passes of the tile search; sampled rows against the oracle."""
    from paper_1807_11824_amd import ivf_knn
    n, d, nlist, tau, k = 140_000, 72, 374, 3, 10
    X, _ = synth.gaussian_mixture(n, d, 40, 4.0, 1.0, seed=12)
    C = ivf.kmeans_init(X, nlist)
    rows = np.sort(np.random.default_rng(2).choice(n, 96, replace=False))
    want_idx, want_d2 = ivf.ivf_knn(X, C, tau, k, rows=rows)
    idx, d2 = ivf_knn(_dev(X), _dev(C), tau, k)
    assert np.array_equal(idx[rows.tolist()].cpu().numpy(), want_idx)
    assert np.allclose(d2[rows.tolist()].cpu().numpy(), want_d2, rtol=1e-13, atol=1e-300)
    idx = idx.cpu().numpy()
    assert idx.min() >= 0 and idx.max() < n and not np.any(idx == np.arange(n)[:, None])


def test_too_few_candidates_is_reported():
    from paper_1807_11824_amd import ivf_knn, TsneError
    X = np.random.default_rng(1).standard_normal((200, 5)).astype(np.float32)
    C = ivf.kmeans_init(X, 50)
    with pytest.raises(TsneError) as e:
        ivf_knn(_dev(X), _dev(C), 1, 30)
    assert e.value.code == -5


# (the last: 8 centroids, so the rounds run on a sample of 2048 of the 6000 rows)
@pytest.mark.parametrize("n,d,nlist,iters", [(4000, 20, 30, 5), (1500, 70, 12, 3), (300, 3, 300, 2), (6000, 10, 8, 4),
                                             (20000, 96, 700, 3), (400, 65, 400, 2)])
def test_kmeans_matches_oracle(n, d, nlist, iters):
    """Same start, same rule; the means are exact sums here and double sums there, both rounded to float."""
    from paper_1807_11824_amd import ivf_train
    X, _ = synth.gaussian_mixture(n, d, 5, 4.0, 1.0, seed=6)
    want, _ = ivf.kmeans_train(X, nlist, iters)
    got = ivf_train(_dev(X), nlist, iters).cpu().numpy()
    scale = np.abs(X).max()
    assert np.abs(got - want).max() <= 1e-6 * scale
    print("centroids equal bit for bit:", float(np.mean(got == want)), flush=True)


def test_P_from_approximate_neighbours():
    """tsne_build_P_approx against the oracle's pieces in the same order: k-means, search, Eq. (1), symmetric CSR."""
    from paper_1807_11824_amd import build_P_approx
    X, _ = synth.gaussian_mixture(3000, 50, 4, 10.0, 1.0, seed=0)
    nlist, tau, k, perp, iters = 55, 6, 45, 15.0, 6            # nlist = round(sqrt(3000))
    C, _ = ivf.kmeans_train(X, nlist, iters)
    idx, d2 = ivf.ivf_knn(X, C, tau, k)
    cond, _, bad = oracle.cond_p(d2, perp)
    rp, col, val = oracle.symmetrise(idx, cond)
    P = build_P_approx(_dev(X), perp, k, tau, nlist=0, kmeans_iters=iters, want_knn=True)
    got_idx = P["knn_idx"].cpu().numpy()
    same_rows = np.mean(np.all(got_idx == idx, axis=1))
    print(f"rows with identical neighbour lists: {same_rows:.4f}", flush=True)
    # (the Lloyd update adds the members' coordinates as exact fixed-point integers and rounds the mean once, as the
    # oracle's double mean does: the centroids, and with them the lists, are the same bit for bit)
    assert same_rows == 1.0
    assert np.array_equal(P["row_ptr"].cpu().numpy(), rp)
    assert np.array_equal(P["col"].cpu().numpy(), col)
    assert np.allclose(P["val"].cpu().numpy(), val, rtol=2e-6, atol=1e-30)
    assert P["unconverged"] == bad
    exact_idx, _ = oracle.knn(X, k)
    print(f"recall at k = {k}: {ivf.recall(got_idx, exact_idx):.4f} (oracle's own lists: {ivf.recall(idx, exact_idx):.4f})",
          flush=True)


def test_P_build_takes_more_lists_when_a_row_runs_short():
    """200 points in 50 lists of about four, k = 30: one list never holds 30 other points, nor do two, four, ... ;
    tsne_build_P_approx doubles tau until every row has its k candidates and says how far it went."""
    from paper_1807_11824_amd import build_P_approx
    X = np.random.default_rng(1).standard_normal((200, 5)).astype(np.float32)
    P = build_P_approx(_dev(X), 10.0, 30, 1, nlist=50, kmeans_iters=3, want_knn=True)
    tau = P["tau_used"]
    assert tau in (16, 32)
    C, _ = ivf.kmeans_train(X, 50, 3)
    idx, d2 = ivf.ivf_knn(X, C, tau, 30)
    assert np.array_equal(P["knn_idx"].cpu().numpy(), idx)
    with pytest.raises(ValueError):
        ivf.ivf_knn(X, C, tau // 2, 30)


# ---------------------------------------------------------------------------- product-quantised second stage
def _pq_case(name):
    r = np.random.default_rng(3)
    if name == "blobs_32d_m8":
        X, _ = synth.gaussian_mixture(4000, 32, 6, 4.0, 1.0, seed=3)
        return X, 40, 6, 30, 8, 64, 4
    if name == "full_codebooks":             # 256 centroids a sub-quantiser, sub-vectors of 5
        X, _ = synth.gaussian_mixture(6000, 20, 5, 3.0, 1.0, seed=5)
        return X, 25, 5, 40, 4, 256, 3
    if name == "one_subvector":              # m = 1: q2 is a plain vector quantiser of the residual
        X = r.standard_normal((1500, 6)).astype(np.float32)
        return X, 12, 4, 15, 1, 32, 3
    if name == "scalar_subvectors":          # m = d: one coordinate per sub-quantiser
        X = r.standard_normal((2000, 8)).astype(np.float32)
        return X, 10, 10, 20, 8, 16, 3
    if name == "long_subvectors":            # sub-vectors of 70 coordinates: the sub-quantisers train through the tiles
        X, _ = synth.gaussian_mixture(2500, 140, 5, 3.0, 1.0, seed=13)
        return X, 20, 4, 25, 2, 32, 3
    if name == "many_equal_codes":           # few centroids: many candidates share a code and tie exactly (index decides)
        X, _ = synth.gaussian_mixture(3000, 12, 4, 5.0, 1.0, seed=8)
        return X, 8, 3, 50, 2, 4, 2
    raise KeyError(name)


@pytest.mark.parametrize("name", ["blobs_32d_m8", "full_codebooks", "one_subvector", "scalar_subvectors", "long_subvectors",
                                  "many_equal_codes"])
def test_ivfpq_matches_oracle(name):
    """Codebooks (k-means per sub-vector of the residuals), codes and the search of Eq. (11) on the codes: the
    GPU's distances are formed by the same double-precision operations in the same order as the oracle's, so
    indices and distances must be the oracle's."""
    from paper_1807_11824_amd import ivfpq_train, ivfpq_knn
    X, nlist, tau, k, m, ksub, iters = _pq_case(name)
    print(f"case={name} n={X.shape[0]} d={X.shape[1]} nlist={nlist} tau={tau} k={k} m={m} ksub={ksub}", flush=True)
    C, _ = ivf.kmeans_train(X, nlist, 4)
    want_cb = ivf.pq_train(X, C, m, ksub, iters)
    cb = ivfpq_train(_dev(X), _dev(C), m, ksub, iters)
    got_cb = cb.cpu().numpy()
    print("codebooks equal bit for bit:", float(np.mean(got_cb == want_cb)), flush=True)
    assert np.abs(got_cb - want_cb).max() <= 1e-6 * np.abs(X).max()
    # the search from the oracle's codebooks (so that a last-bit difference of a centroid cannot move a code)
    rows = np.arange(0, X.shape[0], 5)
    want_idx, want_d2 = ivf.ivfpq_knn(X, C, want_cb, tau, k, rows=rows)
    idx, d2 = ivfpq_knn(_dev(X), _dev(C), _dev(want_cb), tau, k)
    idx, d2 = idx.cpu().numpy()[rows], d2.cpu().numpy()[rows]
    assert np.array_equal(idx, want_idx)
    assert np.array_equal(d2, want_d2)          # same operations, same order: the same bits
    exact_idx, _ = oracle.knn(X, k, rows=rows.astype(np.int32))
    print(f"recall at k = {k} against the exact lists: {ivf.recall(idx, exact_idx):.4f}", flush=True)


def test_ivfpq_bad_arguments():
    from paper_1807_11824_amd import ivfpq_train, TsneError
    X = _dev(np.zeros((100, 6), np.float32))
    C = _dev(np.zeros((4, 6), np.float32))
    with pytest.raises(TsneError):
        ivfpq_train(X, C, 4, 16, 2)           # 6 coordinates do not split into 4 sub-vectors
    with pytest.raises(TsneError):
        ivfpq_train(X, C, 2, 300, 2)          # more than 256 centroids


@pytest.mark.parametrize("d", [48, 96])      # 96: the coarse centroids are trained through the matrix-core tiles
def test_P_from_product_quantised_neighbours(d):
    """tsne_build_P_approx with pq_m > 0 against the oracle's pieces in the same order: coarse k-means, codebooks,
    codes and search (Eq. (8), (11)), Eq. (1) on the distances to the codes, symmetric CSR."""
    from paper_1807_11824_amd import build_P_approx
    X, _ = synth.gaussian_mixture(3000, d, 4, 10.0, 1.0, seed=1)
    nlist, tau, k, perp, iters, m = 55, 8, 45, 15.0, 5, 12
    C, _ = ivf.kmeans_train(X, nlist, iters)
    cb = ivf.pq_train(X, C, m, 256, iters)
    idx, d2 = ivf.ivfpq_knn(X, C, cb, tau, k)
    cond, _, bad = oracle.cond_p(d2, perp)
    rp, col, val = oracle.symmetrise(idx, cond)
    P = build_P_approx(_dev(X), perp, k, tau, nlist=0, kmeans_iters=iters, want_knn=True, pq_m=m)
    got_idx = P["knn_idx"].cpu().numpy()
    same_rows = np.mean(np.all(got_idx == idx, axis=1))
    print(f"rows with identical neighbour lists: {same_rows:.4f}", flush=True)
    assert same_rows == 1.0
    assert np.array_equal(P["row_ptr"].cpu().numpy(), rp)
    assert np.array_equal(P["col"].cpu().numpy(), col)
    assert np.allclose(P["val"].cpu().numpy(), val, rtol=2e-6, atol=1e-30)
    assert P["unconverged"] == bad
    exact_idx, _ = oracle.knn(X, k)
    print(f"recall at k = {k} against the exact lists: {ivf.recall(got_idx, exact_idx):.4f}", flush=True)
