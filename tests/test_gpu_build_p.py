"""GPU vs oracle: kNN indices bit-exact, calibrated and symmetrised P within float rounding."""
import numpy as np
import pytest

import oracle
from paper_1807_11824_amd import synth

pytestmark = pytest.mark.gpu


def _gpu_P(X, perplexity, k):
    import torch
    from paper_1807_11824_amd import build_P
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to("cuda:0")
    r = build_P(Xd, perplexity, k, want_knn=True)
    out = {}
    for key, v in r.items():
        out[key] = v.cpu().numpy() if hasattr(v, "cpu") else v
    return out


def _check_against_oracle(X, perplexity, k, rows=None):
    perplexity = float(np.float32(perplexity))     # the C ABI takes the perplexity as a float
    g = _gpu_P(X, perplexity, k)
    n = X.shape[0]
    if rows is None:
        o = oracle.build_P(X, perplexity, k)
        assert np.array_equal(g["knn_idx"], o["idx"])
        assert np.allclose(g["knn_d2"], o["d2"], rtol=1e-6, atol=0)
        assert g["unconverged"] == o["unconverged"]
        assert np.array_equal(g["row_ptr"], o["row_ptr"])
        assert np.array_equal(g["col"], o["col"])
        # float storage of a double-precision value: half an ulp, plus the bisection's 1e-10 stop
        rel = np.abs(g["val"].astype(np.float64) - o["val"]) / np.maximum(o["val"], 1e-300)
        print("max rel err of val", rel.max(), "at", int(rel.argmax()), "oracle val", o["val"][rel.argmax()], flush=True)
        assert np.allclose(g["val"], o["val"], rtol=2e-7, atol=1e-30)
    else:
        idx, d2 = oracle.knn(X, k, rows=rows)
        assert np.array_equal(g["knn_idx"][rows], idx)
        assert np.allclose(g["knn_d2"][rows], d2, rtol=1e-6, atol=0)
        cond, _, _ = oracle.cond_p(d2, perplexity)
    # invariants that hold at any size (Sec. III-A/B)
    import scipy.sparse as sp
    M = sp.csr_matrix((g["val"], g["col"], g["row_ptr"]), shape=(n, n))
    assert (M != M.T).nnz == 0
    assert abs(g["val"].astype(np.float64).sum() - 1.0) < 1e-5
    assert n * k <= g["nnz"] <= 2 * n * k
    assert np.all(np.diff(g["row_ptr"]) >= k)
    return g


def test_config1_full():
    X, _ = synth.config1()
    g = _check_against_oracle(X, 30.0, 90)
    assert g["unconverged"] == 0


def test_lattice_ties():
    """Exact integer distances with many ties: order by (distance, index), fall-back selection path."""
    X = synth.lattice(700, 6, span=3, seed=1)
    _check_against_oracle(X, 5.0, 17)


@pytest.mark.parametrize("n,d,k", [(300, 51, 20), (1000, 7, 40), (129, 33, 128), (2500, 130, 90)])
def test_ragged_shapes(n, d, k):
    rng = np.random.default_rng(d)
    X = rng.standard_normal((n, d)).astype(np.float32)
    _check_against_oracle(X, min(30.0, k / 3.0), k)


def test_duplicates():
    rng = np.random.default_rng(0)
    X = np.repeat(rng.standard_normal((200, 16)).astype(np.float32), 3, axis=0)
    _check_against_oracle(X, 5.0, 15)


def test_config2_shape_sampled_rows():
    X, _ = synth.config2(n=20000)
    rows = np.random.default_rng(1).choice(20000, 256, replace=False).astype(np.int32)
    _check_against_oracle(X, 30.0, 90, rows=np.sort(rows))


def test_config3_shape_sampled_rows():
    X, _ = synth.config3(n=6000)
    rows = np.random.default_rng(2).choice(6000, 128, replace=False).astype(np.int32)
    _check_against_oracle(X, 50.0, 150, rows=np.sort(rows))


@pytest.mark.parametrize("n,d,k", [(40000, 50, 90), (20000, 20, 30), (16500, 64, 45)])
def test_small_d_many_rows_sampled(n, d, k):
    """Enough rows and few enough columns for the tile kernel that keeps the query rows in LDS
    (one slab at d <= 32, two up to 64); clustered like the scaling workload of Sec. IV-B."""
    X, _ = synth.gaussian_mixture(n, d, 4, 10.0, 1.0, seed=d)
    rows = np.sort(np.random.default_rng(d).choice(n, 192, replace=False).astype(np.int32))
    rows[:3] = [0, 255, 256]
    rows[-2:] = [n - 2, n - 1]
    _check_against_oracle(X, 30.0 if k >= 90 else 10.0, k, rows=np.unique(rows))


@pytest.mark.parametrize("offset,sigma", [(30.0, 1.0), (300.0, 0.01)])
def test_far_from_the_origin(offset, sigma):
    """Norms much larger than the distances.  The candidate search works on X minus its column means
    (distances do not change), so the rows certify as they would around the origin and the lists are the oracle's."""
    import time
    rng = np.random.default_rng(int(offset))
    n = 50_000
    X = (offset + sigma * rng.standard_normal((n, 20))).astype(np.float32)
    rows = np.sort(rng.choice(n, 256, replace=False).astype(np.int32))
    _gpu_P(X[:4000], 10.0, 30)          # (first call: kernels are loaded)
    t0 = time.time()
    _check_against_oracle(X, 10.0, 30, rows=rows)
    print(f"offset {offset}: tsne_build_P + oracle on 256 rows {time.time() - t0:.2f} s", flush=True)


def test_many_rows_without_certificate():
    """Lattice points with heavy duplication: nearly every row has ties at its k-th distance, cannot be certified
    and goes through the exact fall-back, which takes the failed rows 2k at a time."""
    X = synth.lattice(20_000, 6, span=3, seed=3)
    rows = np.sort(np.random.default_rng(5).choice(20_000, 256, replace=False).astype(np.int32))
    _check_against_oracle(X, 5.0, 17, rows=rows)


def test_bad_arguments():
    import torch
    from paper_1807_11824_amd import build_P, TsneError
    X = torch.zeros((10, 4), device="cuda:0")
    with pytest.raises(TsneError):
        build_P(X, 3.0, 10)        # k must be < n
    with pytest.raises(TsneError):
        build_P(X, 9.0, 5)         # perplexity must be <= k


@pytest.mark.parametrize("clusters,scale", [(300, 3.0), (1, 0.0)])
def test_many_long_rows_sampled(clusters, scale):
    """200,001 rows of 96 coordinates (the general tile kernel, several query blocks, a ragged last tile):
    clustered data and a single Gaussian blob, sampled rows against the oracle."""
    n, d, k = 200_001, 96, 60
    X, _ = synth.gaussian_mixture(n, d, clusters, scale, 1.0, seed=11)
    rows = np.sort(np.random.default_rng(2).choice(n, 192, replace=False).astype(np.int32))
    rows[0], rows[-1] = 0, n - 1
    _check_against_oracle(X, 20.0, k, rows=np.unique(rows))


@pytest.mark.parametrize("name", ["plane", "lattice", "copies", "blobs", "tiny", "one_tile_and_a_row"])
def test_rows_of_256_and_more_coordinates(name):
    """Rows this long are swept with the high parts of the split values first and only the rows without a
    certificate go on to the three-product tiles and, failing that, to the exact pass.
    plane: a densely sampled plane in 300 dimensions (neighbours closer together than 2^-8 of the norms: the first
    sweep certifies nobody, the second everybody); lattice: integer points with exact ties (nobody is certified by
    either); copies: every row five times; blobs: clustered data that the first sweep settles."""
    r = np.random.default_rng(21)
    if name == "plane":
        n, d, k = 20_000, 300, 90
        basis, _ = np.linalg.qr(r.standard_normal((d, 2)))
        X = (r.uniform(0.0, 100.0, (n, 2)) @ basis.T).astype(np.float32)
    elif name == "lattice":
        n, d, k = 3000, 256, 40
        X = np.zeros((n, d), np.float32)
        X[:, :3] = r.integers(0, 6, (n, 3)).astype(np.float32)
    elif name == "copies":
        n, d, k = 2500, 320, 23
        X = np.repeat(r.standard_normal((500, d)).astype(np.float32), 5, axis=0)
    elif name == "tiny":
        n, d, k = 70, 260, 10
        X = r.standard_normal((n, d)).astype(np.float32)
    elif name == "one_tile_and_a_row":       # 257 rows: a second tile with a single row in it
        n, d, k = 257, 512, 30
        X, _ = synth.gaussian_mixture(n, d, 3, 2.0, 1.0, seed=23)
    else:
        n, d, k = 70_000, 257, 60
        X, _ = synth.gaussian_mixture(n, d, 50, 3.0, 1.0, seed=22)
    rows = None if n <= 3000 else np.unique(np.sort(r.choice(n, 128, replace=False).astype(np.int32)))
    _check_against_oracle(X, min(20.0, k / 3.0), k, rows=rows)
