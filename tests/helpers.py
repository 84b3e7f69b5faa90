"""Shared helpers of the GPU parity tests (no method arithmetic)."""
import numpy as np


def grid_bits(n):
    """Grid bits per axis the library takes by default for n points (include/tsne.h, morton_bits): the oracle's
    tree takes the depth as a parameter, and a comparison has to build both trees to the same depth."""
    return min(22, (64 - max(0, int(n) - 1).bit_length()) // 2)


def rel_l2(a, b):
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def worst_point(g, o):
    """max over points i of |g_i - o_i| / (|o_i| + median_j |o_j|): a per-point companion of the relative L2 norm,
    which a large error confined to a few of a million points would pass."""
    g = np.asarray(g, np.float64); o = np.asarray(o, np.float64)
    mag = np.linalg.norm(o, axis=1)
    return float((np.linalg.norm(g - o, axis=1) / (mag + np.median(mag) + 1e-300)).max())


def random_symmetric_csr(n, deg, seed=0):
    """A symmetric sparsity pattern with about 2*deg entries per row and positive values summing to 1.

    Stands in for P where only the kernels' handling of a CSR matrix is under test."""
    import scipy.sparse as sp
    rng = np.random.default_rng(seed)
    rows = np.repeat(np.arange(n, dtype=np.int64), deg)
    # neighbours mostly near in index (clustered) with a random tail, so rows differ in length
    near = (rows + rng.integers(1, 2000, rows.shape[0])) % n
    far = rng.integers(0, n, rows.shape[0])
    cols = np.where(rng.random(rows.shape[0]) < 0.7, near, far)
    keep = cols != rows
    M = sp.coo_matrix((rng.random(keep.sum()) + 0.01, (rows[keep], cols[keep])), shape=(n, n)).tocsr()
    M = (M + M.T).tocsr()
    M.sum_duplicates()
    M.sort_indices()
    M.data /= M.data.sum()
    return M.indptr.astype(np.int32), M.indices.astype(np.int32), M.data.astype(np.float32)
