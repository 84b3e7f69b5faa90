"""Seeded synthetic inputs with the shapes of the paper's workloads.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no distances, affinities, trees or forces), so the tests
may hand its arrays to both the GPU library and the CPU oracle.

The paper measures on MNIST, CIFAR-10, ImageNet network codes and GloVe
vectors (Sec. IV-A, V); none of those files exist here, so each configuration
below is a stand-in with the same N, D, value range and cluster structure.
Labels are drawn i.i.d., so rows are not cluster-sorted and the sparsity
pattern of P is as disorganised as Sec. IV-D describes.
"""
import numpy as np

CONFIGS = {
    # name: N, D, perplexity, k
    "cfg1": dict(n=2000, d=50, perplexity=30.0, k=90),
    "cfg2": dict(n=60000, d=784, perplexity=30.0, k=90),
    "cfg3": dict(n=50000, d=3072, perplexity=50.0, k=150),
    "cfg4": dict(n=400000, d=300, perplexity=30.0, k=90),
    "cfg5": dict(n=1281167, d=2048, perplexity=30.0, k=90),
}


def _rngs(seed):
    sx, sy = np.random.SeedSequence(seed).spawn(2)
    return np.random.default_rng(sx), np.random.default_rng(sy)


def y0(n, seed=0):
    """Initial embedding: N(0, 1e-4 I), i.e. sigma = 0.01, float32, n x 2."""
    _, ry = _rngs(seed)
    return (0.01 * ry.standard_normal((n, 2))).astype(np.float32)


def gaussian_mixture(n, d, n_clusters, mean_scale, sigma, seed=0, weights=None, chunk=65536,
                     out=None, relu=False):
    """Rows ~ N(mu_c, sigma^2 I) with mu_c ~ N(0, mean_scale^2 I); labels i.i.d."""
    rx, _ = _rngs(seed)
    means = (mean_scale * rx.standard_normal((n_clusters, d))).astype(np.float32)
    labels = rx.choice(n_clusters, size=n, p=weights)
    X = out if out is not None else np.empty((n, d), np.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        blk = means[labels[s:e]] + sigma * rx.standard_normal((e - s, d), dtype=np.float32)
        if relu:
            np.maximum(blk, 0.0, out=blk)
        X[s:e] = blk
    return X, labels


def config1(n=2000, d=50, seed=0):
    """Paper's simulated data (Sec. IV-A): equal-weight Gaussian clusters in 50-d."""
    return gaussian_mixture(n, d, 10, 10.0, 1.0, seed)


def config2(n=60000, d=784, seed=0):
    """MNIST-shaped: values in [0,1], ten clusters, about 80% of entries zero."""
    rx, _ = _rngs(seed)
    active = rx.random((10, d)) < 0.2                       # per-cluster active dimensions
    means = rx.uniform(0.3, 0.9, (10, d)).astype(np.float32) * active
    labels = rx.integers(0, 10, n)
    X = np.empty((n, d), np.float32)
    for s in range(0, n, 8192):
        e = min(n, s + 8192)
        lab = labels[s:e]
        blk = means[lab] + 0.15 * rx.standard_normal((e - s, d), dtype=np.float32)
        blk *= active[lab]
        np.clip(blk, 0.0, 1.0, out=blk)
        X[s:e] = blk
    return X, labels


def config3(n=50000, d=3072, seed=0):
    """CIFAR-10 raw-pixel shaped: dense values in [0,1], ten clusters."""
    rx, _ = _rngs(seed)
    means = rx.uniform(0.2, 0.8, (10, d)).astype(np.float32)
    labels = rx.integers(0, 10, n)
    X = np.empty((n, d), np.float32)
    for s in range(0, n, 4096):
        e = min(n, s + 4096)
        blk = means[labels[s:e]] + 0.2 * rx.standard_normal((e - s, d), dtype=np.float32)
        np.clip(blk, 0.0, 1.0, out=blk)
        X[s:e] = blk
    return X, labels


def config4(n=400000, d=300, seed=0):
    """GloVe-shaped: 200 clusters with heavy-tailed sizes, row norms ~ N(6,1)."""
    rx, _ = _rngs(seed)
    w = np.abs(rx.standard_t(3, 200)) + 1e-3
    w /= w.sum()
    means = rx.standard_normal((200, d)).astype(np.float32)
    labels = rx.choice(200, size=n, p=w)
    X = np.empty((n, d), np.float32)
    for s in range(0, n, 32768):
        e = min(n, s + 32768)
        blk = means[labels[s:e]] + 0.5 * rx.standard_normal((e - s, d), dtype=np.float32)
        r = np.maximum(rx.normal(6.0, 1.0, e - s), 0.5).astype(np.float32)
        blk *= (r / np.linalg.norm(blk, axis=1))[:, None]
        X[s:e] = blk
    return X, labels


def config5(n=1281167, d=2048, seed=0, out=None):
    """ImageNet-code shaped: ReLU of a 1000-cluster Gaussian mixture, non-negative."""
    return gaussian_mixture(n, d, 1000, 1.0, 1.0, seed, chunk=16384, out=out, relu=True)


def clustered_embedding(n, n_clusters=1000, spread=40.0, sigma=0.6, seed=0):
    """A mid-run-looking embedding (separated blobs), for fixed-Y tests at scale."""
    _, ry = _rngs(seed)
    c = spread * ry.standard_normal((n_clusters, 2))
    lab = ry.integers(0, n_clusters, n)
    return (c[lab] + sigma * ry.standard_normal((n, 2))).astype(np.float32)


def lattice(n, d, span=4, seed=0):
    """Integer-valued rows: every squared distance is an exact integer with many ties."""
    rx, _ = _rngs(seed)
    return rx.integers(0, span, (n, d)).astype(np.float32)
