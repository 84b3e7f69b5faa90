"""GPU vs oracle, integer work: keys, spatial order and quad tree must match bit for bit."""
import numpy as np
import pytest

import oracle
from paper_1807_11824_amd import synth

pytestmark = pytest.mark.gpu


def _gpu_tree(Y, bits, leaf_cap):
    import torch
    from paper_1807_11824_amd import Tsne
    n = Y.shape[0]
    t = Tsne(n, morton_bits=bits, leaf_cap=leaf_cap)
    dev = torch.device("cuda:0")
    rp = torch.zeros(n + 1, dtype=torch.int32, device=dev)
    t.set_P(rp, torch.zeros(0, dtype=torch.int32, device=dev), torch.zeros(0, dtype=torch.float32, device=dev))
    Yd = torch.from_numpy(Y).to(dev)
    t.gradient(Yd)
    out = t.export_tree()
    assert t.status() == 0
    res = {k: (v.cpu().numpy() if hasattr(v, "cpu") else v) for k, v in out.items()}
    t.close()
    return res


def _rng_cases():
    r = np.random.default_rng(7)
    return {
        "one": np.array([[0.5, -2.0]], np.float32),
        "two": np.array([[0, 0], [1, 3]], np.float32),
        "all_same": np.full((300, 2), 1.25, np.float32),
        "duplicates": np.repeat(r.random((50, 2)).astype(np.float32), 13, axis=0),
        "collinear": np.stack([np.linspace(-3, 5, 1000), np.full(1000, 2.0)], 1).astype(np.float32),
        "blob_5003": synth.y0(5003, seed=1),
        # either side of the size up to which one workgroup sorts in LDS
        "blob_8192": synth.clustered_embedding(8192, n_clusters=30, seed=5),
        "blob_8193": synth.clustered_embedding(8193, n_clusters=30, seed=5),
        "outlier": np.vstack([r.random((4097, 2)) * 1e-3, [[100.0, -50.0]]]).astype(np.float32),
        "clusters_100k": synth.clustered_embedding(100_003, n_clusters=300, seed=2),
        "collapsed_clusters": synth.clustered_embedding(30_000, n_clusters=20, spread=5.0, sigma=1e-4, seed=3),
        # every point twice: with leaf_cap = 1 a chain of one-child cells runs to the deepest level under each pair
        # (about 4.7 cells per point, more than any other case here)
        "pairs_20000": np.repeat(r.random((10_000, 2)).astype(np.float32), 2, axis=0),
        # many points in single squares of 1/2048 of the root's side (long runs of equal leading key bits, as the
        # clusters of a late embedding give): copies of one point, a tight clump, twenty clumps of 150-400 points, a
        # uniform background
        "clumps_20011": np.vstack(
            [np.full((3000, 2), 0.3)] + [[0.7, 0.2] + 1e-6 * r.random((2000, 2))]
            + [r.random(2) + 2e-5 * r.random((int(m), 2)) for m in r.integers(150, 400, 20)]
            + [r.random((20011, 2))])[:20011].astype(np.float32),
    }


CASES = _rng_cases()


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("bits,leaf_cap", [(16, 8), (16, 1), (7, 3), (10, 8), (16, 40), (22, 8), (21, 2), (24, 1)])
def test_tree_matches_oracle(name, bits, leaf_cap):
    Y = CASES[name]
    if 2 * bits + (Y.shape[0] - 1).bit_length() > 64:
        pytest.skip("key and point number do not fit one 64-bit word (the library refuses the combination)")
    print(f"case={name} n={Y.shape[0]} bits={bits} leaf_cap={leaf_cap}", flush=True)
    want = oracle.tree(Y, bits=bits, leaf_cap=leaf_cap)
    got = _gpu_tree(Y, bits, leaf_cap)
    assert np.array_equal(got["root"], want["root"])
    assert np.array_equal(got["keys"].view(np.uint64), want["keys"])
    assert np.array_equal(got["perm"], want["perm"])
    assert got["m"] == want["m"]
    for f in ("depth", "lo", "hi", "leaf"):
        assert np.array_equal(got[f], want[f]), f
    # centres of mass: both sides round a double-precision mean to float
    scale = float(want["root"][2])
    assert np.abs(got["com"].astype(np.float64) - want["com"].astype(np.float64)).max() <= 1e-6 * scale
    frac_equal = np.mean(got["com"] == want["com"])
    assert frac_equal > 0.999


def test_nonfinite_is_flagged():
    import torch
    from paper_1807_11824_amd import Tsne, STATUS_NONFINITE
    Y = synth.y0(1000, seed=0)
    Y[17, 1] = np.nan
    t = Tsne(1000)
    dev = torch.device("cuda:0")
    t.set_P(torch.zeros(1001, dtype=torch.int32, device=dev), torch.zeros(0, dtype=torch.int32, device=dev),
            torch.zeros(0, dtype=torch.float32, device=dev))
    t.gradient(torch.from_numpy(Y).to(dev))
    assert t.status() & STATUS_NONFINITE
    t.close()
