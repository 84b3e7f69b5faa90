"""GPU vs oracle on seeded random shapes, sizes and parameters around the kernels' thresholds (row lengths 63/64/65,
255/256/257, sort sizes 8192/8193, leaf sizes 1 … 40, grids of 5 … 22 bits, with and without renumbering).

The fixed cases of the other files pin the paths one by one; these sweep combinations nobody thought of.  Bars as
elsewhere: neighbour indices bit-exact, tree bit-exact, forces within 1e-4, Z within 1e-5."""
import numpy as np
import pytest

import oracle
from oracle import ivf
from oracle.oracle import RunParams
from helpers import grid_bits, random_symmetric_csr, rel_l2
from paper_1807_11824_amd import synth

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _rows_like(rng, n, d, kind, seed):
    if kind == 0:
        return synth.gaussian_mixture(n, d, 7, 3.0, 1.0, seed=seed)[0]
    if kind == 1:
        return (rng.standard_normal((n, d)) * 10 ** rng.uniform(-3, 3) + 10 ** rng.uniform(-2, 2)).astype(np.float32)
    if kind == 2:
        return synth.lattice(n, d, span=3, seed=seed)             # ties at every distance
    base = rng.standard_normal((n // 5 + 1, d)).astype(np.float32)
    return np.ascontiguousarray(np.repeat(base, 5, axis=0)[:n] + (rng.standard_normal((n, d)) * 1e-3).astype(np.float32))


def test_exact_knn_on_random_shapes():
    from paper_1807_11824_amd import build_P
    rng = np.random.default_rng(1)
    dims = [3, 17, 50, 63, 64, 65, 100, 128, 200, 255, 256, 257, 300, 320, 383, 384, 500, 777, 1024, 1500, 2048, 2049]
    for case in range(40):
        d = int(rng.choice(dims))
        n = int(rng.choice([130, 257, 300, 511, 513, 700, 1025, 2000, 3001, 4099]))
        k = min(int(rng.choice([1, 5, 30, 90])), n - 1)
        kind = int(rng.integers(0, 4))
        X = _rows_like(rng, n, d, kind, case)
        print(f"case {case}: n={n} d={d} k={k} kind={kind}", flush=True)
        r = build_P(_dev(X), float(min(30.0, max(1.0, k / 3))), k, want_knn=True)
        rows = np.sort(rng.choice(n, min(n, 150), replace=False))
        want_idx, want_d2 = oracle.knn(X, k, rows=rows)
        assert np.array_equal(r["knn_idx"].cpu().numpy()[rows], want_idx), case
        assert np.allclose(r["knn_d2"].cpu().numpy()[rows], want_d2, rtol=1e-6, atol=0), case


def test_inverted_file_search_on_random_shapes():
    from paper_1807_11824_amd import TsneError, ivf_knn
    rng = np.random.default_rng(4)
    done = 0
    for case in range(40):
        d = int(rng.choice([2, 9, 50, 63, 64, 65, 66, 96, 128, 129, 200, 300]))
        n = int(rng.choice([200, 513, 1000, 2500, 4099, 7000]))
        nlist = min(int(rng.choice([1, 2, 7, 20, 50])), n // 4)
        tau = min(int(rng.integers(1, nlist + 1)), 12)
        kind = int(rng.integers(0, 4))
        X = _rows_like(rng, n, d, kind, case)
        C = ivf.kmeans_init(X, nlist)
        k = int(rng.choice([1, 10, 40, 90]))
        print(f"case {case}: n={n} d={d} nlist={nlist} tau={tau} k={k} kind={kind}", flush=True)
        try:
            want_idx, want_d2 = ivf.ivf_knn(X, C, tau, k)
        except Exception:
            # some query finds fewer than k candidates in its lists: the library must refuse as well
            with pytest.raises(TsneError):
                ivf_knn(_dev(X), _dev(C), tau, k)
            continue
        idx, d2 = ivf_knn(_dev(X), _dev(C), tau, k)
        assert np.array_equal(idx.cpu().numpy(), want_idx), case
        assert np.allclose(d2.cpu().numpy(), want_d2, rtol=1e-13, atol=1e-300), case
        done += 1
    assert done >= 25


def _points_like(rng, n, kind, seed):
    if kind == 0:
        return synth.y0(n, seed=seed)
    if kind == 1:
        return synth.clustered_embedding(n, n_clusters=int(rng.integers(1, 50)), spread=float(10 ** rng.uniform(-1, 2)),
                                         sigma=float(10 ** rng.uniform(-2, 0.5)), seed=seed)
    if kind == 2:
        return np.vstack([rng.random((n - 1, 2)) * 1e-2, [[500.0, -300.0]]]).astype(np.float32)          # an outlier
    if kind == 3:
        return np.repeat(rng.standard_normal((n // 7 + 1, 2)).astype(np.float32), 7, axis=0)[:n].copy()   # every point 7 times
    return (rng.standard_normal((n, 2)) * np.array([1e3, 1e-3])).astype(np.float32)                       # nearly a line


def test_tree_and_forces_on_random_parameters():
    """Sec. III-C step 4 leaves the order of points with equal grid keys open.  Without renumbering the library
    orders them by index, as the oracle does by default, and everything is compared as it is.  With renumbering it
    orders them by its internal number: the test then checks that its order is a sorted one (a permutation along
    which the keys do not decrease), hands the oracle that order as the rank for equal keys, and compares cells,
    order and forces with the oracle's for that rank (kinds 3 and 4 and the coarse grids have many equal keys)."""
    import torch
    from paper_1807_11824_amd import Tsne
    rng = np.random.default_rng(5)
    for case in range(40):
        n = int(rng.choice([3, 70, 129, 1000, 4097, 8192, 8193, 9000, 20011]))
        theta = float(rng.choice([0.0, 0.2, 0.5, 0.7]))
        leaf_cap = int(rng.choice([1, 2, 4, 8, 16, 17, 40]))
        bits = int(rng.choice([5, 9, 12, 16, 20, 22]))
        if 2 * bits + (n - 1).bit_length() > 64:
            bits = 16
        kind = int(rng.integers(0, 5))
        Y = _points_like(rng, n, kind, case)
        deg = min(int(rng.choice([1, 5, 30])), n - 1)
        rp, col, val = random_symmetric_csr(n, deg, seed=case)
        params = dict(theta=theta, leaf_cap=leaf_cap, morton_bits=bits)
        want = oracle.tree(Y, bits=bits, leaf_cap=leaf_cap)
        ties = len(np.unique(want["keys"])) < n
        renumber = bool(rng.integers(0, 2))
        if renumber:
            params.update(max_nnz=len(col), far_tiles=int(rng.choice([0, 1, 2])))
        print(f"case {case}: n={n} kind={kind} deg={deg} ties={ties} {params}", flush=True)
        t = Tsne(n, **params)
        t.set_P(_dev(rp), _dev(col), _dev(val))
        A, R, Z = t.gradient(_dev(Y))
        st = t.status()
        A, R, Z = A.cpu().numpy(), R.cpu().numpy(), float(Z.cpu().numpy()[0])
        tree = {k: (v.cpu().numpy() if hasattr(v, "cpu") else v) for k, v in t.export_tree().items()}
        t.close()
        assert st == 0
        tie_rank = None
        if renumber and ties:
            perm = tree["perm"].astype(np.int64)
            assert np.array_equal(np.sort(perm), np.arange(n)), case
            assert np.all(np.diff(want["keys"][perm].astype(np.int64)) >= 0), case       # (keys < 2^44)
            tie_rank = np.empty(n, np.int32)
            tie_rank[perm] = np.arange(n, dtype=np.int32)
            want = oracle.tree(Y, bits=bits, leaf_cap=leaf_cap, tie_rank=tie_rank)
        assert tree["m"] == want["m"] and np.array_equal(tree["keys"].view(np.uint64), want["keys"]), case
        for f in ("depth", "lo", "hi", "leaf", "perm"):
            assert np.array_equal(tree[f], want[f]), (case, f)
        o = oracle.grad_bh(Y, rp, col, val.astype(np.float64), theta=theta, leaf_cap=leaf_cap, group=64, alpha=1.0, bits=bits,
                           tie_rank=tie_rank)
        assert rel_l2(A, o["A"]) <= 1e-4 and rel_l2(R, o["R"]) <= 1e-4, case
        if o["Z"] > n:        # (a few points very far apart: the point's own term limits Z to 2^-24 absolute per point)
            assert abs(Z - o["Z"]) <= 1e-5 * o["Z"], case


def test_short_runs_on_random_parameters():
    """A few iterations from random places of the schedule (either side of the end of the exaggeration and of the
    momentum switch), with and without renumbering (also during the run), one or two streams."""
    import torch
    from paper_1807_11824_amd import Tsne
    rng = np.random.default_rng(11)
    for case in range(30):
        n = int(rng.choice([500, 2000, 5000, 9000, 12000]))
        deg = int(rng.choice([3, 10, 30]))
        rp, col, val = random_symmetric_csr(n, deg, seed=case)
        Y0 = synth.y0(n, seed=case) if rng.integers(0, 2) == 0 else synth.clustered_embedding(
            n, n_clusters=int(rng.integers(2, 40)), spread=float(rng.uniform(2, 30)), sigma=float(rng.uniform(0.3, 2)), seed=case)
        iters = int(rng.choice([3, 6, 10]))
        iter0 = int(rng.choice([0, 247, 248, 400]))
        kw = dict(theta=float(rng.choice([0.3, 0.5, 0.7])), leaf_cap=int(rng.choice([2, 8, 16])),
                  lr=float(rng.choice([50.0, 200.0, 800.0])), exaggeration=float(rng.choice([4.0, 12.0])),
                  exaggeration_iters=int(rng.choice([250, 249])), momentum_switch_iter=int(rng.choice([250, 251])),
                  momentum_early=0.5, momentum_late=0.8)
        extra = {}
        mode = int(rng.integers(0, 4))
        if mode >= 1:
            extra.update(max_nnz=len(col), far_tiles=int(rng.choice([0, 1, 2])))
        if mode == 3:
            extra.update(reorder_every=int(rng.choice([2, 3])))
        overlap = int(rng.integers(0, 2))
        print(f"case {case}: n={n} deg={deg} iters={iters} iter0={iter0} {kw} {extra} overlap={overlap}", flush=True)
        t = Tsne(n, overlap=overlap, **kw, **extra)
        t.set_P(_dev(rp), _dev(col), _dev(val))
        Yd = _dev(Y0.copy())
        t.run(Yd, iters, iter0=iter0)
        st = t.status()
        Yg = Yd.cpu().numpy()
        t.close()
        Yo, _, _ = oracle.run(Y0, rp, col, val, RunParams.default(bits=grid_bits(n), group=64, **kw), iters, iter0=iter0)
        assert st == 0
        assert rel_l2(Yg - Y0, Yo - Y0.astype(np.float64)) <= 2e-3, case       # the displacement over these iterations
