"""Pins for the oracle's integer work: bounding box, keys, sort, quad tree (Sec. III-C steps 1-4).

The check is a second, geometric construction written here in Python: points
are put in grid cells by comparing integer grid coordinates and cells are split
recursively into quadrants.  It never forms an interleaved key, so a slip in
the bit interleave, the quadrant order, the key-range split or the leaf rule
of the C file shows up as a different set of cells.
"""
import numpy as np
import pytest

import oracle


def _grid_coords(Y, bits):
    """Quantisation restated with numpy float32 scalars (root square and grid index)."""
    Y = np.asarray(Y, np.float32)
    mn = Y.min(0)
    ext = (Y.max(0) - mn).astype(np.float32)
    e = np.float32(max(ext[0], ext[1]))
    W = np.float32(2.0) ** np.float32(-40)
    while W < e:
        W = np.float32(W * np.float32(2))
    S = np.float32(np.float32(2.0 ** bits) / W)
    q = np.floor(((Y - mn).astype(np.float32) * S).astype(np.float32))
    q = np.minimum(q, 2 ** bits - 1).astype(np.int64)
    return mn, W, q


def _brute_cells(q, bits, leaf_cap):
    """Recursive quadrant splitting on integer grid coordinates -> list of (depth, members, leaf)."""
    cells = []

    def rec(members, depth, cx, cy):
        is_leaf = len(members) <= leaf_cap or depth == bits
        cells.append((depth, cx, cy, tuple(sorted(members)), is_leaf))
        if is_leaf:
            return
        sh = bits - depth - 1
        for by in (0, 1):            # lower half in y first, then within it lower x first
            for bx in (0, 1):
                sub = [i for i in members if ((q[i, 0] >> sh) & 1) == bx and ((q[i, 1] >> sh) & 1) == by]
                if sub:
                    rec(sub, depth + 1, cx * 2 + bx, cy * 2 + by)

    rec(list(range(q.shape[0])), 0, 0, 0)
    return cells


CASES = {
    "uniform": lambda r: r.random((257, 2)).astype(np.float32),
    "gauss_blob": lambda r: (0.01 * r.standard_normal((400, 2))).astype(np.float32),
    "duplicates": lambda r: np.repeat(r.random((20, 2)).astype(np.float32), 5, axis=0),
    "collinear": lambda r: np.stack([np.linspace(-3, 5, 100), np.full(100, 2.0)], 1).astype(np.float32),
    "all_same": lambda r: np.full((33, 2), 1.25, np.float32),
    "two": lambda r: np.array([[0, 0], [1, 3]], np.float32),
    "one": lambda r: np.array([[0.5, -2]], np.float32),
    "far_outlier": lambda r: np.vstack([r.random((64, 2)) * 1e-3, [[100.0, -50.0]]]).astype(np.float32),
    # tight clumps far apart: only a grid finer than 2^16 cells per axis separates the members of a clump
    "tiny_clumps": lambda r: (np.repeat(r.random((6, 2)) * 50.0, 40, axis=0)
                              + 2e-4 * r.standard_normal((240, 2))).astype(np.float32),
}


@pytest.mark.parametrize("name", sorted(CASES))
@pytest.mark.parametrize("bits,leaf_cap", [(16, 1), (16, 8), (5, 2), (1, 1), (17, 2), (22, 4), (24, 1)])
def test_tree_equals_geometric_construction(name, bits, leaf_cap):
    Y = CASES[name](np.random.default_rng(11))
    n = Y.shape[0]
    t = oracle.tree(Y, bits=bits, leaf_cap=leaf_cap)
    mn, W, q = _grid_coords(Y, bits)
    assert np.array_equal(t["root"], np.array([mn[0], mn[1], W], np.float32))
    # keys decode to the grid coordinates: even bits x, odd bits y
    for i in range(n):
        kx = sum(((int(t["keys"][i]) >> (2 * b)) & 1) << b for b in range(bits))
        ky = sum(((int(t["keys"][i]) >> (2 * b + 1)) & 1) << b for b in range(bits))
        assert (kx, ky) == (q[i, 0], q[i, 1])
    # sort: stable, by key
    want_perm = np.argsort(t["keys"], kind="stable")
    assert np.array_equal(t["perm"], want_perm)
    assert np.array_equal(t["sorted_keys"], t["keys"][want_perm])
    # cells: same pre-order list of (depth, grid cell, member set, leaf flag)
    cells = _brute_cells(q, bits, leaf_cap)
    assert t["m"] == len(cells)
    for c, (depth, cx, cy, members, is_leaf) in enumerate(cells):
        assert t["depth"][c] == depth and bool(t["leaf"][c]) == is_leaf
        got = tuple(sorted(int(v) for v in t["perm"][t["lo"][c]:t["hi"][c]]))
        assert got == members
        px = sum(((int(t["prefix"][c]) >> (2 * b)) & 1) << b for b in range(depth))
        py = sum(((int(t["prefix"][c]) >> (2 * b + 1)) & 1) << b for b in range(depth))
        assert (px, py) == (cx, cy)
        mean = Y[list(members)].astype(np.float64).mean(0)
        assert np.allclose(t["com"][c], mean, rtol=1e-6, atol=1e-30)


def test_tree_invariants_larger():
    rng = np.random.default_rng(4)
    Y = np.vstack([rng.standard_normal((3000, 2)) * 0.3 + c for c in ((0, 0), (8, 1), (-5, 6))]).astype(np.float32)
    t = oracle.tree(Y, bits=16, leaf_cap=8)
    n, m = Y.shape[0], t["m"]
    assert t["lo"][0] == 0 and t["hi"][0] == n and t["depth"][0] == 0
    covered = np.zeros(n, np.int32)
    for c in range(m):
        ch = t["child"][c][t["child"][c] >= 0]
        if t["leaf"][c]:
            assert len(ch) == 0
            covered[t["lo"][c]:t["hi"][c]] += 1
            assert t["hi"][c] - t["lo"][c] <= 8 or t["depth"][c] == 16
        else:
            assert t["hi"][c] - t["lo"][c] > 8 and len(ch) >= 1
            assert t["lo"][ch[0]] == t["lo"][c] and t["hi"][ch[-1]] == t["hi"][c]
            assert all(t["hi"][a] == t["lo"][b] for a, b in zip(ch[:-1], ch[1:]))
            assert all(t["depth"][k] == t["depth"][c] + 1 for k in ch)
            cnt = (t["hi"][ch] - t["lo"][ch]).astype(np.float64)
            com = (t["com"][ch].astype(np.float64) * cnt[:, None]).sum(0) / cnt.sum()
            assert np.allclose(com, t["com"][c], rtol=1e-5, atol=1e-6)
        # every member lies inside the cell's square
        side = float(t["root"][2]) * 2.0 ** (-int(t["depth"][c]))
        pts = t["Ys"][t["lo"][c]:t["hi"][c]].astype(np.float64)
        span = pts.max(0) - pts.min(0)
        assert span.max() <= side * (1 + 1e-6)
    assert np.all(covered == 1)


def test_non_finite_is_rejected():
    Y = np.zeros((4, 2), np.float32)
    Y[2, 1] = np.nan
    with pytest.raises(ValueError):
        oracle.morton(Y)


def test_deep_grid_splits_what_16_levels_cannot():
    """Clumps much smaller than 2^-16 of the extent: at 16 levels their members share deepest cells, at 22 they
    are split down to the leaf size."""
    rng = np.random.default_rng(2)
    Y = (np.repeat(rng.random((30, 2)) * 40.0, 200, axis=0) + 1e-4 * rng.standard_normal((6000, 2))).astype(np.float32)
    a = oracle.tree(Y, bits=16, leaf_cap=8)
    b = oracle.tree(Y, bits=22, leaf_cap=8)
    size_a = (a["hi"] - a["lo"])[a["leaf"] == 1]
    size_b = (b["hi"] - b["lo"])[b["leaf"] == 1]
    assert size_a.max() > 50 and size_b.max() <= 8
    assert b["depth"].max() > 16
    # the first 16 levels are the same tree: same cells above depth 16, same order of the points up to ties
    top = a["depth"] < 16
    topb = b["depth"] < 16
    assert np.array_equal(a["lo"][top], b["lo"][topb]) and np.array_equal(a["hi"][top], b["hi"][topb])
    assert np.array_equal(b["sorted_keys"] >> np.uint64(12), a["sorted_keys"])


def test_rank_for_equal_keys_only_moves_points_inside_their_runs():
    """Sec. III-C step 4 does not say how points with equal keys are ordered.  The default (by index) and a caller's
    rank must give the same keys and cells; only the members of a run of equal keys change places, as the rank says.
    With theta = 0 nothing is approximated, so the forces do not depend on that order either."""
    rng = np.random.default_rng(3)
    n = 3000
    Y = np.repeat(rng.standard_normal((n // 5, 2)).astype(np.float32), 5, axis=0)      # every point five times
    Y[::7] += rng.standard_normal((len(Y[::7]), 2)).astype(np.float32) * 1e-3           # and some near copies
    a = oracle.tree(Y, bits=12, leaf_cap=4)
    assert len(np.unique(a["keys"])) < n
    same = oracle.tree(Y, bits=12, leaf_cap=4, tie_rank=np.arange(n))
    for f in ("perm", "depth", "lo", "hi", "leaf", "com"):
        assert np.array_equal(a[f], same[f]), f
    rank = rng.permutation(n).astype(np.int32)
    b = oracle.tree(Y, bits=12, leaf_cap=4, tie_rank=rank)
    for f in ("sorted_keys", "depth", "lo", "hi", "leaf"):
        assert np.array_equal(a[f], b[f]), f
    assert not np.array_equal(a["perm"], b["perm"])
    assert np.array_equal(np.sort(b["perm"]), np.arange(n))
    sk = a["sorted_keys"]
    ends = np.flatnonzero(np.r_[True, sk[1:] != sk[:-1], True])
    for s, e in zip(ends[:-1], ends[1:]):
        assert sorted(a["perm"][s:e]) == sorted(b["perm"][s:e])          # the same points share the run
        assert np.all(np.diff(rank[b["perm"][s:e]]) > 0)                  # in the order of the rank
        assert np.all(np.diff(a["perm"][s:e]) > 0)                        # by index without one
    # centres of mass: the same points summed in another order
    assert np.abs(a["com"].astype(np.float64) - b["com"]).max() <= 1e-6 * float(a["root"][2])
    r0 = oracle.repulse_bh(Y, theta=0.0, leaf_cap=4, bits=12)
    r1 = oracle.repulse_bh(Y, theta=0.0, leaf_cap=4, bits=12, tie_rank=rank)
    assert np.abs(r0["R"] - r1["R"]).max() <= 1e-12 * np.abs(r0["R"]).max()
    assert abs(r0["Z"] - r1["Z"]) <= 1e-12 * r0["Z"]
