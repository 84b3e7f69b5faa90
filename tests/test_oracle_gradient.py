"""Pins for the oracle's gradient code: what the paper and the mathematics fix.

CPU only.  A plausible slip in oracle/tsne_oracle.c (a dropped Z, a sign, a
transposed index, a missing factor 4) fails at least one test here.
"""
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _dense(P, n):
    D = np.zeros((n, n))
    for i in range(n):
        D[i, P["col"][P["row_ptr"][i]:P["row_ptr"][i + 1]]] = P["val"][P["row_ptr"][i]:P["row_ptr"][i + 1]]
    return D


def _kl_numpy(Y, Pd):
    """KL(P||Q) written from Eq. (2) and (4) with dense numpy arrays."""
    d2 = ((Y[:, None, :] - Y[None, :, :]) ** 2).sum(-1)
    W = 1.0 / (1.0 + d2)
    np.fill_diagonal(W, 0.0)
    Q = W / W.sum()
    m = Pd > 0
    return float((Pd[m] * np.log(Pd[m] / Q[m])).sum())


def test_kl_matches_dense_definition(small_problem):
    P, Y = small_problem["P"], small_problem["Y"].astype(np.float64)
    got = oracle.kl(Y, P["row_ptr"], P["col"], P["val"])
    want = _kl_numpy(Y, _dense(P, Y.shape[0]))
    assert abs(got - want) <= 1e-12 * abs(want)


def test_exact_gradient_is_gradient_of_kl():
    """Eq. (3)/(7) is stated as dC/dy_i: central differences of KL, N = 48, double."""
    from paper_1807_11824_amd import synth
    X, _ = synth.config1(n=48, d=50, seed=1)
    P = oracle.build_P(X, 5.0, 15)
    rng = np.random.default_rng(0)
    Y = rng.standard_normal((48, 2)) * 2.0
    g = oracle.grad_exact(Y, P["row_ptr"], P["col"], P["val"])["grad"]
    Pd = _dense(P, 48)
    h = 1e-5
    fd = np.zeros_like(Y)
    for i in range(48):
        for c in range(2):
            Yp = Y.copy(); Yp[i, c] += h
            Ym = Y.copy(); Ym[i, c] -= h
            fd[i, c] = (_kl_numpy(Yp, Pd) - _kl_numpy(Ym, Pd)) / (2 * h)
    assert np.linalg.norm(g - fd) <= 1e-6 * np.linalg.norm(fd)


def test_force_decomposition_matches_eq3(small_problem):
    """4 sum_j (p_ij - q_ij) q_ij Z (y_i - y_j) computed densely equals 4 (A - R/Z)."""
    P, Y = small_problem["P"], small_problem["Y"].astype(np.float64)
    n = Y.shape[0]
    Pd = _dense(P, n)
    diff = Y[:, None, :] - Y[None, :, :]
    W = 1.0 / (1.0 + (diff ** 2).sum(-1))
    np.fill_diagonal(W, 0.0)
    Z = W.sum()
    want = 4.0 * (((Pd - W / Z) * W)[:, :, None] * diff).sum(1)
    r = oracle.grad_exact(Y, P["row_ptr"], P["col"], P["val"])
    assert abs(r["Z"] - Z) <= 1e-12 * Z
    assert np.linalg.norm(r["grad"] - want) <= 1e-12 * np.linalg.norm(want)
    # exaggeration multiplies the attractive term only
    r12 = oracle.grad_exact(Y, P["row_ptr"], P["col"], P["val"], alpha=12.0)
    # (compared in the norm: single components of 12 A - R / Z cancel almost completely, and the oracle's
    #  Z is a parallel sum whose last bits depend on the thread schedule)
    want12 = 4.0 * (12.0 * r["A"] - r["R"] / Z)
    assert np.linalg.norm(r12["grad"] - want12) <= 1e-12 * np.linalg.norm(want12)


def test_net_force_is_zero(small_problem):
    P, Y = small_problem["P"], small_problem["Y"].astype(np.float64)
    r = oracle.grad_exact(Y, P["row_ptr"], P["col"], P["val"])
    for F in (r["A"], r["R"]):
        assert np.abs(F.sum(0)).max() <= 1e-12 * np.abs(F).sum()


def _golden_closed_forms():
    out = {}
    with open(os.path.join(HERE, "golden", "closed_forms.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, _q, v = line.split()
            out[name] = float(v)
    return out


def test_closed_forms_for_Z():
    gold = _golden_closed_forms()
    empty = (np.zeros(3, np.int32), np.zeros(0, np.int32), np.zeros(0))
    # two points, symmetric P = 1/2 each way: gradient vanishes identically
    Y = np.array([[0.0, 0.0], [3.0, 0.0]])
    rp, col, val = np.array([0, 1, 2], np.int32), np.array([1, 0], np.int32), np.array([0.5, 0.5])
    r = oracle.grad_exact(Y, rp, col, val)
    assert abs(r["Z"] - gold["two_points_d=3"]) < 1e-15
    assert np.abs(r["grad"]).max() < 1e-15
    # coincident points
    Y = np.ones((7, 2)) * 0.3
    rp = np.zeros(8, np.int32)
    r = oracle.grad_exact(Y, rp, empty[1], empty[2])
    assert r["Z"] == gold["coincident_n=7"]
    assert np.abs(r["R"]).max() == 0.0
    b = oracle.repulse_bh(Y.astype(np.float32), theta=0.5, leaf_cap=2, group=4)
    assert b["Z"] == gold["coincident_n=7"] and np.abs(b["R"]).max() == 0.0
    # three collinear points
    Y = np.array([[0.0, 0.0], [1.0, 0.0], [2.0, 0.0]])
    r = oracle.grad_exact(Y, np.zeros(4, np.int32), empty[1], empty[2])
    assert abs(r["Z"] - gold["collinear_0_1_2"]) < 1e-15
    # R_0 = w01^2 (0-1) + w02^2 (0-2) = -(1/4) - 2/25
    assert abs(r["R"][0, 0] + 0.25 + 0.08) < 1e-15 and abs(r["R"][1, 0]) < 1e-15


@pytest.mark.parametrize("leaf_cap,group", [(1, 1), (4, 1), (8, 64), (3, 7), (1000, 64)])
def test_bh_theta0_equals_exact(small_problem, leaf_cap, group):
    """theta = 0 gives the O(N^2) algorithm (Sec. III-C), for any leaf size and grouping."""
    P, Y = small_problem["P"], small_problem["Y"]
    ex = oracle.grad_exact(Y.astype(np.float64), P["row_ptr"], P["col"], P["val"], alpha=12.0)
    bh = oracle.grad_bh(Y, P["row_ptr"], P["col"], P["val"], theta=0.0, leaf_cap=leaf_cap,
                        group=group, alpha=12.0)
    assert bh["accepted"] == 0
    assert abs(bh["Z"] - ex["Z"]) <= 1e-12 * ex["Z"]
    assert np.linalg.norm(bh["R"] - ex["R"]) <= 1e-12 * np.linalg.norm(ex["R"])
    assert np.linalg.norm(bh["grad"] - ex["grad"]) <= 1e-12 * np.linalg.norm(ex["grad"])


def test_bh_error_shrinks_with_theta_and_is_second_order(small_problem):
    """Eq. (15): a far cell stands in for its points with an error of order (r/d)^2 <= theta^2."""
    Y = small_problem["Y"]
    P = small_problem["P"]
    ex = oracle.grad_exact(Y.astype(np.float64), P["row_ptr"], P["col"], P["val"])
    errs = []
    for th in (0.1, 0.2, 0.4, 0.6):
        bh = oracle.repulse_bh(Y, theta=th, leaf_cap=1, group=1)
        assert bh["accepted"] > 0
        errs.append(np.linalg.norm(bh["R"] - ex["R"]) / np.linalg.norm(ex["R"]))
        assert abs(bh["Z"] - ex["Z"]) / ex["Z"] <= th * th
        assert errs[-1] <= th * th
    assert errs[0] < errs[1] < errs[2] < errs[3]


def test_bh_single_far_cluster_summary():
    """One tight cluster far from a probe: summary force vs direct sum, relative error ~ (r/d)^2."""
    rng = np.random.default_rng(2)
    cl = (rng.random((50, 2)) * 0.1 + np.array([10.0, 10.0])).astype(np.float32)
    Y = np.vstack([np.zeros((1, 2), np.float32), cl])
    d = Y[1:].astype(np.float64) - Y[0].astype(np.float64)
    w = 1.0 / (1.0 + (d ** 2).sum(1))
    direct = -(w[:, None] ** 2 * d).sum(0)          # R_0 = sum w^2 (y_0 - y_j)
    bh = oracle.repulse_bh(Y, theta=0.5, leaf_cap=1, group=1)
    rel = np.linalg.norm(bh["R"][0] - direct) / np.linalg.norm(direct)
    assert 0 < rel < (0.15 / 14.0) ** 2 * 10
    # the grouped walk takes the same decisions for all members of a group, and a larger
    # group can only accept fewer cells
    a1 = oracle.repulse_bh(Y, theta=0.5, leaf_cap=1, group=1)["accepted"]
    a64 = oracle.repulse_bh(Y, theta=0.5, leaf_cap=1, group=64)["accepted"]
    assert a64 <= a1


def test_grouped_walk_is_at_least_as_accurate(small_problem):
    Y, P = small_problem["Y"], small_problem["P"]
    ex = oracle.grad_exact(Y.astype(np.float64), P["row_ptr"], P["col"], P["val"])
    e1 = np.linalg.norm(oracle.repulse_bh(Y, 0.5, 4, 1)["R"] - ex["R"])
    e64 = np.linalg.norm(oracle.repulse_bh(Y, 0.5, 4, 64)["R"] - ex["R"])
    assert e64 <= e1 * 1.05


def test_bh_net_repulsion_small(small_problem):
    Y = small_problem["Y"]
    bh = oracle.repulse_bh(Y, theta=0.5, leaf_cap=8, group=64)
    assert np.abs(bh["R"].sum(0)).max() <= 2e-2 * np.abs(bh["R"]).sum()


def test_update_matches_hand_trace():
    rows = []
    with open(os.path.join(HERE, "golden", "update_trace.txt")) as f:
        for line in f:
            if not line.startswith("#") and line.strip():
                rows.append([float(v) for v in line.split()])
    Y = np.zeros((1, 2)); uY = np.zeros((1, 2)); gains = np.ones((1, 2))
    for _it, g, gain, vel, y in rows:
        oracle.update(Y, uY, gains, np.array([[g, -g]]), momentum=0.5, lr=200.0)
        assert abs(gains[0, 0] - gain) < 1e-12 and abs(uY[0, 0] - vel) < 1e-12 and abs(Y[0, 0] - y) < 1e-12
        # the mirrored coordinate follows the mirrored trace
        assert abs(uY[0, 1] + vel) < 1e-12 and abs(Y[0, 1] + y) < 1e-12
    # floor of the gain
    gains[:] = 0.011
    uY[:] = 1.0
    oracle.update(Y, uY, gains, np.array([[1.0, 1.0]]), momentum=0.5, lr=200.0)
    assert gains[0, 0] == 0.01


def test_run_resume_is_bitwise(small_problem):
    P, Y0 = small_problem["P"], small_problem["Y"] * 1e-3
    pr = oracle.RunParams.default(exaggeration_iters=5, momentum_switch_iter=5, leaf_cap=4)
    full = oracle.run(Y0, P["row_ptr"], P["col"], P["val"], pr, 10)
    a = oracle.run(Y0, P["row_ptr"], P["col"], P["val"], pr, 4)
    b = oracle.run(a[0], P["row_ptr"], P["col"], P["val"], pr, 6, iter0=4, state=(a[1], a[2]))
    for u, v in zip(full, b):
        assert np.array_equal(u, v)


def test_run_lowers_kl(small_problem):
    """A converged Barnes-Hut run ends at the KL of a converged exact run (trajectories are
    chaotic, so only the end value is compared, and only after enough iterations)."""
    P, Y0 = small_problem["P"], small_problem["Y"] * 1e-3
    pr = oracle.RunParams.default(exaggeration_iters=100, momentum_switch_iter=100)
    kl0 = oracle.kl(Y0, P["row_ptr"], P["col"], P["val"])
    Y, _, _ = oracle.run(Y0, P["row_ptr"], P["col"], P["val"], pr, 800)
    kl1 = oracle.kl(Y, P["row_ptr"], P["col"], P["val"])
    pr0 = oracle.RunParams.default(exaggeration_iters=100, momentum_switch_iter=100, theta=0.0)
    Ye, _, _ = oracle.run(Y0, P["row_ptr"], P["col"], P["val"], pr0, 800)
    kle = oracle.kl(Ye, P["row_ptr"], P["col"], P["val"])
    assert kl1 < 0.5 * kl0
    assert abs(kl1 - kle) <= 0.08 * kle
