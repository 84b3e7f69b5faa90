"""ctypes front end of oracle/tsne_oracle.c (test infrastructure only).

Argument marshalling and nothing else: every number is computed by the C file.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

__all__ = [
    "knn", "cond_p", "symmetrise", "build_P", "grad_exact", "attract", "kl", "morton", "sort_keys",
    "tree", "repulse_bh", "grad_bh", "update", "run", "RunParams", "threads",
]

_lib = None


def _L():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
        _lib.oracle_kl.restype = C.c_double
        _lib.oracle_symmetrise.restype = C.c_int64
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def threads():
    return int(_L().oracle_threads())


def knn(X, k, rows=None):
    X = _f32(X)
    n, d = X.shape
    if rows is not None:
        rows = _i32(rows)
        nq = rows.shape[0]
    else:
        nq = n
    idx = np.empty((nq, k), np.int32)
    d2 = np.empty((nq, k), np.float64)
    rc = _L().oracle_knn(_p(X, C.c_float), n, d, k, _p(rows, C.c_int32), nq,
                         _p(idx, C.c_int32), _p(d2, C.c_double))
    if rc != 0:
        raise ValueError("oracle_knn: bad arguments")
    return idx, d2


def cond_p(d2, perplexity, tol=1e-10):
    d2 = _f64(d2)
    n, k = d2.shape
    cond = np.empty((n, k), np.float64)
    beta = np.empty(n, np.float64)
    bad = _L().oracle_cond_p(_p(d2, C.c_double), n, k, C.c_double(perplexity), C.c_double(tol),
                             _p(cond, C.c_double), _p(beta, C.c_double))
    if bad < 0:
        raise ValueError("oracle_cond_p: bad arguments")
    return cond, beta, int(bad)


def symmetrise(idx, cond):
    idx = _i32(idx)
    cond = _f64(cond)
    n, k = idx.shape
    cap = 2 * n * k
    row_ptr = np.empty(n + 1, np.int32)
    col = np.empty(cap, np.int32)
    val = np.empty(cap, np.float64)
    nnz = _L().oracle_symmetrise(_p(idx, C.c_int32), _p(cond, C.c_double), n, k,
                                 _p(row_ptr, C.c_int32), _p(col, C.c_int32), _p(val, C.c_double),
                                 C.c_int64(cap))
    if nnz < 0:
        raise ValueError("oracle_symmetrise: bad arguments")
    return row_ptr, col[:nnz].copy(), val[:nnz].copy()


def build_P(X, perplexity, k):
    """kNN -> conditional P -> symmetric CSR, all in double."""
    idx, d2 = knn(X, k)
    cond, beta, bad = cond_p(d2, perplexity)
    row_ptr, col, val = symmetrise(idx, cond)
    return dict(idx=idx, d2=d2, cond=cond, beta=beta, unconverged=bad,
                row_ptr=row_ptr, col=col, val=val)


def grad_exact(Y, row_ptr, col, val, alpha=1.0):
    Y = _f64(Y)
    n = Y.shape[0]
    row_ptr, col, val = _i32(row_ptr), _i32(col), _f64(val)
    A = np.empty((n, 2)); R = np.empty((n, 2)); g = np.empty((n, 2))
    Z = C.c_double(0)
    _L().oracle_grad_exact(_p(Y, C.c_double), n, _p(row_ptr, C.c_int32), _p(col, C.c_int32),
                           _p(val, C.c_double), C.c_double(alpha), _p(A, C.c_double),
                           _p(R, C.c_double), C.byref(Z), _p(g, C.c_double))
    return dict(A=A, R=R, Z=Z.value, grad=g)


def attract(Y, row_ptr, col, val):
    Y = _f64(Y)
    n = Y.shape[0]
    row_ptr, col, val = _i32(row_ptr), _i32(col), _f64(val)
    A = np.empty((n, 2))
    _L().oracle_attract(_p(Y, C.c_double), n, _p(row_ptr, C.c_int32), _p(col, C.c_int32),
                        _p(val, C.c_double), _p(A, C.c_double))
    return A


def kl(Y, row_ptr, col, val):
    Y = _f64(Y)
    row_ptr, col, val = _i32(row_ptr), _i32(col), _f64(val)
    return float(_L().oracle_kl(_p(Y, C.c_double), Y.shape[0], _p(row_ptr, C.c_int32),
                                _p(col, C.c_int32), _p(val, C.c_double)))


def morton(Y, bits=16):
    Y = _f32(Y)
    n = Y.shape[0]
    root = np.empty(3, np.float32)
    keys = np.empty(n, np.uint64)
    rc = _L().oracle_morton(_p(Y, C.c_float), n, bits, _p(root, C.c_float), _p(keys, C.c_uint64))
    if rc != 0:
        raise ValueError("oracle_morton: bad arguments or non-finite coordinate")
    return root, keys


def _tie(tie_rank, n):
    """Rank that orders points of equal key (None: the original index)."""
    if tie_rank is None:
        return None, None
    t = _i32(tie_rank)
    if t.shape != (n,):
        raise ValueError("tie_rank: one rank per point")
    return t, _p(t, C.c_int32)


def sort_keys(keys, tie_rank=None):
    keys = np.ascontiguousarray(keys, np.uint64)
    n = keys.shape[0]
    sk = np.empty(n, np.uint64)
    perm = np.empty(n, np.int32)
    _keep, tp = _tie(tie_rank, n)
    if _L().oracle_sort_ties(_p(keys, C.c_uint64), n, tp, _p(sk, C.c_uint64), _p(perm, C.c_int32)) != 0:
        raise MemoryError
    return sk, perm


def tree(Y, bits=16, leaf_cap=8, tie_rank=None):
    """Bounding box, keys, sort and the quad tree (pre-order) with summaries."""
    Y = _f32(Y)
    n = Y.shape[0]
    root, keys = morton(Y, bits)
    sk, perm = sort_keys(keys, tie_rank)
    Ys = np.ascontiguousarray(Y[perm])
    cap = n * (bits + 1) + 1        # every level holds at most n cells
    depth = np.empty(cap, np.int32); lo = np.empty(cap, np.int32); hi = np.empty(cap, np.int32)
    leaf = np.empty(cap, np.int32); child = np.empty((cap, 4), np.int32)
    prefix = np.empty(cap, np.uint64); com = np.empty((cap, 2), np.float32)
    m = _L().oracle_tree(_p(sk, C.c_uint64), _p(Ys, C.c_float), n, bits, leaf_cap, cap,
                         _p(depth, C.c_int32), _p(prefix, C.c_uint64), _p(lo, C.c_int32),
                         _p(hi, C.c_int32), _p(leaf, C.c_int32), _p(child, C.c_int32),
                         _p(com, C.c_float))
    if m < 0:
        raise ValueError("oracle_tree: bad arguments or capacity exceeded")
    return dict(root=root, keys=keys, sorted_keys=sk, perm=perm, Ys=Ys, m=m,
                depth=depth[:m].copy(), prefix=prefix[:m].copy(), lo=lo[:m].copy(),
                hi=hi[:m].copy(), leaf=leaf[:m].copy(), child=child[:m].copy(), com=com[:m].copy())


def repulse_bh(Y, theta=0.5, leaf_cap=8, group=64, bits=16, tie_rank=None):
    Y = _f32(Y)
    n = Y.shape[0]
    R = np.empty((n, 2)); z = np.empty(n)
    Z = C.c_double(0)
    stats = np.zeros(3, np.int64)
    _keep, tp = _tie(tie_rank, n)
    m = _L().oracle_repulse_bh_ties(_p(Y, C.c_float), n, C.c_float(theta), leaf_cap, group, bits, tp,
                                    _p(R, C.c_double), _p(z, C.c_double), C.byref(Z),
                                    _p(stats, C.c_int64))
    if m < 0:
        raise ValueError("oracle_repulse_bh: bad arguments")
    return dict(R=R, z=z, Z=Z.value, n_cells=m, accepted=int(stats[0]), opened=int(stats[1]),
                point_terms=int(stats[2]))


def grad_bh(Y, row_ptr, col, val, theta=0.5, leaf_cap=8, group=64, bits=16, alpha=1.0, tie_rank=None):
    Y = _f32(Y)
    n = Y.shape[0]
    row_ptr, col, val = _i32(row_ptr), _i32(col), _f64(val)
    A = np.empty((n, 2)); R = np.empty((n, 2)); g = np.empty((n, 2))
    Z = C.c_double(0)
    stats = np.zeros(3, np.int64)
    _keep, tp = _tie(tie_rank, n)
    m = _L().oracle_grad_bh_ties(_p(Y, C.c_float), n, _p(row_ptr, C.c_int32), _p(col, C.c_int32),
                                 _p(val, C.c_double), C.c_float(theta), leaf_cap, group, bits, tp,
                                 C.c_double(alpha), _p(A, C.c_double), _p(R, C.c_double), C.byref(Z),
                                 _p(g, C.c_double), _p(stats, C.c_int64))
    if m < 0:
        raise ValueError("oracle_grad_bh: bad arguments")
    return dict(A=A, R=R, Z=Z.value, grad=g, n_cells=m, accepted=int(stats[0]),
                opened=int(stats[1]), point_terms=int(stats[2]))


def update(Y, uY, gains, grad, momentum, lr, gain_inc=0.2, gain_dec=0.8, gain_min=0.01):
    """In place on float64 arrays Y, uY, gains."""
    for a in (Y, uY, gains):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    grad = _f64(grad)
    _L().oracle_update(_p(Y, C.c_double), _p(uY, C.c_double), _p(gains, C.c_double),
                       _p(grad, C.c_double), Y.shape[0], C.c_double(momentum), C.c_double(lr),
                       C.c_double(gain_inc), C.c_double(gain_dec), C.c_double(gain_min))


class RunParams(C.Structure):
    _fields_ = [("theta", C.c_float), ("leaf_cap", C.c_int32), ("group", C.c_int32),
                ("bits", C.c_int32), ("lr", C.c_double), ("exaggeration", C.c_double),
                ("exaggeration_iters", C.c_int32), ("momentum_early", C.c_double),
                ("momentum_late", C.c_double), ("momentum_switch_iter", C.c_int32),
                ("gain_inc", C.c_double), ("gain_dec", C.c_double), ("gain_min", C.c_double)]

    @classmethod
    def default(cls, **kw):
        p = cls(theta=0.5, leaf_cap=8, group=64, bits=16, lr=200.0, exaggeration=12.0,
                exaggeration_iters=250, momentum_early=0.5, momentum_late=0.8,
                momentum_switch_iter=250, gain_inc=0.2, gain_dec=0.8, gain_min=0.01)
        for k, v in kw.items():
            setattr(p, k, v)
        return p


def run(Y0, row_ptr, col, val, params, n_iter, iter0=0, state=None):
    """Alg. 1 lines 3-9.  Returns (Y, uY, gains) as float64 arrays."""
    Y = _f64(Y0).copy()
    n = Y.shape[0]
    if state is None:
        uY = np.zeros((n, 2)); gains = np.ones((n, 2))
    else:
        uY, gains = (_f64(s).copy() for s in state)
    row_ptr, col, val = _i32(row_ptr), _i32(col), _f64(val)
    rc = _L().oracle_run(_p(Y, C.c_double), _p(uY, C.c_double), _p(gains, C.c_double), n,
                         _p(row_ptr, C.c_int32), _p(col, C.c_int32), _p(val, C.c_double),
                         C.byref(params), iter0, n_iter)
    if rc != 0:
        raise RuntimeError("oracle_run failed")
    return Y, uY, gains
