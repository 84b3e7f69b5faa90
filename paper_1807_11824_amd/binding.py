"""ctypes binding of include/tsne.h.  Argument marshalling only: torch supplies device memory
and the stream, every step of the method runs inside libtsne_hip.so.

There is no CPU fallback: if the library is missing, loading fails loudly.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtsne_hip.so")

STATUS_NONFINITE = 1
STATUS_CELL_OVERFLOW = 2
STATUS_WALK_OVERFLOW = 4


class TsneError(RuntimeError):
    def __init__(self, code, what, detail=""):
        self.code = code
        super().__init__(f"{what}: {code} {detail}")


class TsneParams(C.Structure):
    _fields_ = [("n", C.c_int32), ("theta", C.c_float), ("lr", C.c_float), ("exaggeration", C.c_float),
                ("exaggeration_iters", C.c_int32), ("momentum_early", C.c_float), ("momentum_late", C.c_float),
                ("momentum_switch_iter", C.c_int32), ("gain_inc", C.c_float), ("gain_dec", C.c_float),
                ("gain_min", C.c_float), ("morton_bits", C.c_int32), ("leaf_cap", C.c_int32),
                ("overlap", C.c_int32), ("graph_order_iters", C.c_int32), ("reorder_every", C.c_int32),
                ("attract_resident", C.c_int32), ("walk_resident", C.c_int32),
                ("far_tiles", C.c_int32), ("max_nnz", C.c_int64)]


_lib = None


def lib():
    """Loads libtsne_hip.so (building it first if the file is absent)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _b
        _b.build()
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    PP = C.POINTER(TsneParams)
    sig = {
        "tsne_default_params": (C.c_int, [PP, i32]),
        "tsne_workspace_bytes": (C.c_int, [PP, C.POINTER(C.c_size_t)]),
        "tsne_create": (C.c_int, [C.POINTER(vp), PP, vp, vp, C.c_size_t]),
        "tsne_destroy": (None, [vp]),
        "tsne_build_P_workspace_bytes": (C.c_int, [i32, i32, i32, C.POINTER(C.c_size_t)]),
        "tsne_build_P": (C.c_int, [vp, i32, i32, f32, i32, vp, vp, vp, i64, C.POINTER(i64), vp, vp,
                                   C.POINTER(i32), vp, C.c_size_t, vp]),
        "tsne_ivf_workspace_bytes": (C.c_int, [i32, i32, i32, i32, i32, C.POINTER(C.c_size_t)]),
        "tsne_ivf_train": (C.c_int, [vp, i32, i32, i32, i32, vp, vp, C.c_size_t, vp]),
        "tsne_ivf_knn": (C.c_int, [vp, i32, i32, vp, i32, i32, i32, vp, vp, vp, C.c_size_t, vp]),
        "tsne_ivfpq_workspace_bytes": (C.c_int, [i32, i32, i32, i32, i32, i32, i32, C.POINTER(C.c_size_t)]),
        "tsne_ivfpq_train": (C.c_int, [vp, i32, i32, vp, i32, i32, i32, i32, vp, vp, C.c_size_t, vp]),
        "tsne_ivfpq_knn": (C.c_int, [vp, i32, i32, vp, i32, vp, i32, i32, i32, i32, vp, vp, vp, C.c_size_t, vp]),
        "tsne_build_P_approx_workspace_bytes": (C.c_int, [i32, i32, i32, i32, i32, i32, C.POINTER(C.c_size_t)]),
        "tsne_build_P_approx": (C.c_int, [vp, i32, i32, f32, i32, i32, i32, i32, i32, vp, vp, vp, i64, C.POINTER(i64), vp, vp,
                                          C.POINTER(i32), C.POINTER(i32), vp, C.c_size_t, vp]),
        "tsne_set_P": (C.c_int, [vp, vp, vp, vp, i64]),
        "tsne_P_layout": (C.c_int, [vp, C.POINTER(i64), C.POINTER(i64)]),
        "tsne_init_state": (C.c_int, [vp]),
        "tsne_get_state": (C.c_int, [vp, vp, vp]),
        "tsne_set_state": (C.c_int, [vp, vp, vp]),
        "tsne_step": (C.c_int, [vp, vp, i32]),
        "tsne_run": (C.c_int, [vp, vp, i32, i32]),
        "tsne_gradient": (C.c_int, [vp, vp, vp, vp, vp]),
        "tsne_export_tree": (C.c_int, [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, C.POINTER(i32)]),
        "tsne_kl": (C.c_int, [vp, vp, C.POINTER(C.c_double)]),
        "tsne_kl_static": (C.c_int, [vp, i32, vp, vp, vp, vp, vp]),
        "tsne_status": (C.c_int, [vp, C.POINTER(C.c_uint32)]),
        "tsne_timing_begin": (C.c_int, [vp, i32]),
        "tsne_timing_begin_every": (C.c_int, [vp, i32, i32]),
        "tsne_timing_end": (C.c_int, [vp, C.POINTER(i32), C.POINTER(C.c_float)]),
        "tsne_strerror": (C.c_char_p, [C.c_int]),
        "tsne_last_error": (C.c_char_p, [vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dev(t, dtype, what):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{what}: need a contiguous {dtype} CUDA tensor")
    return t


def default_params(n, **kw):
    p = TsneParams()
    rc = lib().tsne_default_params(C.byref(p), n)
    if rc:
        raise TsneError(rc, "tsne_default_params")
    for k, v in kw.items():
        if not hasattr(p, k):
            raise AttributeError(k)
        setattr(p, k, v)
    return p


def build_P_workspace_bytes(n, d, k):
    b = C.c_size_t(0)
    rc = lib().tsne_build_P_workspace_bytes(n, d, k, C.byref(b))
    if rc:
        raise TsneError(rc, "tsne_build_P_workspace_bytes", lib().tsne_strerror(rc).decode())
    return b.value


def build_P(X, perplexity, k, stream=None, want_knn=False):
    """tsne_build_P on a device tensor X (n x d float32).  Returns a dict of device tensors."""
    _dev(X, torch.float32, "X")
    n, d = X.shape
    L = lib()
    wb = build_P_workspace_bytes(n, d, k)
    work = torch.empty(wb, dtype=torch.uint8, device=X.device)
    cap = 2 * n * k
    row_ptr = torch.empty(n + 1, dtype=torch.int32, device=X.device)
    col = torch.empty(cap, dtype=torch.int32, device=X.device)
    val = torch.empty(cap, dtype=torch.float32, device=X.device)
    knn_idx = torch.empty((n, k), dtype=torch.int32, device=X.device) if want_knn else None
    knn_d2 = torch.empty((n, k), dtype=torch.float32, device=X.device) if want_knn else None
    nnz = C.c_int64(0)
    bad = C.c_int32(0)
    rc = L.tsne_build_P(_ptr(X), n, d, perplexity, k, _ptr(row_ptr), _ptr(col), _ptr(val), cap, C.byref(nnz),
                        _ptr(knn_idx), _ptr(knn_d2), C.byref(bad), _ptr(work), wb, _stream_ptr(stream))
    if rc:
        raise TsneError(rc, "tsne_build_P", L.tsne_strerror(rc).decode())
    m = nnz.value
    return dict(row_ptr=row_ptr, col=col[:m], val=val[:m], nnz=m, unconverged=bad.value,
                knn_idx=knn_idx, knn_d2=knn_d2)


def _ivf_workspace(n, d, k, nlist, tau, device, extra_bytes=0):
    b = C.c_size_t(0)
    rc = lib().tsne_ivf_workspace_bytes(n, d, k, nlist, tau, C.byref(b))
    if rc:
        raise TsneError(rc, "tsne_ivf_workspace_bytes", lib().tsne_strerror(rc).decode())
    return torch.empty(b.value + extra_bytes, dtype=torch.uint8, device=device)


def ivf_train(X, nlist, iters, stream=None):
    """tsne_ivf_train on a device tensor X (n x d float32): the nlist x d centroids (device float32)."""
    _dev(X, torch.float32, "X")
    n, d = X.shape
    L = lib()
    work = _ivf_workspace(n, d, 1, nlist, 1, X.device)
    cent = torch.empty((nlist, d), dtype=torch.float32, device=X.device)
    rc = L.tsne_ivf_train(_ptr(X), n, d, nlist, iters, _ptr(cent), _ptr(work), work.numel(), _stream_ptr(stream))
    if rc:
        raise TsneError(rc, "tsne_ivf_train", L.tsne_strerror(rc).decode())
    return cent


def ivf_knn(X, centroids, tau, k, stream=None, extra_workspace_bytes=0):
    """tsne_ivf_knn: (idx int32 n x k, squared distances float64 n x k), device tensors."""
    _dev(X, torch.float32, "X")
    _dev(centroids, torch.float32, "centroids")
    n, d = X.shape
    nlist = centroids.shape[0]
    if centroids.shape[1] != d:
        raise ValueError("centroids: wrong width")
    L = lib()
    work = _ivf_workspace(n, d, k, nlist, tau, X.device, extra_workspace_bytes)
    idx = torch.empty((n, k), dtype=torch.int32, device=X.device)
    d2 = torch.empty((n, k), dtype=torch.float64, device=X.device)
    rc = L.tsne_ivf_knn(_ptr(X), n, d, _ptr(centroids), nlist, tau, k, _ptr(idx), _ptr(d2), _ptr(work), work.numel(),
                        _stream_ptr(stream))
    if rc:
        raise TsneError(rc, "tsne_ivf_knn", L.tsne_strerror(rc).decode())
    return idx, d2


def _ivfpq_workspace(n, d, k, nlist, tau, m, ksub, device):
    b = C.c_size_t(0)
    rc = lib().tsne_ivfpq_workspace_bytes(n, d, k, nlist, tau, m, ksub, C.byref(b))
    if rc:
        raise TsneError(rc, "tsne_ivfpq_workspace_bytes", lib().tsne_strerror(rc).decode())
    return torch.empty(b.value, dtype=torch.uint8, device=device)


def ivfpq_train(X, centroids, m, ksub, iters, stream=None):
    """tsne_ivfpq_train: the m x ksub x (d / m) codebooks of the product quantiser (device float32)."""
    _dev(X, torch.float32, "X"); _dev(centroids, torch.float32, "centroids")
    n, d = X.shape
    L = lib()
    work = _ivfpq_workspace(n, d, 1, centroids.shape[0], 1, m, ksub, X.device)
    cb = torch.empty((m, ksub, d // max(m, 1)), dtype=torch.float32, device=X.device)
    rc = L.tsne_ivfpq_train(_ptr(X), n, d, _ptr(centroids), centroids.shape[0], m, ksub, iters, _ptr(cb), _ptr(work),
                            work.numel(), _stream_ptr(stream))
    if rc:
        raise TsneError(rc, "tsne_ivfpq_train", L.tsne_strerror(rc).decode())
    return cb


def ivfpq_knn(X, centroids, codebooks, tau, k, stream=None):
    """tsne_ivfpq_knn: (idx int32 n x k, distances to the codes float64 n x k), device tensors."""
    _dev(X, torch.float32, "X"); _dev(centroids, torch.float32, "centroids"); _dev(codebooks, torch.float32, "codebooks")
    n, d = X.shape
    m, ksub, ds = codebooks.shape
    if m * ds != d or centroids.shape[1] != d:
        raise ValueError("codebooks / centroids: wrong shape")
    L = lib()
    nlist = centroids.shape[0]
    work = _ivfpq_workspace(n, d, k, nlist, tau, m, ksub, X.device)
    idx = torch.empty((n, k), dtype=torch.int32, device=X.device)
    d2 = torch.empty((n, k), dtype=torch.float64, device=X.device)
    rc = L.tsne_ivfpq_knn(_ptr(X), n, d, _ptr(centroids), nlist, _ptr(codebooks), m, ksub, tau, k, _ptr(idx), _ptr(d2),
                          _ptr(work), work.numel(), _stream_ptr(stream))
    if rc:
        raise TsneError(rc, "tsne_ivfpq_knn", L.tsne_strerror(rc).decode())
    return idx, d2


def build_P_approx(X, perplexity, k, tau, nlist=0, kmeans_iters=10, stream=None, want_knn=False, pq_m=0):
    """tsne_build_P_approx on a device tensor X (n x d float32); pq_m > 0: product-quantised second stage with
    pq_m sub-vectors.  Returns a dict of device tensors."""
    _dev(X, torch.float32, "X")
    n, d = X.shape
    L = lib()
    b = C.c_size_t(0)
    rc = L.tsne_build_P_approx_workspace_bytes(n, d, k, nlist, tau, pq_m, C.byref(b))
    if rc:
        raise TsneError(rc, "tsne_build_P_approx_workspace_bytes", L.tsne_strerror(rc).decode())
    work = torch.empty(b.value, dtype=torch.uint8, device=X.device)
    cap = 2 * n * k
    row_ptr = torch.empty(n + 1, dtype=torch.int32, device=X.device)
    col = torch.empty(cap, dtype=torch.int32, device=X.device)
    val = torch.empty(cap, dtype=torch.float32, device=X.device)
    knn_idx = torch.empty((n, k), dtype=torch.int32, device=X.device) if want_knn else None
    knn_d2 = torch.empty((n, k), dtype=torch.float32, device=X.device) if want_knn else None
    nnz = C.c_int64(0)
    bad = C.c_int32(0)
    used = C.c_int32(0)
    rc = L.tsne_build_P_approx(_ptr(X), n, d, perplexity, k, nlist, tau, kmeans_iters, pq_m, _ptr(row_ptr), _ptr(col),
                               _ptr(val), cap, C.byref(nnz), _ptr(knn_idx), _ptr(knn_d2), C.byref(bad), C.byref(used),
                               _ptr(work), b.value, _stream_ptr(stream))
    if rc:
        raise TsneError(rc, "tsne_build_P_approx", L.tsne_strerror(rc).decode())
    m = nnz.value
    return dict(row_ptr=row_ptr, col=col[:m], val=val[:m], nnz=m, unconverged=bad.value,
                knn_idx=knn_idx, knn_d2=knn_d2, tau_used=used.value)


def kl_static(Y, row_ptr, col, val, out, stream=None):
    """tsne_kl_static: KL(P||Q) and the exact Z into the caller's device tensor `out` (2 doubles).  Enqueues only;
    allocates nothing."""
    _dev(Y, torch.float32, "Y"); _dev(row_ptr, torch.int32, "row_ptr"); _dev(out, torch.float64, "out")
    if out.numel() < 2:
        raise ValueError("out: need two doubles")
    L = lib()
    rc = L.tsne_kl_static(_ptr(Y), Y.shape[0], _ptr(row_ptr), _ptr(col), _ptr(val), _ptr(out), _stream_ptr(stream))
    if rc:
        raise TsneError(rc, "tsne_kl_static", L.tsne_strerror(rc).decode())


class Tsne:
    """One optimisation context (tsne_create ... tsne_destroy) with its torch-owned workspace."""

    def __init__(self, n, device="cuda:0", stream=None, **params):
        self.L = lib()
        self.params = default_params(n, **params)
        self.n = n
        self.device = torch.device(device)
        b = C.c_size_t(0)
        rc = self.L.tsne_workspace_bytes(C.byref(self.params), C.byref(b))
        if rc:
            raise TsneError(rc, "tsne_workspace_bytes", self.L.tsne_strerror(rc).decode())
        self.workspace = torch.empty(b.value, dtype=torch.uint8, device=self.device)
        self.stream = stream
        self._ctx = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = self.L.tsne_create(C.byref(self._ctx), C.byref(self.params), _stream_ptr(stream),
                                    _ptr(self.workspace), b.value)
        if rc:
            raise TsneError(rc, "tsne_create", self.L.tsne_strerror(rc).decode())
        self._P = None

    def _check(self, rc, what):
        if rc:
            raise TsneError(rc, what, self.L.tsne_last_error(self._ctx).decode())

    def close(self):
        if getattr(self, "_ctx", None):
            self.L.tsne_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_P(self, row_ptr, col, val):
        _dev(row_ptr, torch.int32, "row_ptr"); _dev(col, torch.int32, "col"); _dev(val, torch.float32, "val")
        if row_ptr.numel() != self.n + 1 or col.numel() != val.numel():
            raise ValueError("CSR arrays do not fit n")
        self._P = (row_ptr, col, val)            # keep the borrowed arrays alive
        self._check(self.L.tsne_set_P(self._ctx, _ptr(row_ptr), _ptr(col), _ptr(val), col.numel()), "tsne_set_P")

    def P_layout(self):
        near, far = C.c_int64(0), C.c_int64(0)
        self._check(self.L.tsne_P_layout(self._ctx, C.byref(near), C.byref(far)), "tsne_P_layout")
        return near.value, far.value

    def init_state(self):
        self._check(self.L.tsne_init_state(self._ctx), "tsne_init_state")

    def get_state(self):
        u = torch.empty((self.n, 2), dtype=torch.float32, device=self.device)
        g = torch.empty((self.n, 2), dtype=torch.float32, device=self.device)
        self._check(self.L.tsne_get_state(self._ctx, _ptr(u), _ptr(g)), "tsne_get_state")
        return u, g

    def set_state(self, u, g):
        _dev(u, torch.float32, "velocity"); _dev(g, torch.float32, "gains")
        self._check(self.L.tsne_set_state(self._ctx, _ptr(u), _ptr(g)), "tsne_set_state")

    def step(self, Y, it):
        _dev(Y, torch.float32, "Y")
        self._check(self.L.tsne_step(self._ctx, _ptr(Y), it), "tsne_step")

    def run(self, Y, n_iter, iter0=0):
        _dev(Y, torch.float32, "Y")
        self._check(self.L.tsne_run(self._ctx, _ptr(Y), iter0, n_iter), "tsne_run")
        return Y

    def gradient(self, Y):
        _dev(Y, torch.float32, "Y")
        A = torch.empty((self.n, 2), dtype=torch.float32, device=self.device)
        R = torch.empty((self.n, 2), dtype=torch.float32, device=self.device)
        Z = torch.empty(1, dtype=torch.float64, device=self.device)
        self._check(self.L.tsne_gradient(self._ctx, _ptr(Y), _ptr(A), _ptr(R), _ptr(Z)), "tsne_gradient")
        return A, R, Z

    def export_tree(self, cap_cells=None):
        n = self.n
        cap = cap_cells if cap_cells is not None else n + self.params.morton_bits * (n // (self.params.leaf_cap + 1)) + 1
        dev = self.device
        keys = torch.empty(n, dtype=torch.int64, device=dev)
        perm = torch.empty(n, dtype=torch.int32, device=dev)
        depth = torch.empty(cap, dtype=torch.int32, device=dev)
        lo = torch.empty(cap, dtype=torch.int32, device=dev)
        hi = torch.empty(cap, dtype=torch.int32, device=dev)
        leaf = torch.empty(cap, dtype=torch.int32, device=dev)
        com = torch.empty((cap, 2), dtype=torch.float32, device=dev)
        root = torch.empty(3, dtype=torch.float32, device=dev)
        m = C.c_int32(0)
        self._check(self.L.tsne_export_tree(self._ctx, _ptr(keys), _ptr(perm), cap, _ptr(depth), _ptr(lo), _ptr(hi),
                                            _ptr(leaf), _ptr(com), _ptr(root), C.byref(m)), "tsne_export_tree")
        m = m.value
        return dict(keys=keys, perm=perm, m=m, depth=depth[:m], lo=lo[:m], hi=hi[:m], leaf=leaf[:m], com=com[:m],
                    root=root)

    def n_cells(self):
        """Cell count of the last tree (tsne_export_tree with no arrays)."""
        m = C.c_int32(0)
        self._check(self.L.tsne_export_tree(self._ctx, None, None, 0, None, None, None, None, None, None, C.byref(m)),
                    "tsne_export_tree")
        return m.value

    def kl(self, Y):
        _dev(Y, torch.float32, "Y")
        v = C.c_double(0)
        self._check(self.L.tsne_kl(self._ctx, _ptr(Y), C.byref(v)), "tsne_kl")
        return v.value

    def timing_begin(self, max_steps, every=1):
        self._check(self.L.tsne_timing_begin_every(self._ctx, max_steps, every), "tsne_timing_begin_every")

    def timing_end(self):
        steps = C.c_int32(0)
        ms = (C.c_float * 4)()
        self._check(self.L.tsne_timing_end(self._ctx, C.byref(steps), ms), "tsne_timing_end")
        return dict(steps=steps.value, tree_ms=ms[0], walk_ms=ms[1], attract_ms=ms[2], update_ms=ms[3])

    def status(self):
        s = C.c_uint32(0)
        self._check(self.L.tsne_status(self._ctx, C.byref(s)), "tsne_status")
        return s.value
