"""CPU-side checks of the C ABI: the library loads, exports what include/tsne.h declares, and
validates arguments on the host before touching the GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_1807_11824_amd import binding
    return binding.lib()


def _declared():
    src = open(os.path.join(ROOT, "include", "tsne.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(tsne_[a-z_A-Z]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(L):
    names = _declared()
    assert "tsne_build_P" in names and "tsne_step" in names and "tsne_run" in names
    for name in names:
        assert hasattr(L, name), name


def test_binding_covers_the_header(L):
    from paper_1807_11824_amd import binding
    src = open(binding.__file__).read()
    for name in _declared():
        assert f'"{name}"' in src, name


def test_strerror(L):
    assert L.tsne_strerror(0) == b"ok"
    for code in range(-5, 0):
        assert L.tsne_strerror(code) not in (b"ok", b"unknown error")
    assert L.tsne_strerror(-99) == b"unknown error"


def test_host_side_validation(L):
    from paper_1807_11824_amd.binding import TsneParams
    p = TsneParams()
    assert L.tsne_default_params(C.byref(p), 1000) == 0
    assert (p.n, p.morton_bits, p.leaf_cap, p.exaggeration_iters) == (1000, 22, 8, 250)
    assert abs(p.theta - 0.5) < 1e-7 and p.lr == 200.0 and p.exaggeration == 12.0
    b = C.c_size_t(0)
    assert L.tsne_workspace_bytes(C.byref(p), C.byref(b)) == 0 and b.value > 1000 * 100
    small = b.value
    p.n = 2000
    assert L.tsne_workspace_bytes(C.byref(p), C.byref(b)) == 0 and b.value > small
    for field, bad in (("n", 0), ("theta", 0.8), ("theta", -0.1), ("theta", float("nan")), ("morton_bits", 25),
                       ("morton_bits", 0), ("leaf_cap", 0), ("lr", float("inf"))):
        q = TsneParams()
        L.tsne_default_params(C.byref(q), 1000)
        setattr(q, field, bad)
        assert L.tsne_workspace_bytes(C.byref(q), C.byref(b)) == -1, (field, bad)
        ctx = C.c_void_p()
        assert L.tsne_create(C.byref(ctx), C.byref(q), None, C.c_void_p(256), 1 << 40) == -1
        assert not ctx.value
    # the grid key and the point's number share a 64-bit word: 2 bits + ceil(log2 n) <= 64
    q = TsneParams()
    L.tsne_default_params(C.byref(q), 1281167)
    assert q.morton_bits == 21 and L.tsne_workspace_bytes(C.byref(q), C.byref(b)) == 0
    q.morton_bits = 22
    assert L.tsne_workspace_bytes(C.byref(q), C.byref(b)) == -1
    L.tsne_default_params(C.byref(q), 1 << 20)
    assert q.morton_bits == 22
    L.tsne_default_params(C.byref(q), 1 << 27)
    assert q.morton_bits == 18 and L.tsne_workspace_bytes(C.byref(q), C.byref(b)) == 0
    L.tsne_default_params(C.byref(q), (1 << 27) + 1)      # more points than one launch axis holds at 16 lanes each
    assert L.tsne_workspace_bytes(C.byref(q), C.byref(b)) == -1
    # the call for callers that cannot allocate refuses sizes beyond its limit before touching the GPU
    assert L.tsne_kl_static(C.c_void_p(256), (1 << 22) + 1, C.c_void_p(256), None, None, C.c_void_p(256), None) == -1
    assert L.tsne_kl_static(C.c_void_p(256), 0, C.c_void_p(256), None, None, C.c_void_p(256), None) == -1
    # null / misaligned / too small workspace
    q = TsneParams()
    L.tsne_default_params(C.byref(q), 1000)
    ctx = C.c_void_p()
    assert L.tsne_create(C.byref(ctx), C.byref(q), None, None, 1 << 40) == -1
    assert L.tsne_create(C.byref(ctx), C.byref(q), None, C.c_void_p(128), 1 << 40) == -1
    assert L.tsne_create(C.byref(ctx), C.byref(q), None, C.c_void_p(256), 1024) == -2
    # null contexts
    assert L.tsne_step(None, None, 0) == -1
    assert L.tsne_run(None, None, 0, 1) == -1
    assert L.tsne_set_P(None, None, None, None, 0) == -1
    assert L.tsne_last_error(None) == b""


def test_build_P_validation(L):
    b = C.c_size_t(0)
    assert L.tsne_build_P_workspace_bytes(2000, 50, 90, C.byref(b)) == 0 and b.value > 0
    assert L.tsne_build_P_workspace_bytes(10, 4, 10, C.byref(b)) == -1      # k >= n
    assert L.tsne_build_P_workspace_bytes(1, 4, 1, C.byref(b)) == -1
    assert L.tsne_build_P_workspace_bytes(100, 0, 5, C.byref(b)) == -1
    nnz = C.c_int64(0)
    one = C.c_void_p(256)
    # perplexity out of range, null pointers, workspace too small: all refused before any launch
    assert L.tsne_build_P(one, 100, 8, 0.0, 10, one, one, one, 2000, C.byref(nnz), None, None, None, one, 1 << 40, None) == -1
    assert L.tsne_build_P(one, 100, 8, 11.0, 10, one, one, one, 2000, C.byref(nnz), None, None, None, one, 1 << 40, None) == -1
    assert L.tsne_build_P(None, 100, 8, 3.0, 10, one, one, one, 2000, C.byref(nnz), None, None, None, one, 1 << 40, None) == -1
    assert L.tsne_build_P(one, 100, 8, 3.0, 10, one, one, one, 2000, C.byref(nnz), None, None, None, one, 16, None) == -2
