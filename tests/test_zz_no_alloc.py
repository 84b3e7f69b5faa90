"""tsne_kl_static (the entry point for callers that cannot allocate) against tsne_kl, through the C ABI."""
import ctypes as C

import numpy as np
import pytest

from paper_1807_11824_amd import synth
from helpers import random_symmetric_csr

pytestmark = pytest.mark.gpu


def _both(n, seed, out):
    """KL and Z of one (P, Y) from tsne_kl (context, workspace) and from tsne_kl_static (no context)."""
    import torch
    from paper_1807_11824_amd import Tsne, lib
    dev = torch.device("cuda:0")
    rp, col, val = random_symmetric_csr(n, 12, seed=seed)
    P = [torch.from_numpy(a).to(dev) for a in (rp, col, val)]
    Y = torch.from_numpy(synth.clustered_embedding(n, n_clusters=25, seed=seed)).to(dev)
    t = Tsne(n)
    t.set_P(*P)
    want = t.kl(Y)
    t.close()
    L = lib()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = L.tsne_kl_static(C.c_void_p(Y.data_ptr()), n, C.c_void_p(P[0].data_ptr()), C.c_void_p(P[1].data_ptr()),
                          C.c_void_p(P[2].data_ptr()), C.c_void_p(out.data_ptr()), stream)
    assert rc == 0
    torch.cuda.synchronize()
    got = out.cpu().numpy().copy()
    return want, got


def test_static_kl_equals_context_kl_twice_second_smaller():
    import torch
    out = torch.full((2,), -1.0, dtype=torch.float64, device="cuda:0")
    for n, seed in ((20_011, 3), (1_501, 4)):      # the second call is smaller and sees the first call's leftovers
        want, got = _both(n, seed, out)
        print(f"n={n}: tsne_kl {want!r}  tsne_kl_static {got[0]!r}  Z {got[1]!r}", flush=True)
        assert np.isfinite(got).all() and got[1] > 0
        assert abs(got[0] - want) <= 1e-12 * abs(want)       # same kernels, same order of additions


def test_static_kl_rejects_bad_sizes():
    import torch
    from paper_1807_11824_amd import lib
    L = lib()
    out = torch.zeros(2, dtype=torch.float64, device="cuda:0")
    Y = torch.zeros((4, 2), dtype=torch.float32, device="cuda:0")
    rp = torch.zeros(5, dtype=torch.int32, device="cuda:0")
    args = (C.c_void_p(rp.data_ptr()), None, None, C.c_void_p(out.data_ptr()), None)
    assert L.tsne_kl_static(C.c_void_p(Y.data_ptr()), (1 << 22) + 1, *args) == -1
    assert L.tsne_kl_static(C.c_void_p(Y.data_ptr()), 0, *args) == -1
    assert L.tsne_kl_static(None, 4, *args) == -1
