"""The entry point that allocates nothing (moba_topk_static) against moba_topk, through the C ABI:
two calls in a row on one GPU, the second with a smaller input, so that what the first call left
in the library's static scratch must not reach the second call's result."""
import pytest
import torch

import paper_2511_11571_amd as moba
import workloads
from paper_2511_11571_amd import binding

pytestmark = pytest.mark.gpu

W = workloads.Workload


def _case(w):
    t = workloads.generate(w)
    sh = moba.Shape(w.batch, w.heads, w.N, w.d, w.B, w.k, 0, binding.BF16)
    Q, K = t["Q"].cuda(), t["K"].cuda()
    _, cent = moba.centroids(sh, K)
    return sh, Q, cent


def test_static_scratch_topk_matches_the_workspace_call():
    big = _case(W("static_big", 1, 4, 4096, 64, 32, 16, seed=71))
    small = _case(W("static_small", 1, 2, 1344, 64, 32, 5, seed=72))      # 1344 = 10.5 chunks of 128
    assert moba.workspace_bytes(big[0])[0] > moba.workspace_bytes(small[0])[0]
    for sh, Q, cent in (big, small):
        want_idx, (want_off, want_ql) = moba.topk(sh, Q, cent)
        # outputs allocated here, poisoned, so that the call under test allocates and keeps nothing
        idx = torch.full_like(want_idx, -7)
        off = torch.full_like(want_off, -7)
        ql = torch.full_like(want_ql, -7)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        moba.topk_static(sh, Q, cent, out=(idx, (off, ql)))
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(idx, want_idx)          # integer results: bit-exact
        assert torch.equal(off, want_off)
        assert torch.equal(ql, want_ql)


def test_static_scratch_rejects_oversized_shapes():
    """Host-side check: a shape whose workspace exceeds the static array is refused before any launch."""
    import ctypes
    sh = moba.Shape(2, 16, 131072, 64, 32, 8, 0, binding.BF16)
    assert moba.workspace_bytes(sh)[0] > (32 << 20)
    one = ctypes.c_void_p(256)                     # never dereferenced on this path
    st = moba.lib().moba_topk_static(ctypes.byref(sh.c()), one, one, one, one, one, None)
    assert st == -3
