"""GPU parity on seeded random shapes: every case draws head dim, block size, number of blocks,
top-k (from 0 to beyond the number of past blocks), head sharing, batch, I/O type and key-conv
width, and runs the whole chain with each choice of kernels (default pick, plain kernels, key-block
major forced, query tiles forced) against the oracle: centroids, routing under the gap rule, lists
bit-exact and, at the oracle's routing, outputs, lse and all three gradients.  The shapes reach
block sizes and ragged tile tails that the hand-picked workloads do not (B = 1 ... 512, a single
block, a sequence shorter than a tile)."""
import numpy as np
import pytest
import torch

import paper_2511_11571_amd as moba
import workloads
from paper_2511_11571_amd import binding
from tests import parity
from tests.test_gpu_parity import dev, np64, npi, oracle_inputs, shape_of, to_io

pytestmark = pytest.mark.gpu

KERNELS = [pytest.param(0, id="default"), pytest.param(binding.FLAG_REFERENCE_KERNELS, id="plain"),
           pytest.param(binding.FLAG_KEY_MAJOR, id="keymajor"), pytest.param(binding.FLAG_QUERY_TILES, id="tiles")]


def draw(case):
    rng = np.random.default_rng(8800 + case)
    d = int(rng.choice([64, 128]))
    B = int(rng.choice([1, 8, 24, 32, 64, 96, 128, 160, 256, 384, 512]))
    n = int(rng.integers(1, min(48, max(2, 2560 // B)) + 1))
    k = int(rng.integers(0, min(n + 2, 24)))
    heads = int(rng.choice([1, 2, 4]))
    kv = int(rng.choice([h for h in (1, 2, 4) if heads % h == 0]))
    return workloads.Workload(
        "random%d_d%d_B%d_n%d_k%d" % (case, d, B, n, k), int(rng.choice([1, 2])), heads, B * n, d, B, k,
        backward=True, seed=8800 + case, kv_heads=0 if kv == heads else kv,
        dtype="f32" if rng.random() < 0.2 else "bf16",
        conv_width=int(rng.integers(1, 9)) if rng.random() < 0.3 else 0)


CASES = [draw(c) for c in range(20)]


@pytest.mark.parametrize("flags", KERNELS)
@pytest.mark.parametrize("w", CASES, ids=[w.name for w in CASES])
def test_random_shape(oracle, w, flags):
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    C = oracle.centroids(Kp, w.B)
    Ke, Ve, Ce = (oracle.gqa_expand(x, w.heads, w.hkv) for x in (Kp, V, C))
    ref_idx, kth = oracle.topk(Q, Ce, w.B, w.k)
    sh = shape_of(w, flags)
    d = dev(t)
    Keff, cent = moba.centroids(sh, d["K"], d["conv_w"])
    assert parity.max_abs(np64(cent), C) < (2e-6 if not w.conv_width else 2e-3)
    cent_ref = torch.from_numpy(C).float().reshape(w.batch, w.hkv, w.n, w.d).cuda()
    got_idx, _ = moba.topk(sh, d["Q"], cent_ref)
    parity.routing_check(oracle, npi(got_idx).reshape(w.bh * w.N, w.k), ref_idx.reshape(w.bh * w.N, w.k),
                         kth.reshape(-1), Q, Ce, w.B)
    # attention at the oracle's routing
    idx = torch.from_numpy(ref_idx).reshape(w.batch, w.heads, w.N, w.k).cuda()
    lists = moba.build_lists(sh, idx)
    r_off, r_ql = oracle.csr(ref_idx, w.B)
    parity.check_lists(npi(lists[0]), npi(lists[1]), ref_idx, r_off, r_ql, w.k)
    Kdev = to_io(w, Kp, t["K"])
    O, lse = moba.forward(sh, d["Q"], Kdev, d["V"], idx, lists)
    rO, rlse = oracle.attn_fwd(Q, Ke, Ve, ref_idx, w.B, w.scale)
    assert parity.max_abs(np64(O), rO) < parity.O_TOL[w.dtype]
    assert parity.max_abs(np64(lse), rlse) < parity.LSE_TOL[w.dtype]
    dQ, dK, dV = moba.backward(sh, d["Q"], Kdev, d["V"], O, lse, d["dO"], idx, lists)
    rQ, rKe, rVe = oracle.attn_bwd(Q, Ke, Ve, ref_idx, dO, w.B, w.scale)
    tol = parity.GRAD_TOL[w.dtype]
    for name, got, ref in (("dQ", dQ, rQ), ("dK", dK, oracle.gqa_reduce(rKe, w.heads, w.hkv)),
                           ("dV", dV, oracle.gqa_reduce(rVe, w.heads, w.hkv))):
        ref_norm = float(np.linalg.norm(ref))
        # a gradient that is exactly zero (a query alone with its own key): absolute bound
        err = parity.rel_l2(np64(got), ref) if ref_norm > 1e-6 else parity.max_abs(np64(got), ref)
        assert err < tol, (name, err)
