"""GPU parity of packed variable-length batches against the oracle (oracle.moba_forward_varlen /
attn_varlen: every sequence the operator on its own, ragged last block).  The library pads the
batch to whole blocks (moba_varlen_pad), takes each query's routing candidates from its own
sequence (moba_topk_varlen) and runs the ordinary centroid, forward and backward calls on the
padded tensors; results come back through moba_varlen_unpad."""
import numpy as np
import pytest
import torch

import paper_2511_11571_amd as moba
from paper_2511_11571_amd import binding
from tests import parity

pytestmark = pytest.mark.gpu

#         name           heads kv   d   B   k   dtype   sequence lengths
CASES = [("mixed_B32",      2,  0,  64, 32,  4, "bf16", [130, 64, 5, 257, 300, 244]),
         ("short_seqs_B64", 3,  0,  64, 64,  3, "bf16", [63, 1, 64, 65, 700, 129, 20]),
         ("d128_gqa",       4,  2, 128, 32,  5, "bf16", [500, 333, 1000]),
         ("f32_B16",        2,  0,  64, 16,  6, "f32",  [100, 17, 48, 260]),
         ("one_long_k20",   1,  0,  64, 32, 20, "bf16", [2049, 700]),
         ("empty_and_tiny", 2,  0,  64, 32,  2, "bf16", [0, 3, 0, 40, 96])]
FLAGS = [pytest.param(0, id="default"), pytest.param(binding.FLAG_REFERENCE_KERNELS, id="plain"),
         pytest.param(binding.FLAG_KEY_MAJOR, id="keymajor")]


def f64(x):
    a = x.detach().float().cpu().to(torch.float64).numpy()
    return a.reshape((a.shape[0] * a.shape[1],) + a.shape[2:])


@pytest.mark.parametrize("flags", FLAGS)
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_packed_variable_length_batch(oracle, case, flags):
    name, heads, kv, d, B, k, dtype, lens = case
    hkv = kv if kv else heads
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(offs[-1])
    g = torch.Generator().manual_seed(5000 + len(name))
    Q, dO = (torch.randn((1, heads, T, d), generator=g).to(dt) for _ in range(2))
    K, V = (torch.randn((1, hkv, T, d), generator=g).to(dt) for _ in range(2))
    scale = 1.0 / np.sqrt(d)

    lay = moba.VarlenLayout(offs, B)
    Tp = lay.padded_tokens
    assert Tp == sum(-(-L // B) * B for L in lens)
    sh = moba.Shape(1, heads, Tp, d, B, k, 0, binding.BF16 if dtype == "bf16" else binding.F32, 0.0, flags, kv)
    Qp, Kp, Vp, dOp = (lay.pad(x.cuda()) for x in (Q, K, V, dO))
    assert torch.equal(lay.unpad(Qp).cpu(), Q)                     # the two copies are inverse to each other
    _, cent = moba.centroids(sh, Kp)
    idx, lists = moba.topk_varlen(sh, lay, Qp, cent)

    # ---- routing against the oracle, sequence by sequence (block numbers inside the sequence)
    Q64, K64, V64, dO64 = f64(Q), f64(K), f64(V), f64(dO)
    Ke, Ve = (oracle.gqa_expand(x, heads, hkv) for x in (K64, V64))
    ref = oracle.moba_forward_varlen(Q64, Ke, Ve, offs, B, k, scale)
    got = lay.unpad(idx).cpu().numpy().reshape(heads, T, k)
    first = np.zeros(T, np.int64)
    for i in range(len(lens)):
        first[offs[i]:offs[i + 1]] = lay.pad_offsets_host[i] // B
    local = np.where(got >= 0, got - first[None, :, None], -1).astype(np.int32)
    exempt_rows = 0
    for i, L in enumerate(lens):
        if L == 0:
            continue
        lo, hi = offs[i], offs[i + 1]
        Lp = -(-L // B) * B
        qpad = np.zeros((heads, Lp, d)); qpad[:, :L] = Q64[:, lo:hi]
        kpad = np.zeros((heads, Lp, d)); kpad[:, :L] = Ke[:, lo:hi]
        C = oracle.centroids(kpad, B)
        rows = (np.arange(heads)[:, None] * Lp + np.arange(L)[None, :]).ravel().astype(np.int64)
        ridx, kth = oracle.topk(qpad, C, B, k, rows=rows)
        assert np.array_equal(np.sort(ridx.reshape(heads, L, k), -1), np.sort(ref["idx"][:, lo:hi], -1))
        exact, frac = parity.routing_check(oracle, local[:, lo:hi].reshape(heads * L, k), ridx, kth, qpad, C, B,
                                           rows=rows)
        exempt_rows += int(round(frac * heads * L))
    assert exempt_rows <= 0.02 * heads * T + 1

    # ---- attention and gradients at the ORACLE's routing (every row comparable)
    gidx = np.where(ref["idx"] >= 0, ref["idx"] + first[None, :, None], -1).astype(np.int32)
    gidx_p = torch.full((1, heads, Tp, k), -1, dtype=torch.int32)
    for i in range(len(lens)):                                     # padded queries keep nothing
        gidx_p[0, :, lay.pad_offsets_host[i]:lay.pad_offsets_host[i] + lens[i]] = torch.from_numpy(
            gidx[:, offs[i]:offs[i + 1]])
    # a query keeps exactly min(candidates, k) blocks: give the padded rows a valid routing too
    bf = lay.block_first.cpu().numpy()
    for i, L in enumerate(lens):
        p0 = lay.pad_offsets_host[i]
        for p in range(p0 + L, p0 + -(-L // B) * B):
            c = p // B
            n_keep = min(k, c - int(bf[c]))
            gidx_p[0, :, p, :n_keep] = torch.arange(int(bf[c]), int(bf[c]) + n_keep, dtype=torch.int32)
    gidx_p = gidx_p.cuda()
    rlists = moba.build_lists(sh, gidx_p)
    O, lse = moba.forward(sh, Qp, Kp, Vp, gidx_p, rlists)
    dQ, dK, dV = moba.backward(sh, Qp, Kp, Vp, O, lse, dOp, gidx_p, rlists)
    rO, rlse, rQ, rK, rV = oracle.attn_varlen(Q64, Ke, Ve, ref["idx"], dO64, offs, B, scale)
    rK, rV = (oracle.gqa_reduce(x, heads, hkv) for x in (rK, rV))
    assert parity.max_abs(f64(lay.unpad(O)), rO) < parity.O_TOL[dtype]
    assert parity.max_abs(lay.unpad(lse).double().cpu().numpy().reshape(heads, T), rlse) < parity.LSE_TOL[dtype]
    for a, b in ((dQ, rQ), (dK, rK), (dV, rV)):
        assert parity.rel_l2(f64(lay.unpad(a)), b) < parity.GRAD_TOL[dtype]
    # padding rows receive nothing
    pad_rows = np.ones(Tp, bool)
    for i, L in enumerate(lens):
        pad_rows[lay.pad_offsets_host[i]:lay.pad_offsets_host[i] + L] = False
    if pad_rows.any():
        sel = torch.from_numpy(pad_rows).cuda()
        assert float(dK[0, :, sel].abs().max()) == 0.0 and float(dV[0, :, sel].abs().max()) == 0.0


def test_varlen_layout_rejects_bad_offsets():
    import ctypes
    L = moba.lib()
    po = (ctypes.c_int32 * 4)()
    tp = ctypes.c_int32(0)
    bad = (ctypes.c_int32 * 4)(0, 10, 5, 20)                       # not ascending
    assert L.moba_varlen_layout(3, bad, 32, po, ctypes.byref(tp)) == -1
    nz = (ctypes.c_int32 * 4)(1, 10, 15, 20)                       # does not start at 0
    assert L.moba_varlen_layout(3, nz, 32, po, ctypes.byref(tp)) == -1
    ok = (ctypes.c_int32 * 4)(0, 10, 15, 80)
    assert L.moba_varlen_layout(3, ok, 32, po, ctypes.byref(tp)) == 0
    assert list(po) == [0, 32, 64, 160] and tp.value == 160
