"""GPU parity of the decode-shaped forward (moba_decode_forward) against the oracle.

The oracle knows only whole sequences whose length is a multiple of the block.  A decode call
covers the last q_len positions of N keys, N arbitrary: the oracle is run on the sequence
padded with zero rows to the next multiple of B and evaluated on those positions only -- a
query never sees keys after itself, and the centroid of its own (possibly ragged) block is
never a candidate, so the padding cannot reach the result.  Where N is a multiple of B the
same rows are also compared with moba_forward on the whole sequence."""
import numpy as np
import pytest
import torch

import paper_2511_11571_amd as moba
from paper_2511_11571_amd import binding
from tests import parity

pytestmark = pytest.mark.gpu

#        name             batch heads kv    N    d    B   k  q_len dtype
CASES = [("bf16_ragged",      1,   4,  0, 1000,  64,  32,  4,   5, "bf16"),
         ("bf16_one_query",   2,   2,  0, 4133,  64, 128,  8,   1, "bf16"),
         ("f32_d128",         1,   2,  0,  777, 128,  64,  3,   7, "f32"),
         ("gqa_ragged",       1,   8,  2, 2050,  64,  64,  6,  16, "bf16"),
         ("mqa_d128",         2,   4,  1, 1500, 128,  32,  5,   3, "bf16"),
         ("all_in_block_0",   1,   2,  0,   20,  64,  32,  4,  20, "bf16"),
         ("aligned",          1,   2,  0, 1024,  64,  32,  4,  64, "bf16"),
         ("k0",               1,   2,  0,  300,  64,  32,  0,   3, "bf16"),
         ("k64_of_128",       1,   1,  0, 4113,  64,  32, 64,   4, "bf16"),
         ("k_ge_past",        1,   1,  0,  200,  64,  32, 100,  8, "f32"),
         ("B1",               1,   1,  0,  300,  64,   1,  7,   2, "f32")]


def make(batch, heads, kv, N, d, dtype, seed, q_len):
    g = torch.Generator().manual_seed(seed)
    hkv = kv if kv else heads
    dt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Q = torch.randn((batch, heads, q_len, d), generator=g).to(dt)
    K = torch.randn((batch, hkv, N, d), generator=g).to(dt)
    V = torch.randn((batch, hkv, N, d), generator=g).to(dt)
    return Q, K, V


def f64(x):
    a = x.detach().cpu().to(torch.float64).numpy()
    return a.reshape((a.shape[0] * a.shape[1],) + a.shape[2:])


def oracle_decode(oracle, Q, K, V, heads, hkv, N, B, k, q_len, scale):
    """-> (idx [bh*q_len, k], kth, O [bh*q_len, d], lse, rows, Qfull, Ce) from the padded sequence."""
    Np = -(-N // B) * B
    Q64, K64, V64 = f64(Q), f64(K), f64(V)
    bh, bhk, d = Q64.shape[0], K64.shape[0], Q64.shape[2]
    Kp = np.zeros((bhk, Np, d))
    Vp = np.zeros((bhk, Np, d))
    Kp[:, :N], Vp[:, :N] = K64, V64
    Qf = np.zeros((bh, Np, d))
    Qf[:, N - q_len:N] = Q64
    C = oracle.centroids(Kp, B)
    Ke, Ve, Ce = (oracle.gqa_expand(x, heads, hkv) for x in (Kp, Vp, C))
    rows = (np.arange(bh)[:, None] * Np + np.arange(N - q_len, N)[None, :]).ravel().astype(np.int64)
    idx, kth = oracle.topk(Qf, Ce, B, k, rows=rows)
    idx_full = np.full((bh, Np, k), -1, np.int32)
    idx_full.reshape(bh * Np, k)[rows] = idx
    O, lse = oracle.attn_fwd(Qf, Ke, Ve, idx_full, B, scale, rows=rows)
    return idx, kth, O, lse, rows, Qf, Ce, C


def random_case(i):
    """Seeded random decode shapes: any sequence length (ragged own block), any top-k from 0 to
    beyond the number of past blocks, shared heads, both I/O types."""
    rng = np.random.default_rng(9900 + i)
    d = int(rng.choice([64, 128]))
    B = int(rng.choice([1, 8, 24, 32, 64, 128, 200]))
    N = int(rng.integers(1, 40 * B + 1))
    heads = int(rng.choice([1, 2, 4]))
    kv = int(rng.choice([h for h in (1, 2, 4) if heads % h == 0]))
    k = int(rng.integers(0, min((N - 1) // B + 3, 20)))
    q_len = int(rng.integers(1, min(N, 24) + 1))
    return ("random%d_N%d_B%d_k%d_q%d" % (i, N, B, k, q_len), int(rng.choice([1, 2])), heads,
            0 if kv == heads else kv, N, d, B, k, q_len, "f32" if rng.random() < 0.3 else "bf16")


CASES = CASES + [random_case(i) for i in range(16)]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_decode_forward(oracle, case):
    name, batch, heads, kv, N, d, B, k, q_len, dtype = case
    hkv = kv if kv else heads
    Q, K, V = make(batch, heads, kv, N, d, dtype, 500 + len(name), q_len)
    scale = 1.0 / np.sqrt(d)
    ridx, kth, rO, rlse, rows, Qf, Ce, C = oracle_decode(oracle, Q, K, V, heads, hkv, N, B, k, q_len, scale)
    sh = moba.Shape(batch, heads, N, d, B, k, 0, binding.BF16 if dtype == "bf16" else binding.F32, 0.0, 0, kv)
    npast = (N - 1) // B
    # the caller's centroid cache: the complete blocks (here with two spare rows of capacity)
    cent = torch.zeros((batch, hkv, npast + 2, d), dtype=torch.float32)
    cent[:, :, :npast] = torch.from_numpy(C[:, :npast]).float().reshape(batch, hkv, npast, d)
    O, lse, idx = moba.decode_forward(sh, q_len, Q.cuda(), K.cuda(), V.cuda(), cent.cuda())
    got = idx.cpu().numpy().reshape(batch * heads * q_len, k)
    # kept blocks ascending, unused slots at the end
    srt = np.where(got < 0, np.iinfo(np.int32).max, got)
    assert (np.diff(srt, axis=-1) >= 0).all()
    exact, exempt = parity.routing_check(oracle, got, ridx, kth, Qf, Ce, B, rows=rows)
    assert exempt < 0.2
    gO = f64(O).reshape(-1, d)
    glse = lse.double().cpu().numpy().reshape(-1)
    assert np.abs(gO - rO)[exact].max() < parity.O_TOL[dtype]
    assert np.abs(glse - rlse)[exact].max() < parity.LSE_TOL[dtype]
    if N % B == 0 and hkv == heads:
        # the same rows through the training-shaped path on the whole sequence
        g = torch.Generator().manual_seed(1)
        Qall = torch.randn((batch, heads, N, d), generator=g).to(Q.dtype)
        Qall[:, :, N - q_len:] = Q
        cent_all = torch.from_numpy(C).float().reshape(batch, hkv, N // B, d).cuda()
        idx_all, lists = moba.topk(sh, Qall.cuda(), cent_all)
        O_all, lse_all = moba.forward(sh, Qall.cuda(), K.cuda(), V.cuda(), idx_all, lists)
        same = (np.sort(idx_all[:, :, N - q_len:].cpu().numpy().reshape(got.shape), -1) == np.sort(got, -1)).all(-1)
        a = f64(O_all[:, :, N - q_len:]).reshape(-1, d)
        assert np.abs(a - gO)[same].max() < 2 * parity.O_TOL[dtype]


def test_decode_ties_go_to_the_lower_block():
    """All keys zero: every gate score is 0, so the kept blocks are 0 .. k-1, and the output is the
    mean of the attended values."""
    batch, heads, N, d, B, k, q_len = 1, 2, 1000, 64, 32, 5, 3
    g = torch.Generator().manual_seed(3)
    Q = torch.randn((batch, heads, q_len, d), generator=g).to(torch.bfloat16)
    K = torch.zeros((batch, heads, N, d), dtype=torch.bfloat16)
    V = torch.randn((batch, heads, N, d), generator=g).to(torch.bfloat16)
    npast = (N - 1) // B
    cent = torch.zeros((batch, heads, npast, d), dtype=torch.float32)
    sh = moba.Shape(batch, heads, N, d, B, k, 0, binding.BF16)
    O, lse, idx = moba.decode_forward(sh, q_len, Q.cuda(), K.cuda(), V.cuda(), cent.cuda())
    assert (idx.cpu().numpy() == np.arange(k)).all()
    for r in range(q_len):
        t = N - q_len + r
        keys = list(range(k * B)) + list(range((t // B) * B, t + 1))
        ref = V[0, :, keys].double().mean(1)
        assert (O[0, :, r].double().cpu() - ref).abs().max() < 2e-2
        assert abs(float(lse[0, 0, r]) - np.log(len(keys))) < 1e-4


def test_decode_argument_checks():
    sh = moba.Shape(1, 2, 1000, 64, 32, 4, 0, binding.BF16)
    Q = torch.zeros((1, 2, 4, 64), dtype=torch.bfloat16).cuda()
    K = torch.zeros((1, 2, 1000, 64), dtype=torch.bfloat16).cuda()
    few = torch.zeros((1, 2, 5, 64), dtype=torch.float32).cuda()          # needs 31 centroid rows
    with pytest.raises(moba.MobaError):
        moba.decode_forward(sh, 4, Q, K, K, few)
    with pytest.raises(moba.MobaError):
        moba.decode_forward(sh, 4, Q, K, K, None)
