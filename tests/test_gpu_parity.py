"""GPU parity: every stage of the library, called through the C ABI, against the CPU
oracle on the same seeded inputs.  Sizes here are ones the oracle finishes in
seconds while still spanning several tiles, ragged query chunks and the degenerate
cases; the benchmark-size checks live in test_gpu_full_size.py."""
import numpy as np
import pytest
import torch

import paper_2511_11571_amd as moba
import workloads
from paper_2511_11571_amd import binding
from tests import parity

pytestmark = pytest.mark.gpu

REF = binding.FLAG_REFERENCE_KERNELS
FLAGS = [pytest.param(0, id="default"), pytest.param(REF, id="plain")]
# attention kernels also exist in two cuts, query tiles and key-block major: force each
ATTN_FLAGS = FLAGS + [pytest.param(binding.FLAG_KEY_MAJOR, id="keymajor"),
                      pytest.param(binding.FLAG_QUERY_TILES, id="tiles")]


def shape_of(w, flags=0):
    return moba.Shape(w.batch, w.heads, w.N, w.d, w.B, w.k, w.conv_width,
                      binding.BF16 if w.dtype == "bf16" else binding.F32, 0.0, flags, w.kv_heads)


def dev(t):
    return {k: (v.cuda() if v is not None else None) for k, v in t.items()}


def np64(x):
    a = x.detach().float().cpu().to(torch.float64).numpy()
    return a.reshape((a.shape[0] * a.shape[1],) + a.shape[2:])


def npi(x):
    a = x.detach().cpu().numpy()
    return a.reshape((a.shape[0] * a.shape[1],) + a.shape[2:])


def oracle_inputs(orc, w, t):
    Q, K, V, dO = (workloads.to_f64(t[x]) for x in ("Q", "K", "V", "dO"))
    mode = orc.ROUND_BF16 if w.dtype == "bf16" else orc.ROUND_F32
    Kp = K
    if w.conv_width:
        Kp = orc.key_conv(K, t["conv_w"].double().numpy(), w.hkv, mode)
    return Q, K, Kp, V, dO


def to_io(w, a64, like):
    """Oracle array [bh, ...] -> device tensor [b, h, ...] in the I/O type (exact when the
    values are already representable, as K' is)."""
    x = torch.from_numpy(a64).reshape(like.shape).to(w.torch_dtype)
    return x.cuda()


W = workloads.Workload

SMALL = [
    W("bf16_B32", 1, 2, 1024, 64, 32, 4, seed=11),
    W("bf16_B64_d128", 2, 2, 768, 128, 64, 3, seed=12),
    W("bf16_B16_ragged", 1, 3, 320, 64, 16, 5, seed=13),       # 320 = 256 + 64: ragged chunk
    W("bf16_B128", 1, 2, 1024, 64, 128, 2, seed=14),
    W("f32_B32", 1, 2, 512, 64, 32, 3, dtype="f32", seed=15),
    W("f32_d128", 1, 1, 512, 128, 64, 2, dtype="f32", seed=16),
    W("bf16_dense", 1, 2, 512, 64, 32, 100, seed=17),          # k >= n: full causal attention
    W("bf16_k0", 1, 2, 512, 64, 32, 0, seed=18),               # own block only
    W("bf16_one_block", 1, 1, 128, 64, 128, 4, seed=19),       # n = 1
    W("bf16_B1", 1, 1, 256, 64, 1, 7, seed=20),                # centroid = key
    W("bf16_skew", 1, 2, 2048, 64, 64, 6, skew=True, seed=21),
    # more (row, block) pairs per query tile than one set of LDS row lists holds: several ranges
    W("bf16_k80_ranges", 1, 1, 4096, 64, 32, 80, seed=22),
]
IDS = [w.name for w in SMALL]


# ------------------------------------------------------------------ centroids / conv

@pytest.mark.parametrize("w", SMALL[:6], ids=IDS[:6])
def test_centroids_without_conv(oracle, w):
    t = workloads.generate(w)
    sh = shape_of(w)
    Keff, cent = moba.centroids(sh, t["K"].cuda())
    ref = oracle.centroids(workloads.to_f64(t["K"]), w.B)
    assert parity.max_abs(np64(cent), ref) < 2e-6
    # with no convolution an explicit K_eff buffer receives a copy of K
    buf = torch.empty_like(t["K"]).cuda()
    moba.centroids(sh, t["K"].cuda(), K_eff=buf)
    assert torch.equal(buf.cpu(), t["K"])


@pytest.mark.parametrize("dtype,d,width", [("bf16", 64, 4), ("bf16", 128, 3), ("bf16", 64, 1),
                                           ("bf16", 64, 8), ("f32", 64, 5), ("f32", 128, 2)])
def test_key_conv_and_centroids(oracle, dtype, d, width):
    w = W("conv", 2, 3, 640, d, 32, 2, dtype=dtype, conv_width=width, seed=30 + width)
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    Keff, cent = moba.centroids(shape_of(w), t["K"].cuda(), t["conv_w"].cuda())
    got = np64(Keff)
    if dtype == "bf16":
        # the GPU rounds an fp32 result, the oracle a binary64 one: a 1-ulp difference is
        # possible where the exact value sits next to a rounding boundary, and nowhere else
        diff = got != Kp
        assert diff.mean() < 2e-3
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(Kp), 1e-30))) - 7)
        # plus the fp32 evaluation error itself where k + SiLU(.) nearly cancels
        assert (np.abs(got - Kp)[diff] <= ulp[diff] * 1.0001 + 1e-6 * (1 + np.abs(K))[diff]).all()
        clean = ~diff.reshape(w.bh, w.n, w.B, d).any(axis=2)          # blocks with no such element
        ref = oracle.centroids(Kp, w.B)
        assert np.abs(np64(cent) - ref)[clean].max() < 2e-6
        assert np.abs(np64(cent) - ref).max() < 2e-6 + (np.abs(got - Kp).reshape(w.bh, w.n, w.B, d).sum(2) / w.B).max()
    else:
        assert parity.max_abs(got, Kp) < 2e-5
        assert parity.max_abs(np64(cent), oracle.centroids(Kp, w.B)) < 2e-5


@pytest.mark.parametrize("dtype,d,width,N", [("bf16", 64, 4, 640), ("bf16", 128, 3, 320), ("bf16", 64, 1, 256),
                                             ("bf16", 64, 8, 416), ("f32", 64, 5, 640), ("f32", 128, 2, 96)])
def test_key_conv_backward(oracle, dtype, d, width, N):
    """dK and dw of the convolution's backward against the oracle on the same inputs; N covers
    several 128-row chunks with a ragged last one, and a sequence shorter than a chunk."""
    w = W("convbwd", 2, 3, N, d, 32, 2, dtype=dtype, conv_width=width, seed=130 + width)
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    G = t["dO"]                                     # any tensor of the right shape and type
    dK, dw = moba.key_conv_backward(shape_of(w), t["K"].cuda(), t["conv_w"].cuda(), G.cuda())
    ref_dK, ref_dw = oracle.key_conv_bwd(K, t["conv_w"].double().numpy(), workloads.to_f64(G), w.heads)
    got = np64(dK)
    if dtype == "bf16":         # fp32 arithmetic, one rounding to bf16 at the end
        assert (np.abs(got - ref_dK) <= 2.0 ** -8 * np.abs(ref_dK) + 1e-5).all()
    else:
        assert (np.abs(got - ref_dK) <= 1e-5 * (1 + np.abs(ref_dK))).all()
    assert dw.dtype == torch.float32 and dw.shape == t["conv_w"].shape
    assert parity.rel_l2(dw.double().cpu().numpy(), ref_dw) < 1e-5
    # bit-reproducible (fixed summation order), and dK == dK_eff where the weights vanish
    dK2, dw2 = moba.key_conv_backward(shape_of(w), t["K"].cuda(), t["conv_w"].cuda(), G.cuda())
    assert torch.equal(dK, dK2) and torch.equal(dw, dw2)
    dK0, _ = moba.key_conv_backward(shape_of(w), t["K"].cuda(), torch.zeros_like(t["conv_w"]).cuda(), G.cuda())
    assert torch.equal(dK0.cpu(), G)


# ------------------------------------------------------------------ routing

# the largest number of key blocks per head the library takes (4096), ragged against the bit rows
MANY_BLOCKS = [W("n4096_B2", 1, 1, 8192, 64, 2, 8, seed=23), W("n4000_B2_k40", 1, 1, 8000, 64, 2, 40, seed=24)]


# more blocks than the plain gate kernel takes: kept lists of 64 entries (top-k 40 of 12000 blocks),
# bit rows of 6000 blocks (top-k 80; 48 KB of LDS per strip), and 16384 blocks, the most the
# library takes, with the short kept lists of a small top-k
HUGE_BLOCKS = [W("n12000_B2_k40", 1, 1, 24000, 64, 2, 40, seed=25), W("n6000_B2_k80", 1, 1, 12000, 64, 2, 80, seed=27),
               W("n16384_B2", 1, 1, 32768, 64, 2, 8, seed=26)]


@pytest.mark.parametrize("flags", [pytest.param(0, id="default"),
                                   pytest.param(binding.FLAG_GATE_EXACT_SEARCH, id="exact_search")])
@pytest.mark.parametrize("w", HUGE_BLOCKS, ids=[w.name for w in HUGE_BLOCKS])
def test_topk_beyond_4096_blocks(oracle, w, flags):
    """Routing of sampled queries (the late ones, which have the most candidates, and a spread of the
    rest) and the lists as the exact inverse of the GPU's routing."""
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    C = oracle.centroids(Kp, w.B)
    rng = np.random.default_rng(w.seed)
    rows = np.unique(np.concatenate([rng.integers(0, w.N, 1500), np.arange(w.N - 300, w.N)])).astype(np.int64)
    ref_idx, kth = oracle.topk(Q, C, w.B, w.k, rows=rows)
    sh = shape_of(w, flags)
    cent = torch.from_numpy(C).float().reshape(w.batch, w.heads, w.n, w.d).cuda()
    idx, (off, ql) = moba.topk(sh, t["Q"].cuda(), cent)
    got = npi(idx).reshape(w.bh * w.N, w.k)
    exact, exempt = parity.routing_check(oracle, got[rows], ref_idx, kth, Q, C, w.B, rows=rows)
    assert exempt < 0.02
    srt = np.where(got < 0, np.iinfo(np.int32).max, got)
    assert (np.diff(srt, axis=-1) >= 0).all()
    g_off, g_ql = oracle.csr(npi(idx), w.B)
    parity.check_lists(npi(off), npi(ql), npi(idx), g_off, g_ql, w.k)
    # the plain gate kernel keeps a row of scores per wave in LDS and stops at 4096 blocks
    with pytest.raises(RuntimeError):
        moba.topk(shape_of(w, binding.FLAG_REFERENCE_KERNELS), t["Q"].cuda(), cent)


# the selection with and without its approximate first look (the exact search alone is also what
# queries with many equal scores fall back to)
TOPK_FLAGS = FLAGS + [pytest.param(binding.FLAG_GATE_EXACT_SEARCH, id="exact_search")]


@pytest.mark.parametrize("flags", TOPK_FLAGS)
@pytest.mark.parametrize("w", SMALL + MANY_BLOCKS, ids=IDS + [w.name for w in MANY_BLOCKS])
def test_topk_and_lists(oracle, w, flags):
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    C = oracle.centroids(Kp, w.B)
    ref_idx, kth = oracle.topk(Q, C, w.B, w.k)
    sh = shape_of(w, flags)
    cent = torch.from_numpy(C).float().reshape(w.batch, w.heads, w.n, w.d).cuda()
    idx, (off, ql) = moba.topk(sh, t["Q"].cuda(), cent)
    got = npi(idx).reshape(w.bh * w.N, w.k)
    exact, exempt = parity.routing_check(oracle, got, ref_idx.reshape(w.bh * w.N, w.k), kth.reshape(-1),
                                         Q, C, w.B)
    assert exempt < 0.02
    # rows are in ascending block order with the unused slots at the end
    srt = np.where(got < 0, np.iinfo(np.int32).max, got)
    assert (np.diff(srt, axis=-1) >= 0).all()
    # the lists must be exactly the inverse of the GPU's own routing, ascending
    g_off, g_ql = oracle.csr(npi(idx), w.B)
    parity.check_lists(npi(off), npi(ql), npi(idx), g_off, g_ql, w.k)


@pytest.mark.parametrize("topk", [5, 20])
@pytest.mark.parametrize("flags", [0, binding.FLAG_GATE_EXACT_SEARCH], ids=["default", "exact_search"])
def test_topk_ties_go_to_the_lower_block(flags, topk):
    """K = 0 makes every gate score equal: the kept blocks must be 0..min(k,c)-1.  With
    three bit-identical blocks the kept copies must be a prefix of them.  (top-k 5: kept blocks
    as short lists; 20: as bit rows.)"""
    w = W("ties", 1, 2, 1024, 64, 32, topk, seed=40)
    t = workloads.generate(w)
    sh = shape_of(w, flags)
    cent0 = torch.zeros((1, 2, w.n, w.d), dtype=torch.float32).cuda()
    idx, _ = moba.topk(sh, t["Q"].cuda(), cent0)
    got = npi(idx)
    for tq in range(0, w.N, 7):
        c = tq // w.B
        want = list(range(min(w.k, c))) + [-1] * (w.k - min(w.k, c))
        assert got[0, tq].tolist() == want and got[1, tq].tolist() == want
    K = t["K"].clone()
    for j in (9, 20):
        K[:, :, j * w.B:(j + 1) * w.B] = K[:, :, 4 * w.B:5 * w.B]
    _, cent = moba.centroids(sh, K.cuda())
    idx, _ = moba.topk(sh, t["Q"].cuda(), cent)
    got = npi(idx)
    hits = 0
    for s in range(2):
        for tq in range(21 * w.B, w.N):
            kept = sorted(set(got[s, tq].tolist()) & {4, 9, 20})
            assert kept in ([], [4], [4, 9], [4, 9, 20])
            hits += len(kept) > 0
    assert hits > 0


@pytest.mark.parametrize("w", [SMALL[0], SMALL[2], SMALL[6]], ids=[IDS[0], IDS[2], IDS[6]])
def test_build_lists_from_a_given_routing(oracle, w):
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    ref_idx, _ = oracle.topk(Q, oracle.centroids(Kp, w.B), w.B, w.k)     # best-first order
    off, ql = moba.build_lists(shape_of(w), torch.from_numpy(ref_idx).reshape(
        w.batch, w.heads, w.N, w.k).cuda())
    r_off, r_ql = oracle.csr(ref_idx, w.B)
    parity.check_lists(npi(off), npi(ql), ref_idx, r_off, r_ql, w.k)


# ------------------------------------------------------------------ attention at the oracle's routing

@pytest.mark.parametrize("flags", ATTN_FLAGS)
@pytest.mark.parametrize("w", SMALL, ids=IDS)
def test_forward_backward_at_oracle_routing(oracle, w, flags):
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    ref_idx, _ = oracle.topk(Q, oracle.centroids(Kp, w.B), w.B, w.k)
    sh = shape_of(w, flags)
    d = dev(t)
    idx = torch.from_numpy(ref_idx).reshape(w.batch, w.heads, w.N, w.k).cuda()
    lists = moba.build_lists(sh, idx)
    O, lse = moba.forward(sh, d["Q"], d["K"], d["V"], idx, lists)
    rO, rlse = oracle.attn_fwd(Q, K, V, ref_idx, w.B, w.scale)
    assert parity.max_abs(np64(O), rO) < parity.O_TOL[w.dtype]
    assert parity.max_abs(np64(lse), rlse) < parity.LSE_TOL[w.dtype]
    dQ, dK, dV = moba.backward(sh, d["Q"], d["K"], d["V"], O, lse, d["dO"], idx, lists)
    # the oracle's backward starts from its own forward (binary64 O and lse)
    rQ, rK, rV = oracle.attn_bwd(Q, K, V, ref_idx, dO, w.B, w.scale)
    tol = parity.GRAD_TOL[w.dtype]
    assert parity.rel_l2(np64(dQ), rQ) < tol
    assert parity.rel_l2(np64(dK), rK) < tol
    assert parity.rel_l2(np64(dV), rV) < tol


# shapes that reach every variant of the key-block-major kernels: key blocks in 128-key parts,
# three 32-key groups, and rows of kept blocks searched in one, two and more steps
KEY_MAJOR = [
    W("km_B256_parts", 1, 2, 2048, 64, 256, 3, seed=61),
    W("km_B512_d128", 1, 1, 2048, 128, 512, 2, seed=62),
    W("km_B96", 1, 1, 960, 64, 96, 3, seed=63),
    W("km_d128_B128_parts", 1, 2, 2048, 128, 128, 3, seed=69),
    W("km_k16", 1, 1, 2048, 64, 32, 16, seed=64),
    W("km_k40", 1, 1, 4096, 64, 32, 40, seed=65),
    W("km_d128_k20", 1, 1, 2048, 128, 32, 20, seed=66),
    W("km_d128_k40", 1, 1, 4096, 128, 64, 40, seed=67),
    W("km_sparse_default", 1, 2, 16384, 64, 128, 2, seed=68),   # sparse enough that the library picks key-major by itself
]


@pytest.mark.parametrize("w", KEY_MAJOR, ids=[w.name for w in KEY_MAJOR])
def test_key_major_variants(oracle, w):
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    ref_idx, _ = oracle.topk(Q, oracle.centroids(Kp, w.B), w.B, w.k)
    sh = shape_of(w, 0 if w.name.endswith("default") else binding.FLAG_KEY_MAJOR)
    d = dev(t)
    idx = torch.from_numpy(ref_idx).reshape(w.batch, w.heads, w.N, w.k).cuda()
    lists = moba.build_lists(sh, idx)
    O, lse = moba.forward(sh, d["Q"], d["K"], d["V"], idx, lists)
    rO, rlse = oracle.attn_fwd(Q, K, V, ref_idx, w.B, w.scale)
    assert parity.max_abs(np64(O), rO) < parity.O_TOL[w.dtype]
    assert parity.max_abs(np64(lse), rlse) < parity.LSE_TOL[w.dtype]
    # the same forward by query tiles: the two cuts must agree far inside the tolerance
    O2, lse2 = moba.forward(shape_of(w, binding.FLAG_QUERY_TILES), d["Q"], d["K"], d["V"], idx, lists)
    assert parity.max_abs(np64(lse), np64(lse2)) < 1e-4
    dQ, dK, dV = moba.backward(sh, d["Q"], d["K"], d["V"], O, lse, d["dO"], idx, lists)
    rQ, rK, rV = oracle.attn_bwd(Q, K, V, ref_idx, dO, w.B, w.scale)
    tol = parity.GRAD_TOL[w.dtype]
    assert parity.rel_l2(np64(dQ), rQ) < tol
    assert parity.rel_l2(np64(dK), rK) < tol
    assert parity.rel_l2(np64(dV), rV) < tol


# ------------------------------------------------------------------ grouped-query / multi-query attention

GQA = [
    W("gqa_G4_B32", 1, 8, 1024, 64, 32, 4, kv_heads=2, seed=81),
    W("mqa_d128_B64", 2, 4, 768, 128, 64, 3, kv_heads=1, seed=82),
    W("gqa_f32", 1, 4, 512, 64, 32, 3, dtype="f32", kv_heads=2, seed=83),
    W("gqa_B128", 2, 4, 1024, 64, 128, 2, kv_heads=2, seed=84),
    W("gqa_conv", 1, 4, 640, 64, 32, 2, kv_heads=2, conv_width=3, seed=85),
    W("gqa_B16", 1, 6, 320, 64, 16, 5, kv_heads=3, seed=86),               # plain kernels for bf16 too
    W("gqa_B256_parts", 1, 4, 2048, 64, 256, 2, kv_heads=2, seed=87),      # key-major: two parts per block
]


@pytest.mark.parametrize("flags", ATTN_FLAGS)
@pytest.mark.parametrize("w", GQA, ids=[w.name for w in GQA])
def test_grouped_query_heads(oracle, w, flags):
    """Query head h reads key/value head h // G; dK and dV are summed over the sharing heads
    (Appendix C, last paragraph).  The oracle computes on copies of the shared heads."""
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)          # K, Kp, V: [b*kv_heads, N, d]
    sh = shape_of(w, flags)
    d = dev(t)
    C = oracle.centroids(Kp, w.B)
    Keff, cent = moba.centroids(sh, d["K"], d["conv_w"])
    assert tuple(cent.shape) == (w.batch, w.hkv, w.n, w.d)
    assert parity.max_abs(np64(cent), C) < (2e-6 if not w.conv_width else 1e-3)
    Ke, Ve, Ce = (oracle.gqa_expand(x, w.heads, w.hkv) for x in (Kp, V, C))
    ref_idx, kth = oracle.topk(Q, Ce, w.B, w.k)
    cent_ref = torch.from_numpy(C).float().reshape(w.batch, w.hkv, w.n, w.d).cuda()
    idx, (off, ql) = moba.topk(sh, d["Q"], cent_ref)
    exact, exempt = parity.routing_check(oracle, npi(idx).reshape(w.bh * w.N, w.k),
                                         ref_idx.reshape(w.bh * w.N, w.k), kth.reshape(-1), Q, Ce, w.B)
    assert exempt < 0.02
    # attention at the oracle's routing
    idx = torch.from_numpy(ref_idx).reshape(w.batch, w.heads, w.N, w.k).cuda()
    lists = moba.build_lists(sh, idx)
    Kdev = to_io(w, Kp, t["K"])
    O, lse = moba.forward(sh, d["Q"], Kdev, d["V"], idx, lists)
    rO, rlse = oracle.attn_fwd(Q, Ke, Ve, ref_idx, w.B, w.scale)
    assert parity.max_abs(np64(O), rO) < parity.O_TOL[w.dtype]
    assert parity.max_abs(np64(lse), rlse) < parity.LSE_TOL[w.dtype]
    dQ, dK, dV = moba.backward(sh, d["Q"], Kdev, d["V"], O, lse, d["dO"], idx, lists)
    assert dK.shape == t["K"].shape and dV.shape == t["V"].shape
    rQ, rKe, rVe = oracle.attn_bwd(Q, Ke, Ve, ref_idx, dO, w.B, w.scale)
    tol = parity.GRAD_TOL[w.dtype]
    assert parity.rel_l2(np64(dQ), rQ) < tol
    assert parity.rel_l2(np64(dK), oracle.gqa_reduce(rKe, w.heads, w.hkv)) < tol
    assert parity.rel_l2(np64(dV), oracle.gqa_reduce(rVe, w.heads, w.hkv)) < tol
    if w.conv_width:
        # the convolution and its backward run per key/value head
        gK, gw = moba.key_conv_backward(sh, d["K"], d["conv_w"], dK)
        rgK, rgw = oracle.key_conv_bwd(K, t["conv_w"].double().numpy(), np64(dK), w.hkv)
        assert parity.rel_l2(np64(gK), rgK) < 1e-2
        assert parity.rel_l2(gw.double().cpu().numpy(), rgw) < 1e-4


# ------------------------------------------------------------------ ragged sequence by zero padding

def test_ragged_sequence_by_zero_padding():
    """N % B != 0 in a training-shaped call: pad Q, K, V and dO with zero rows to the next
    multiple of B.  A query never sees a later key, the padded block is never a routing
    candidate of a real query (candidates are blocks before the query's own), and zero dO rows
    add nothing to dK and dV -- so the real rows are exact.  Checked against a dense fp64
    evaluation of the ragged sequence itself (tail block shorter than B), not of the padded one."""
    from tests import brute
    N, B, k, d, heads = 1000, 32, 4, 64, 2
    Np = -(-N // B) * B
    g = torch.Generator().manual_seed(91)
    Q, K, V, dO = (torch.randn((1, heads, N, d), generator=g).to(torch.bfloat16) for _ in range(4))
    pad = lambda x: torch.cat([x, torch.zeros((1, heads, Np - N, d), dtype=x.dtype)], dim=2).cuda()
    sh = moba.Shape(1, heads, Np, d, B, k, 0, binding.BF16)
    Keff, cent = moba.centroids(sh, pad(K))
    idx, lists = moba.topk(sh, pad(Q), cent)
    O, lse = moba.forward(sh, pad(Q), Keff, pad(V), idx, lists)
    dQ, dK, dV = moba.backward(sh, pad(Q), Keff, pad(V), O, lse, pad(dO), idx, lists)
    scale = 1.0 / np.sqrt(d)
    for h in range(heads):
        q, kk, v, go = (x[0, h].double().numpy() for x in (Q, K, V, dO))
        # the ragged definition: complete past blocks are the candidates, own block up to t
        nfull = N // B
        cen = kk[:nfull * B].reshape(nfull, B, d).mean(1).astype(np.float32).astype(np.float64)
        mask = np.zeros((N, N), dtype=bool)
        for t in range(N):
            own = t // B
            cand = sorted(range(own), key=lambda j: (-float(q[t] @ cen[j]), j))[:k]
            for j in cand:
                mask[t, j * B:(j + 1) * B] = True
            mask[t, own * B:t + 1] = True
        rO, rlse, _ = brute.dense_attention(q, kk, v, mask, scale)
        rQ, rK, rV = brute.dense_backward(q, kk, v, mask, scale, go)
        got = lambda x: x[0, h, :N].double().cpu().numpy()
        same = np.ones(N, bool)
        gi = idx[0, h, :N].cpu().numpy()
        for t in range(N):       # rows whose routing matches (fp32 near-ties aside) compare one by one
            own = t // B
            ref = sorted(sorted(range(own), key=lambda j: (-float(q[t] @ cen[j]), j))[:k])
            same[t] = ref == sorted(int(x) for x in gi[t] if x >= 0)
        assert same.mean() > 0.99
        assert np.abs(got(O) - rO)[same].max() < parity.O_TOL["bf16"]
        assert np.abs(lse[0, h, :N].double().cpu().numpy() - rlse)[same].max() < parity.LSE_TOL["bf16"]
        assert parity.rel_l2(got(dQ)[same], rQ[same]) < parity.GRAD_TOL["bf16"]
        if same.all():
            assert parity.rel_l2(got(dK), rK) < parity.GRAD_TOL["bf16"]
            assert parity.rel_l2(got(dV), rV) < parity.GRAD_TOL["bf16"]
        # the padded rows take nothing and give nothing
        assert float(dK[0, h, N:].abs().max()) == 0.0 and float(dV[0, h, N:].abs().max()) == 0.0


# ------------------------------------------------------------------ the whole chain on its own routing

@pytest.mark.parametrize("flags", FLAGS)
@pytest.mark.parametrize("w", [W("chain_bf16", 1, 2, 1024, 64, 32, 4, backward=True, seed=50),
                               W("chain_conv", 1, 2, 1024, 128, 64, 3, conv_width=4, seed=51),
                               W("chain_f32", 1, 2, 512, 64, 32, 3, dtype="f32", seed=52),
                               # the largest top-k the library takes (rows of 4096 entries, full causal
                               # attention): the plain kernels then need more LDS than the default limit
                               W("chain_k4096", 1, 1, 256, 64, 2, 4096, dtype="f32", seed=53),
                               W("chain_k4096_bf16", 1, 1, 256, 64, 2, 4096, seed=54)],
                         ids=["bf16", "conv_d128", "f32", "f32_k4096", "bf16_k4096"])
def test_whole_chain(oracle, w, flags):
    t = workloads.generate(w)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    sh = shape_of(w, flags)
    d = dev(t)
    Keff, cent = moba.centroids(sh, d["K"], d["conv_w"])
    idx, lists = moba.topk(sh, d["Q"], cent)
    O, lse = moba.forward(sh, d["Q"], Keff, d["V"], idx, lists)
    dQ, dK, dV = moba.backward(sh, d["Q"], Keff, d["V"], O, lse, d["dO"], idx, lists)
    C = oracle.centroids(Kp, w.B)
    ref_idx, kth = oracle.topk(Q, C, w.B, w.k)
    exact, exempt = parity.routing_check(oracle, npi(idx).reshape(w.bh * w.N, w.k), ref_idx.reshape(w.bh * w.N, w.k),
                                         kth.reshape(-1), Q, C, w.B)
    assert exempt < 0.02
    rO, rlse = oracle.attn_fwd(Q, Kp, V, ref_idx, w.B, w.scale)
    # rows whose routing is identical are comparable one by one
    got_O = np64(O).reshape(-1, w.d)
    assert np.abs(got_O - rO.reshape(-1, w.d))[exact].max() < parity.O_TOL[w.dtype]
    assert np.abs(np64(lse).reshape(-1) - rlse.reshape(-1))[exact].max() < parity.LSE_TOL[w.dtype]
    rQ, rK, rV = oracle.attn_bwd(Q, Kp, V, ref_idx, dO, w.B, w.scale)
    tol = parity.GRAD_TOL[w.dtype] if exact.all() and not w.conv_width else 5e-2
    assert parity.rel_l2(np64(dQ).reshape(-1, w.d)[exact], rQ.reshape(-1, w.d)[exact]) < tol
    assert parity.rel_l2(np64(dK), rK) < tol
    assert parity.rel_l2(np64(dV), rV) < tol


def test_results_are_reproducible():
    w = W("repro", 1, 2, 1024, 64, 32, 4, backward=True, seed=60)
    d = dev(workloads.generate(w))
    sh = shape_of(w)
    outs = []
    for _ in range(2):
        Keff, cent = moba.centroids(sh, d["K"])
        idx, lists = moba.topk(sh, d["Q"], cent)
        O, lse = moba.forward(sh, d["Q"], Keff, d["V"], idx, lists)
        grads = moba.backward(sh, d["Q"], Keff, d["V"], O, lse, d["dO"], idx, lists)
        outs.append((idx,) + tuple(lists) + (O, lse) + tuple(grads))
    for a, b in zip(*outs):
        if a.dtype == torch.int32:
            assert torch.equal(a, b)
        else:
            assert parity.rel_l2(np64(a) if a.dim() == 4 else a.double().cpu().numpy(),
                                 np64(b) if b.dim() == 4 else b.double().cpu().numpy()) < 1e-5


@pytest.mark.parametrize("flags", FLAGS)
def test_logit_far_above_the_own_block(oracle, flags):
    """A routed key whose logit exceeds everything in the query's own block by ~80 (natural
    log units): the fast forward path cannot represent exp(80) relative to its per-row
    reference and must hand the row to its exact fallback."""
    w = W("outlier", 1, 2, 1024, 64, 32, 4, backward=True, seed=70)
    t = workloads.generate(w)
    for tq, u in ((700, 100), (701, 333), (1023, 5)):
        t["K"][0, :, u] = (10.0 * t["Q"][0, :, tq].float()).to(torch.bfloat16)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    ref_idx, _ = oracle.topk(Q, oracle.centroids(Kp, w.B), w.B, w.k)
    assert 100 // w.B in ref_idx[0, 700] and 333 // w.B in ref_idx[1, 701]
    sh = shape_of(w, flags)
    d = dev(t)
    idx = torch.from_numpy(ref_idx).reshape(w.batch, w.heads, w.N, w.k).cuda()
    lists = moba.build_lists(sh, idx)
    O, lse = moba.forward(sh, d["Q"], d["K"], d["V"], idx, lists)
    rO, rlse = oracle.attn_fwd(Q, K, V, ref_idx, w.B, w.scale)
    assert rlse[0, 700] > 60
    assert parity.max_abs(np64(O), rO) < parity.O_TOL[w.dtype]
    assert parity.max_abs(np64(lse), rlse) < 1e-2
    dQ, dK, dV = moba.backward(sh, d["Q"], d["K"], d["V"], O, lse, d["dO"], idx, lists)
    rQ, rK, rV = oracle.attn_bwd(Q, K, V, ref_idx, dO, w.B, w.scale)
    for a, b in ((dQ, rQ), (dK, rK), (dV, rV)):
        assert parity.rel_l2(np64(a), b) < parity.GRAD_TOL[w.dtype]


@pytest.mark.parametrize("N,flags", [(4096, 0), (4096, binding.FLAG_QUERY_TILES), (16384, 0),
                                     (16384, binding.FLAG_QUERY_TILES), (32768, 0)],
                         ids=["4K_default", "4K_tiles", "16K_default", "16K_tiles", "32K_default"])
def test_dense_rows_with_a_dominant_logit(oracle, N, flags):
    """Full causal attention (every past block kept) over long rows in which one key's logit
    stands ~14 above thousands of others: the denominators of such rows are made of one 1 and very
    many tiny terms, which fixed-point sums with too few fraction bits would drop.  The query-tile
    forward takes at most 4096 keys per query; these rows must go to a kernel that sums in floating
    point whatever the flags say.  Sampled rows against the oracle."""
    B = 128
    w = W("dense_dominant", 1, 1, N, 64, B, N // B, seed=77)
    t = workloads.generate(w)
    rows = np.array([N - 1, N - 2, N - 200, N // 2 + 3, 3 * N // 4, 129, 5], dtype=np.int64)
    for r in rows[:3]:                       # dominant key far in the past of these queries
        q = t["Q"][0, 0, r].float()
        t["K"][0, 0, 777 + int(r) % 50] = (q * (14.0 / (w.scale * float(q @ q)))).to(torch.bfloat16)
    Q, K, Kp, V, dO = oracle_inputs(oracle, w, t)
    n = N // B
    idx = np.full((1, N, n), -1, np.int32)   # dense routing: all past blocks, ascending
    for c in range(n):
        idx[0, c * B:(c + 1) * B, :c] = np.arange(c, dtype=np.int32)
    sh = shape_of(w, flags)
    d = dev(t)
    gidx = torch.from_numpy(idx).reshape(1, 1, N, n).cuda()
    lists = moba.build_lists(sh, gidx)
    O, lse = moba.forward(sh, d["Q"], d["K"], d["V"], gidx, lists)
    rO, rlse = oracle.attn_fwd(Q, K, V, idx, B, w.scale, rows=rows)
    got_O, got_lse = np64(O)[0][rows], lse.double().cpu().numpy().reshape(-1)[rows]
    assert parity.max_abs(got_O, rO) < parity.O_TOL[w.dtype]
    assert parity.max_abs(got_lse, rlse) < parity.LSE_TOL[w.dtype]


def test_shared_workspace_gives_the_same_results():
    """MOBA_FLAG_SHARED_WORKSPACE: forward and backward on one workspace, the copies of K and V made
    once by the forward call -- bit-identical to separate workspaces (and no effect where the
    key-major kernels run)."""
    for w, extra in ((W("shared_ws", 1, 2, 2048, 64, 32, 8, backward=True, seed=81), 0),
                     (W("shared_ws_d128", 2, 2, 1024, 128, 64, 3, backward=True, seed=82), binding.FLAG_QUERY_TILES),
                     (W("shared_ws_gqa", 1, 4, 1024, 64, 32, 4, backward=True, kv_heads=2, seed=83), 0),
                     (W("shared_ws_km", 1, 2, 1024, 64, 128, 2, backward=True, seed=84), binding.FLAG_KEY_MAJOR)):
        d = dev(workloads.generate(w))
        outs = []
        for shared in (0, binding.FLAG_SHARED_WORKSPACE):
            sh = shape_of(w, extra | shared)
            Keff, cent = moba.centroids(sh, d["K"])
            idx, lists = moba.topk(sh, d["Q"], cent)
            sizes = moba.workspace_bytes(sh)
            if shared:                  # (equal sizes where the flag takes effect; the larger one serves both)
                ws_f = ws_b = torch.empty(max(sizes[1:]), dtype=torch.uint8, device="cuda")
            else:
                ws_f, ws_b = (torch.empty(x, dtype=torch.uint8, device="cuda") for x in sizes[1:])
            O, lse = moba.forward(sh, d["Q"], Keff, d["V"], idx, lists, ws=ws_f)
            grads = moba.backward(sh, d["Q"], Keff, d["V"], O, lse, d["dO"], idx, lists, ws=ws_b)
            outs.append((O, lse) + tuple(grads))
        for a, b in zip(*outs):
            assert torch.equal(a, b)


@pytest.mark.parametrize("flags", ATTN_FLAGS)
def test_nonfinite_inputs_reach_the_outputs(flags):
    """A NaN in Q, K, V or dO must not vanish inside the attention kernels (a training loop's
    overflow detection looks for it in the outputs): every row that attends the poisoned key, or is
    the poisoned query, comes out NaN, whichever kernels run; the other head stays finite.
    (A kernel may mark more than those rows -- e.g. a whole channel of the head.)"""
    w = W("nonfinite", 1, 2, 1024, 64, 32, 4, backward=True, seed=88)
    t = workloads.generate(w)
    sh = shape_of(w, flags)
    d = dev(t)
    _, cent = moba.centroids(sh, d["K"])
    idx, lists = moba.topk(sh, d["Q"], cent)               # routing of the clean inputs, kept fixed
    hidx = npi(idx)[0]
    u, tq = 300, 777
    attends = np.array([(tt >= u and tt // w.B == u // w.B) or (u // w.B) in hidx[tt] for tt in range(w.N)])
    assert attends.sum() > 10

    def run(**poison):
        x = {k: v.clone() for k, v in d.items() if v is not None}
        for name, (row, col) in poison.items():
            x[name][0, 0, row, col] = float("nan")
        O, lse = moba.forward(sh, x["Q"], x["K"], x["V"], idx, lists)
        dQ, dK, dV = moba.backward(sh, x["Q"], x["K"], x["V"], O, lse, x["dO"], idx, lists)
        return [a.float().cpu().numpy()[0] for a in (O, dQ, dK, dV)] + [lse.cpu().numpy()[0]]

    O, dQ, dK, dV, lse = run(K=(u, 5))
    assert np.isnan(O[0][attends]).all() and np.isnan(lse[0][attends]).all() and np.isnan(dQ[0][attends]).all()
    for a in (O, dQ, dK, dV):
        assert np.isfinite(a[1]).all()
    O, dQ, dK, dV, lse = run(V=(u, 5))
    assert np.isnan(O[0][attends][:, 5]).all() and np.isnan(dQ[0][attends]).all()
    assert np.isfinite(O[1]).all() and np.isfinite(dQ[1]).all()
    O, dQ, dK, dV, lse = run(Q=(tq, 9))
    assert np.isnan(O[0][tq]).all() and np.isnan(dQ[0][tq]).all() and np.isfinite(O[1]).all()
    O, dQ, dK, dV, lse = run(dO=(tq, 9))
    assert np.isfinite(O).all() and np.isnan(dQ[0][tq]).all() and np.isfinite(dQ[1]).all()
    assert np.isnan(dV[0][tq - 1]).any()                  # the row's own block receives the NaN


def test_kernel_timing_session():
    """moba_profile_begin/_end: one event pair per launch of a main kernel, results unchanged."""
    w = W("timing", 1, 2, 2048, 64, 32, 8, backward=True, seed=72)
    d = dev(workloads.generate(w))
    sh = shape_of(w)
    Ke, c = moba.centroids(sh, d["K"])

    def chain():
        idx, lists = moba.topk(sh, d["Q"], c)
        O, lse = moba.forward(sh, d["Q"], Ke, d["V"], idx, lists)
        g = moba.backward(sh, d["Q"], Ke, d["V"], O, lse, d["dO"], idx, lists)
        torch.cuda.synchronize()
        return [x.clone() for x in (idx, O, lse, *g)]

    plain = chain()
    moba.profile_begin()
    timed = [chain() for _ in range(2)]
    times = moba.profile_end()
    assert set(times) == {"topk", "forward", "bwd_dq", "bwd_dkdv"}
    for name, (ms, calls) in times.items():
        assert calls == 2 and 0.0 < ms < 1e3, (name, ms, calls)
    for run in timed:
        for a, b in zip(plain, run):
            assert torch.equal(a, b)
    assert moba.profile_end.__doc__ and all(v == (0.0, 0) for v in _closed_session().values())


def _closed_session():
    moba.profile_begin()
    return moba.profile_end()


# ------------------------------------------------------------------ buffers

GUARD = 4096


def _guarded(nbytes, like_dtype=torch.uint8, shape=None):
    """A buffer of nbytes (or of `shape` elements of like_dtype) inside a larger allocation whose
    GUARD bytes in front and behind hold a pattern: -> (view, check) where check() fails if a kernel
    wrote outside the view."""
    if shape is not None:
        nbytes = int(np.prod(shape)) * torch.empty((), dtype=like_dtype).element_size()
    nbytes = max(int(nbytes), 256)
    padded = (nbytes + 255) // 256 * 256
    big = torch.full((padded + 2 * GUARD,), 0x5A, dtype=torch.uint8, device="cuda")
    view = big[GUARD:GUARD + nbytes]
    if shape is not None:
        view = view.view(like_dtype).reshape(shape)

    def check(what):
        torch.cuda.synchronize()
        assert bool((big[:GUARD] == 0x5A).all()) and bool((big[GUARD + nbytes:] == 0x5A).all()), \
            "%s: bytes outside the buffer were written" % what
    return view, check


@pytest.mark.parametrize("flags", [pytest.param(0, id="default"), pytest.param(REF, id="plain"),
                                   pytest.param(binding.FLAG_KEY_MAJOR, id="keymajor"),
                                   pytest.param(binding.FLAG_QUERY_TILES, id="tiles"),
                                   pytest.param(binding.FLAG_QUERY_TILES | binding.FLAG_SHARED_WORKSPACE, id="tiles_shared")])
@pytest.mark.parametrize("w", [SMALL[0], SMALL[1], SMALL[2], SMALL[10], SMALL[11],
                               W("gqa_B64", 1, 4, 1536, 64, 64, 5, kv_heads=2, seed=81),
                               W("conv_d128_B128", 1, 2, 1280, 128, 128, 3, conv_width=3, seed=82)],
                         ids=lambda w: w.name)
def test_no_kernel_writes_outside_its_buffers(w, flags):
    """Every workspace and every output the caller hands over lies between guard bytes; the whole
    chain (centroids, gate top-k + lists, forward, backward) must leave them as they were."""
    t = dev(workloads.generate(w))
    sh = shape_of(w, flags)
    dt = t["Q"].dtype
    sizes = moba.workspace_bytes(sh)
    ws_topk, c_topk = _guarded(sizes[0])
    if flags & binding.FLAG_SHARED_WORKSPACE:
        ws_fwd, c_fwd = _guarded(max(sizes[1], sizes[2]))
        ws_bwd, c_bwd = ws_fwd, c_fwd
    else:
        ws_fwd, c_fwd = _guarded(sizes[1])
        ws_bwd, c_bwd = _guarded(sizes[2])
    cent, c_cent = _guarded(0, torch.float32, (w.batch, w.hkv, w.n, w.d))
    Keff, c_keff = _guarded(0, dt, tuple(t["K"].shape))
    O, c_O = _guarded(0, dt, tuple(t["Q"].shape))
    lse, c_lse = _guarded(0, torch.float32, (w.batch, w.heads, w.N))
    dQ, c_dQ = _guarded(0, dt, tuple(t["Q"].shape))
    dK, c_dK = _guarded(0, dt, tuple(t["K"].shape))
    dV, c_dV = _guarded(0, dt, tuple(t["V"].shape))
    Ke, c = moba.centroids(sh, t["K"], t["conv_w"], K_eff=Keff, out=cent)
    idx, lists = moba.topk(sh, t["Q"], c, ws=ws_topk)
    moba.forward(sh, t["Q"], Ke, t["V"], idx, lists, ws=ws_fwd, O=O, lse=lse)
    moba.backward(sh, t["Q"], Ke, t["V"], O, lse, t["dO"], idx, lists, ws=ws_bwd, out=(dQ, dK, dV))
    for what, chk in (("top-k workspace", c_topk), ("forward workspace", c_fwd), ("backward workspace", c_bwd),
                      ("centroids", c_cent), ("K_eff", c_keff), ("O", c_O), ("lse", c_lse), ("dQ", c_dQ),
                      ("dK", c_dK), ("dV", c_dV)):
        chk(what)
    assert torch.isfinite(O.float()).all() and torch.isfinite(dK.float()).all()
