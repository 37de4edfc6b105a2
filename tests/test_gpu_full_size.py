"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The whole chain runs on the GPU for all slices.  The oracle then evaluates, for a few
(batch, head) slices: the centroids (all), the routing of sampled query rows (under the
gap rule), forward outputs / lse / dQ of sampled rows, and dK / dV of sampled key blocks.
For dK/dV the oracle needs the routing of every query of the slice, so those slices get
a full oracle top-k.  Nothing the oracle reads comes from the GPU: where the GPU's
routing of a row differs (near-ties), the row is left out of the one-by-one output
comparison, and dK/dV -- sums over ~2000 queries each -- are compared as they are.
Properties that hold at any size (list structure, row sums) cover the rest."""
import numpy as np
import pytest
import torch

import paper_2511_11571_amd as moba
import workloads
from tests import parity
from paper_2511_11571_amd import binding
from tests.test_gpu_parity import dev, np64, npi, shape_of

pytestmark = pytest.mark.gpu


def run_gpu(w, flags=0):
    t = workloads.generate(w)
    d = dev(t)
    sh = shape_of(w, flags)
    Keff, cent = moba.centroids(sh, d["K"], d["conv_w"])
    idx, lists = moba.topk(sh, d["Q"], cent)
    O, lse = moba.forward(sh, d["Q"], Keff, d["V"], idx, lists)
    out = dict(Keff=Keff, cent=cent, idx=idx, off=lists[0], ql=lists[1], O=O, lse=lse)
    if w.backward:
        out["dQ"], out["dK"], out["dV"] = moba.backward(sh, d["Q"], Keff, d["V"], O, lse, d["dO"],
                                                        idx, lists)
    torch.cuda.synchronize()
    return t, out


def slice64(x, s, heads):
    b, h = divmod(s, heads)
    return x[b, h].detach().float().cpu().to(torch.float64).numpy()[None]


def check_slice(oracle, w, t, out, s, n_rows, blocks, rng):
    heads = w.heads
    Q, K, V, dO = (slice64(t[x], s, heads) for x in ("Q", "K", "V", "dO"))
    Kp = K
    if w.conv_width:
        cw = t["conv_w"][s % heads:s % heads + 1].double().numpy()
        Kp = oracle.key_conv(K, cw, 1, oracle.ROUND_BF16 if w.dtype == "bf16" else oracle.ROUND_F32)
        got = slice64(out["Keff"], s, heads)
        diff = got != Kp
        assert diff.mean() < 2e-3
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(Kp), 1e-30))) - 7)
        # plus the fp32 evaluation error itself where k + SiLU(.) nearly cancels
        assert (np.abs(got - Kp)[diff] <= ulp[diff] * 1.0001 + 1e-6 * (1 + np.abs(K))[diff]).all()
    C = oracle.centroids(Kp, w.B)
    cent = slice64(out["cent"], s, heads)
    tol_c = 5e-6 if not w.conv_width else 5e-6 + 2.0 ** -6 / w.B * 4
    assert parity.max_abs(cent, C) < tol_c

    full = bool(blocks)
    if full:
        rows = np.arange(w.N, dtype=np.int64)
    else:
        edge = [0, w.B - 1, w.B, w.k * w.B - 1, w.k * w.B, (w.k + 1) * w.B, w.N - 1]
        rows = np.unique(np.concatenate([rng.integers(0, w.N, n_rows), np.array(edge)])).astype(np.int64)
        rows = rows[(rows >= 0) & (rows < w.N)]
    ref_idx, kth = oracle.topk(Q, C, w.B, w.k, rows=rows)
    b, h = divmod(s, heads)
    g_idx = out["idx"][b, h].cpu().numpy()
    exact, exempt = parity.routing_check(oracle, g_idx[rows], ref_idx, kth, Q, C, w.B, rows=rows)
    assert exempt < 0.03, exempt

    # lists: the GPU's lists are exactly the inverse of the GPU's routing (any size)
    g_off = out["off"][b, h].cpu().numpy()
    g_ql = out["ql"][b, h].cpu().numpy()
    assert g_off[0] == 0 and g_off[-1] == oracle.routes_per_slice(w.N, w.B, w.k)
    counts = np.bincount(g_idx[g_idx >= 0].ravel(), minlength=w.n)
    assert np.array_equal(np.diff(g_off), counts)
    for j in rng.integers(0, w.n, 8):
        lst = g_ql[g_off[j]:g_off[j + 1]]
        assert np.array_equal(lst & 0xffffff, np.nonzero((g_idx == j).any(-1))[0])
        if (lst >> 24).any():              # high byte: where j sits in the query's row of kept blocks
            assert (g_idx[lst & 0xffffff, lst >> 24] == j).all()

    # forward / dQ on sampled rows, with the oracle's own routing
    sample = rows if not full else np.unique(rng.integers(0, w.N, n_rows)).astype(np.int64)
    idx_full = np.full((1, w.N, w.k), -1, np.int32)
    idx_full[0, rows] = ref_idx
    rO, rlse = oracle.attn_fwd(Q, Kp, V, idx_full, w.B, w.scale, rows=sample)
    same = exact[np.searchsorted(rows, sample)]
    gO = slice64(out["O"], s, heads)[0][sample]
    glse = out["lse"][b, h].double().cpu().numpy()[sample]
    assert np.abs(gO - rO)[same].max() < parity.O_TOL[w.dtype]
    assert np.abs(glse - rlse)[same].max() < parity.LSE_TOL[w.dtype]
    stats = dict(exempt=exempt, O_err=float(np.abs(gO - rO)[same].max()))
    if w.backward:
        lse_full = np.zeros((1, w.N))
        Dv = np.zeros((1, w.N))
        lse_full[0, sample] = rlse
        Dv[0, sample] = (dO[0, sample] * rO).sum(-1)
        rdQ = oracle.attn_bwd_dq(Q, Kp, V, idx_full, dO, lse_full, Dv, w.B, w.scale, rows=sample)
        gdQ = slice64(out["dQ"], s, heads)[0][sample]
        stats["dQ_rel"] = parity.rel_l2(gdQ[same], rdQ[same])
        assert stats["dQ_rel"] < parity.GRAD_TOL[w.dtype]
    if w.backward and full:
        r_off, r_ql = oracle.csr(ref_idx[None], w.B)
        need = np.unique(np.concatenate(
            [r_ql[0, r_off[0, j]:r_off[0, j + 1]] for j in blocks] +
            [np.arange(j * w.B, (j + 1) * w.B) for j in blocks])).astype(np.int64)
        nO, nlse = oracle.attn_fwd(Q, Kp, V, ref_idx[None], w.B, w.scale, rows=need)
        lse_full = np.zeros((1, w.N))
        Dv = np.zeros((1, w.N))
        lse_full[0, need] = nlse
        Dv[0, need] = (dO[0, need] * nO).sum(-1)
        rK, rV = oracle.attn_bwd_dkdv(Q, Kp, V, dO, lse_full, Dv, r_off, r_ql, w.B, w.scale,
                                      blocks=np.array(blocks, dtype=np.int64))
        gK = slice64(out["dK"], s, heads)[0].reshape(w.n, w.B, w.d)[blocks]
        gV = slice64(out["dV"], s, heads)[0].reshape(w.n, w.B, w.d)[blocks]
        stats["dK_rel"] = parity.rel_l2(gK, rK)
        stats["dV_rel"] = parity.rel_l2(gV, rV)
        assert stats["dK_rel"] < parity.GRAD_TOL[w.dtype]
        assert stats["dV_rel"] < parity.GRAD_TOL[w.dtype]
        for i in range(len(blocks)):                      # no single block may hide in the average
            assert parity.rel_l2(gK[i], rK[i]) < 2 * parity.GRAD_TOL[w.dtype]
            assert parity.rel_l2(gV[i], rV[i]) < 2 * parity.GRAD_TOL[w.dtype]
    return stats


def test_config1_fp32_forward_full(oracle):
    """N = 2048, fp32: small enough for the oracle to check every row of every slice."""
    w = workloads.CONFIGS[1]
    t, out = run_gpu(w)
    Q, K, V = (workloads.to_f64(t[x]) for x in ("Q", "K", "V"))
    C = oracle.centroids(K, w.B)
    ref_idx, kth = oracle.topk(Q, C, w.B, w.k)
    exact, exempt = parity.routing_check(oracle, npi(out["idx"]).reshape(-1, w.k),
                                         ref_idx.reshape(-1, w.k), kth.reshape(-1), Q, C, w.B)
    assert exempt < 0.01
    rO, rlse = oracle.attn_fwd(Q, K, V, ref_idx, w.B, w.scale)
    assert np.abs(np64(out["O"]).reshape(-1, w.d) - rO.reshape(-1, w.d))[exact].max() < 1e-4
    assert np.abs(np64(out["lse"]).reshape(-1) - rlse.reshape(-1))[exact].max() < 1e-4


@pytest.mark.parametrize("flags", [pytest.param(0, id="default"),
                                   pytest.param(binding.FLAG_QUERY_TILES, id="tiles")])
def test_config2_bf16_forward(oracle, flags):
    """(by default the library runs this shape on the key-block-major kernels)"""
    w = workloads.CONFIGS[2]
    t, out = run_gpu(w, flags)
    rng = np.random.default_rng(2)
    for s in (0, 9, 15):
        print(w.name, s, check_slice(oracle, w, t, out, s, 1024, [], rng), flush=True)


def test_config3_bf16_forward_backward(oracle):
    """The headline shape: N = 32768, B = 32, top-k 64."""
    w = workloads.CONFIGS[3]
    t, out = run_gpu(w)
    rng = np.random.default_rng(3)
    print(w.name, 5, check_slice(oracle, w, t, out, 5, 768, [0, 1, 63, 64, 300, 777, 1022, 1023], rng),
          flush=True)
    for s in (0, 15):
        print(w.name, s, check_slice(oracle, w, t, out, s, 1024, [], rng), flush=True)


def test_config5_skewed_routing(oracle):
    """Planted hot blocks: a few key blocks are kept by most later queries."""
    w = workloads.CONFIGS[5]
    t, out = run_gpu(w)
    rng = np.random.default_rng(5)
    s = 18
    b, h = divmod(s, w.heads)
    lens = np.diff(out["off"][b, h].cpu().numpy())
    hot = np.argsort(-lens)[:3]
    assert lens[hot].min() > 3 * lens.mean()              # the workload really is skewed
    blocks = sorted(set(int(x) for x in hot) | {0, 100, w.n - 1})
    print(w.name, s, check_slice(oracle, w, t, out, s, 768, blocks, rng), flush=True)
    print(w.name, 0, check_slice(oracle, w, t, out, 0, 1024, [], rng), flush=True)


def test_config4_conv_long_sequence(oracle):
    """N = 131072, d = 128, key convolution: 64-bit indexing, 2 GiB of inputs."""
    w = workloads.CONFIGS[4]
    t, out = run_gpu(w)
    rng = np.random.default_rng(4)
    for s in (0, 11):
        print(w.name, s, check_slice(oracle, w, t, out, s, 512, [], rng), flush=True)


def test_latency_sweep_shape_key_major(oracle):
    """The paper's latency-sweep shape at N = 65536 (batch 2, 16 heads, B = 128, top-k 8), where
    the library picks the key-block-major forward and dQ kernels by itself."""
    w = workloads.Workload("sweep_N65536", 2, 16, 65536, 64, 128, 8, backward=True, seed=9100)
    t, out = run_gpu(w)
    rng = np.random.default_rng(6)
    print(w.name, 21, check_slice(oracle, w, t, out, 21, 768, [0, 1, 7, 8, 200, 511], rng), flush=True)
    for s in (0, 31):
        print(w.name, s, check_slice(oracle, w, t, out, s, 1024, [], rng), flush=True)


def test_long_sequence_slice_after_slice(oracle):
    """N = 131072 of the sweep's shape with three heads: Q and dO of a slice take 32 MB, from where
    on the key-block-major dQ kernel and the dK/dV kernel work through one slice at a time over
    the whole chip instead of one slice per XCD (the forward does at the config-4 shape)."""
    w = workloads.Workload("sweep_N131072_h3", 1, 3, 131072, 64, 128, 8, backward=True, seed=9200)
    t, out = run_gpu(w)
    rng = np.random.default_rng(8)
    print(w.name, 1, check_slice(oracle, w, t, out, 1, 768, [0, 3, 500, 1023], rng), flush=True)
    for s in (0, 2):
        print(w.name, s, check_slice(oracle, w, t, out, s, 512, [], rng), flush=True)


def test_config4_conv_backward(oracle):
    """Backward of the key convolution at the config-4 shape (1024 chunks of 128 rows per slice,
    row offsets beyond 2^31 bytes): two whole slices against the oracle.  The weights are per
    head and config 4 has batch 1, so every head's dw comes from exactly one slice."""
    w = workloads.CONFIGS[4]
    t = workloads.generate(w)
    G = torch.randn(t["K"].shape, generator=torch.Generator().manual_seed(44)).to(t["K"].dtype)
    dK, dw = moba.key_conv_backward(shape_of(w), t["K"].cuda(), t["conv_w"].cuda(), G.cuda())
    torch.cuda.synchronize()
    for s in (0, 13):
        K1 = workloads.to_f64(t["K"][:, s:s + 1])
        G1 = workloads.to_f64(G[:, s:s + 1])
        ref_dK, ref_dw = oracle.key_conv_bwd(K1, t["conv_w"][s:s + 1].double().numpy(), G1, 1)
        got = slice64(dK, s, w.heads)
        assert (np.abs(got - ref_dK) <= 2.0 ** -8 * np.abs(ref_dK) + 1e-5).all()
        assert parity.rel_l2(dw[s:s + 1].double().cpu().numpy(), ref_dw) < 1e-5
        print(w.name, "conv backward, slice", s, "ok", flush=True)
