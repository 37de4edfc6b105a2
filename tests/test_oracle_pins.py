"""Pins of the CPU oracle against things other than itself: brute force with an
explicit mask, textbook / library causal attention, closed forms, invariants,
finite differences and autograd.  None of these tests touches the GPU."""
import itertools
import os

import numpy as np
import pytest
import torch

from tests import brute

RNG = np.random.default_rng


def _rand(seed, N, d, bh=1):
    r = RNG(seed)
    return (r.standard_normal((bh, N, d)), r.standard_normal((bh, N, d)),
            r.standard_normal((bh, N, d)))


def _sets(idx_row):
    return set(int(x) for x in idx_row if x >= 0)


# ---------------------------------------------------------------- ragged sequences by zero padding

@pytest.mark.parametrize("N,B,k", [(37, 8, 2), (50, 4, 3), (23, 8, 5), (9, 16, 2), (64, 8, 0)])
def test_zero_padded_sequence_equals_the_ragged_definition(oracle, N, B, k):
    """The reading used for a ragged last block (training-shaped calls with caller-side padding,
    the decode call, packed variable-length batches): run the operator on the sequence padded with
    zero rows to the next multiple of B and keep the real rows.  A query never sees a later key,
    the padded block is never a routing candidate of a real query, and zero dO rows add nothing to
    dK and dV -- so the result must equal a dense evaluation of the ragged sequence itself."""
    d = 8
    Np = -(-N // B) * B
    r = RNG(4000 + N)
    Q, K, V, dO = (r.standard_normal((1, N, d)) for _ in range(4))
    pad = lambda x: np.concatenate([x, np.zeros((1, Np - N, d))], axis=1)
    scale = 1.0 / np.sqrt(d)
    res = oracle.moba_forward(pad(Q), pad(K), pad(V), B, k, scale)
    mask, chosen = brute.ragged_block_mask(Q[0], K[0], B, k)
    for t in range(N):
        assert _sets(res["idx"][0, t]) == chosen[t], t
    O, lse, _ = brute.dense_attention(Q[0], K[0], V[0], mask, scale)
    np.testing.assert_allclose(res["O"][0, :N], O, rtol=0, atol=1e-12)
    np.testing.assert_allclose(res["lse"][0, :N], lse, rtol=0, atol=1e-12)
    gQ, gK, gV = oracle.attn_bwd(pad(Q), pad(K), pad(V), res["idx"], pad(dO), B, scale)
    rQ, rK, rV = brute.dense_backward(Q[0], K[0], V[0], mask, scale, dO[0])
    np.testing.assert_allclose(gQ[0, :N], rQ, rtol=0, atol=1e-11)
    np.testing.assert_allclose(gK[0, :N], rK, rtol=0, atol=1e-11)
    np.testing.assert_allclose(gV[0, :N], rV, rtol=0, atol=1e-11)
    assert not gK[0, N:].any() and not gV[0, N:].any()      # the padded rows receive nothing


def test_packed_variable_length_batch_is_each_sequence_on_its_own(oracle):
    """moba_forward_varlen / attn_varlen against a dense evaluation of every ragged sequence by
    itself (lengths below, equal to and above multiples of B, one shorter than a block, one empty)."""
    B, k, d, bh = 4, 2, 8, 2
    lens = [13, 4, 0, 3, 22, 8]
    offs = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(offs[-1])
    r = RNG(515)
    Q, K, V, dO = (r.standard_normal((bh, T, d)) for _ in range(4))
    scale = 1.0 / np.sqrt(d)
    res = oracle.moba_forward_varlen(Q, K, V, offs, B, k, scale)
    O2, lse2, gQ, gK, gV = oracle.attn_varlen(Q, K, V, res["idx"], dO, offs, B, scale)
    np.testing.assert_allclose(O2, res["O"], rtol=0, atol=1e-13)
    for s in range(bh):
        for lo, hi in zip(offs[:-1], offs[1:]):
            if hi == lo:
                continue
            mask, chosen = brute.ragged_block_mask(Q[s, lo:hi], K[s, lo:hi], B, k)
            for t in range(hi - lo):
                assert _sets(res["idx"][s, lo + t]) == chosen[t], (s, lo, t)
            O, lse, _ = brute.dense_attention(Q[s, lo:hi], K[s, lo:hi], V[s, lo:hi], mask, scale)
            np.testing.assert_allclose(res["O"][s, lo:hi], O, rtol=0, atol=1e-12)
            np.testing.assert_allclose(res["lse"][s, lo:hi], lse, rtol=0, atol=1e-12)
            rQ, rK, rV = brute.dense_backward(Q[s, lo:hi], K[s, lo:hi], V[s, lo:hi], mask, scale, dO[s, lo:hi])
            np.testing.assert_allclose(gQ[s, lo:hi], rQ, rtol=0, atol=1e-11)
            np.testing.assert_allclose(gK[s, lo:hi], rK, rtol=0, atol=1e-11)
            np.testing.assert_allclose(gV[s, lo:hi], rV, rtol=0, atol=1e-11)


# ---------------------------------------------------------------- brute force

@pytest.mark.parametrize("B,d", [(1, 4), (2, 4), (4, 8), (8, 8)])
def test_forward_matches_brute_force(oracle, B, d):
    N = 32 if B < 8 else 64
    n = N // B
    for seed, k in itertools.product(range(3), sorted({0, 1, 2, 3, n // 2, n - 1, n})):
        Q, K, V = _rand(100 * seed + k, N, d)
        scale = 1.0 / np.sqrt(d)
        res = oracle.moba_forward(Q, K, V, B, k, scale)
        mask, chosen = brute.block_mask(Q[0], K[0], B, k)
        for t in range(N):
            assert _sets(res["idx"][0, t]) == chosen[t], (seed, k, t)
        O, lse, _ = brute.dense_attention(Q[0], K[0], V[0], mask, scale)
        np.testing.assert_allclose(res["O"][0], O, rtol=0, atol=1e-12)
        np.testing.assert_allclose(res["lse"][0], lse, rtol=0, atol=1e-12)


@pytest.mark.parametrize("B,d,k", [(2, 4, 2), (4, 8, 3), (8, 4, 1), (4, 4, 0), (1, 4, 5)])
def test_backward_matches_brute_force(oracle, B, d, k):
    N = 32
    for seed in range(3):
        Q, K, V = _rand(7 + seed, N, d)
        dO = RNG(99 + seed).standard_normal((1, N, d))
        scale = 1.0 / np.sqrt(d)
        res = oracle.moba_forward(Q, K, V, B, k, scale)
        dQ, dK, dV = oracle.attn_bwd(Q, K, V, res["idx"], dO, B, scale)
        mask, _ = brute.block_mask(Q[0], K[0], B, k)
        bQ, bK, bV = brute.dense_backward(Q[0], K[0], V[0], mask, scale, dO[0])
        np.testing.assert_allclose(dQ[0], bQ, rtol=0, atol=1e-11)
        np.testing.assert_allclose(dK[0], bK, rtol=0, atol=1e-11)
        np.testing.assert_allclose(dV[0], bV, rtol=0, atol=1e-11)


# ------------------------------------------------- reductions to causal attention

def _sdpa_causal(Q, K, V, scale):
    q, k, v = (torch.from_numpy(x)[None] for x in (Q, K, V))
    return torch.nn.functional.scaled_dot_product_attention(
        q, k, v, is_causal=True, scale=scale)[0].numpy()


@pytest.mark.parametrize("B,k_extra", [(4, 0), (8, 3), (16, 100)])
def test_all_past_blocks_kept_is_full_causal_attention(oracle, B, k_extra):
    N, d = 64, 8
    Q, K, V = _rand(3, N, d, bh=2)
    k = N // B - 1 + k_extra
    scale = 0.37
    res = oracle.moba_forward(Q, K, V, B, k, scale)
    for s in range(2):
        np.testing.assert_allclose(res["O"][s], _sdpa_causal(Q[s], K[s], V[s], scale),
                                   rtol=0, atol=1e-12)


def test_single_block_is_full_causal_attention(oracle):
    N, d = 48, 8
    Q, K, V = _rand(4, N, d)
    res = oracle.moba_forward(Q, K, V, N, 5, 0.5)
    np.testing.assert_allclose(res["O"][0], _sdpa_causal(Q[0], K[0], V[0], 0.5), atol=1e-12)
    assert (res["idx"] == -1).all()


def test_k0_is_block_diagonal_causal_attention(oracle):
    N, d, B = 64, 8, 16
    Q, K, V = _rand(5, N, d)
    res = oracle.moba_forward(Q, K, V, B, 0, 0.3)
    for j in range(N // B):
        sl = slice(j * B, (j + 1) * B)
        np.testing.assert_allclose(res["O"][0, sl], _sdpa_causal(Q[0, sl], K[0, sl], V[0, sl], 0.3),
                                   atol=1e-12)


def test_lse_is_log_sum_exp_of_scaled_logits(oracle):
    N, d, B, k = 64, 8, 8, 3
    Q, K, V = _rand(6, N, d)
    scale = 0.25
    res = oracle.moba_forward(Q, K, V, B, k, scale)
    mask, _ = brute.block_mask(Q[0], K[0], B, k)
    S = scale * Q[0] @ K[0].T
    for t in range(N):
        assert abs(res["lse"][0, t] - np.log(np.exp(S[t][mask[t]]).sum())) < 1e-12


def test_probabilities_sum_to_one_and_blockwise_merge(oracle):
    """V = ones gives O = 1 (rows of P sum to one).  And the one-shot softmax equals
    per-block partial softmaxes merged by their log-sum-exp, the identity a split
    GPU evaluation relies on."""
    N, d, B, k = 64, 8, 8, 3
    Q, K, V = _rand(8, N, d)
    scale = 0.4
    res = oracle.moba_forward(Q, K, np.ones_like(V), B, k, scale)
    np.testing.assert_allclose(res["O"], 1.0, atol=1e-13)
    res = oracle.moba_forward(Q, K, V, B, k, scale)
    for t in (9, 37, 63):
        own = t // B
        parts = []
        for blk in sorted(_sets(res["idx"][0, t])) + [own]:
            hi = (blk + 1) * B if blk != own else t + 1
            z = scale * K[0, blk * B:hi] @ Q[0, t]
            lse_p = np.log(np.exp(z).sum())
            parts.append((lse_p, np.exp(z - lse_p) @ V[0, blk * B:hi]))
        lse = np.log(sum(np.exp(p[0]) for p in parts))
        O = sum(np.exp(p[0] - lse) * p[1] for p in parts)
        np.testing.assert_allclose(res["O"][0, t], O, atol=1e-12)
        assert abs(res["lse"][0, t] - lse) < 1e-12


# ------------------------------------------------------ centroids and selection

def test_block_size_one_selects_top_keys(oracle):
    """B = 1: the centroid is the key itself (up to the fp32 store), so MoBA keeps the
    k past keys with the largest q.k plus the query's own key."""
    N, d, k = 24, 4, 3
    r = RNG(11)
    # values exactly representable in fp32 so the stored centroid is the key
    Q = r.integers(-8, 9, (1, N, d)).astype(np.float64) / 4
    K = r.integers(-8, 9, (1, N, d)).astype(np.float64) / 4 + np.arange(N)[None, :, None] * 2.0 ** -10
    V = r.standard_normal((1, N, d))
    res = oracle.moba_forward(Q, K, V, 1, k, 0.5)
    np.testing.assert_array_equal(res["centroids"], K)
    for t in range(N):
        s = K[0, :t] @ Q[0, t]
        order = sorted(range(t), key=lambda j: (-s[j], j))[:k]
        assert _sets(res["idx"][0, t]) == set(order)
        keys = order + [t]
        z = 0.5 * K[0, keys] @ Q[0, t]
        p = np.exp(z - z.max())
        p /= p.sum()
        np.testing.assert_allclose(res["O"][0, t], p @ V[0, keys], atol=1e-12)


def test_planted_scores_closed_form(oracle):
    """Keys of block j all equal a_j * e1 and q = e1, so the gate score of block j
    is a_j exactly and the kept set is known in closed form."""
    B, d, n, k = 4, 8, 10, 3
    N = B * n
    a = np.array([3, -1, 7, 0, 5, 9, 2, 8, -4, 6], dtype=np.float64)
    K = np.zeros((1, N, d))
    K[0, :, 0] = np.repeat(a, B)
    Q = np.zeros((1, N, d))
    Q[0, :, 0] = 1.0
    C = oracle.centroids(K, B)
    np.testing.assert_array_equal(C[0, :, 0], a)
    idx, kth = oracle.topk(Q, C, B, k)
    for t in range(N):
        own = t // B
        want = sorted(range(own), key=lambda j: -a[j])[:k]
        assert list(idx[0, t, :len(want)]) == want          # best first
        assert (idx[0, t, len(want):] == -1).all()
        if want:
            assert kth[0, t] == a[want[-1]]
        else:
            assert np.isnan(kth[0, t])


def test_zero_keys_tie_break_and_mean_of_values(oracle):
    """K = 0: every gate score is 0, so the lowest indices win, and every logit is 0,
    so O is the plain mean of V over the kept blocks and the own prefix."""
    N, d, B, k = 48, 4, 4, 3
    r = RNG(12)
    Q = r.standard_normal((1, N, d))
    V = r.standard_normal((1, N, d))
    K = np.zeros((1, N, d))
    res = oracle.moba_forward(Q, K, V, B, k, 0.5)
    for t in range(N):
        own = t // B
        keep = list(range(min(k, own)))
        assert list(res["idx"][0, t, :len(keep)]) == keep
        rows = [u for j in keep for u in range(j * B, (j + 1) * B)] + list(range(own * B, t + 1))
        np.testing.assert_allclose(res["O"][0, t], V[0, rows].mean(axis=0), atol=1e-13)
        assert abs(res["lse"][0, t] - np.log(len(rows))) < 1e-13


def test_duplicated_blocks_lower_index_wins(oracle):
    N, d, B, k = 64, 8, 8, 2
    Q, K, V = _rand(13, N, d)
    K[0, 3 * B:4 * B] = K[0, 1 * B:2 * B]      # block 3 is a copy of block 1
    K[0, 5 * B:6 * B] = K[0, 1 * B:2 * B]      # so is block 5
    C = oracle.centroids(K, B)
    idx, _ = oracle.topk(Q, C, B, k)
    rows = np.arange(N, dtype=np.int64)
    S = oracle.gate_scores(Q, C, rows, B)
    seen = 0
    for t in range(6 * B, N):
        sel = _sets(idx[0, t])
        # the kept copies must be a prefix of (1, 3, 5): a higher copy is never kept
        # while a lower, bit-identical one is left out
        assert sorted(sel & {1, 3, 5}) in ([], [1], [1, 3])
        seen += len(sel & {1, 3, 5}) > 0
        assert S[t, 1] == S[t, 3] == S[t, 5]
    assert seen > 0


def test_topk_agrees_with_stable_argsort_of_gate_scores(oracle):
    N, d, B, k = 96, 8, 4, 5
    Q, K, V = _rand(14, N, d, bh=2)
    C = oracle.centroids(K, B)
    idx, kth = oracle.topk(Q, C, B, k)
    S = oracle.gate_scores(Q, C, np.arange(2 * N, dtype=np.int64), B).reshape(2, N, N // B)
    for s in range(2):
        for t in range(N):
            own = t // B
            assert np.isneginf(S[s, t, own:]).all()
            ref = S[s, t, :own]
            np.testing.assert_allclose(ref, C[s, :own] @ Q[s, t], atol=1e-12)
            order = np.argsort(-ref, kind="stable")[:k]
            assert list(idx[s, t, :len(order)]) == list(order)


def test_centroid_is_block_mean_in_fp32(oracle):
    N, d, B = 64, 8, 16
    K = RNG(15).standard_normal((2, N, d))
    C = oracle.centroids(K, B)
    ref = K.reshape(2, N // B, B, d).mean(axis=2)
    np.testing.assert_array_equal(C, ref.astype(np.float32).astype(np.float64))


# ------------------------------------------------------------------ values

def test_constant_values_and_in_block_permutation(oracle):
    N, d, B, k = 64, 8, 8, 3
    Q, K, V = _rand(16, N, d)
    row = np.arange(d, dtype=np.float64)
    res = oracle.moba_forward(Q, K, np.broadcast_to(row, V.shape).copy(), B, k, 0.3)
    np.testing.assert_allclose(res["O"], np.broadcast_to(row, V.shape), atol=1e-12)
    # permuting keys and values together inside block 2 leaves the outputs of every
    # query beyond block 2 unchanged (the centroid does not change either)
    perm = RNG(17).permutation(B) + 2 * B
    K2, V2 = K.copy(), V.copy()
    K2[0, 2 * B:3 * B] = K[0, perm]
    V2[0, 2 * B:3 * B] = V[0, perm]
    a = oracle.moba_forward(Q, K, V, B, k, 0.3)
    b = oracle.moba_forward(Q, K2, V2, B, k, 0.3)
    np.testing.assert_allclose(a["O"][0, 3 * B:], b["O"][0, 3 * B:], atol=1e-12)
    assert (np.sort(a["idx"][0, 3 * B:], axis=-1) == np.sort(b["idx"][0, 3 * B:], axis=-1)).mean() > 0.98


# ------------------------------------------------------------------- conv

def test_conv_zero_weights_and_width_one(oracle):
    N, d, heads = 40, 6, 2
    K = RNG(18).standard_normal((4, N, d))
    Kp = oracle.key_conv(K, np.zeros((heads, d, 3)), heads, oracle.ROUND_NONE)
    np.testing.assert_array_equal(Kp, K)              # SiLU(0) = 0
    w = RNG(19).standard_normal((heads, d, 1))
    Kp = oracle.key_conv(K, w, heads, oracle.ROUND_NONE)
    for s in range(4):
        a = K[s] * w[s % heads, :, 0]
        np.testing.assert_allclose(Kp[s], K[s] + a / (1 + np.exp(-a)), atol=1e-13)


@pytest.mark.parametrize("W", [2, 3, 4, 5])
def test_conv_matches_torch_depthwise_conv1d(oracle, W):
    N, d, heads, batch = 50, 8, 3, 2
    K = RNG(20 + W).standard_normal((batch * heads, N, d))
    w = RNG(30 + W).standard_normal((heads, d, W)) * 0.5
    Kp = oracle.key_conv(K, w, heads, oracle.ROUND_NONE)
    for s in range(batch * heads):
        x = torch.from_numpy(K[s].T.copy())[None]                 # [1, d, N]
        # conv1d is a correlation: output[t] = sum_j weight[j] * x_padded[t + j]; with
        # W-1 zeros on the left, weight[j] multiplies x[t - (W-1-j)], so lag l = W-1-j
        wt = torch.from_numpy(w[s % heads][:, ::-1].copy())[:, None, :]
        y = torch.nn.functional.conv1d(torch.nn.functional.pad(x, (W - 1, 0)), wt, groups=d)
        ref = x + torch.nn.functional.silu(y)
        np.testing.assert_allclose(Kp[s], ref[0].numpy().T, atol=1e-12)


def test_conv_is_causal_and_rounds_to_io_type(oracle):
    N, d = 32, 4
    K = RNG(40).standard_normal((1, N, d))
    w = RNG(41).standard_normal((1, d, 4))
    a = oracle.key_conv(K, w, 1, oracle.ROUND_NONE)
    K2 = K.copy()
    K2[0, 20:] += 1.0
    b = oracle.key_conv(K2, w, 1, oracle.ROUND_NONE)
    np.testing.assert_array_equal(a[0, :20], b[0, :20])
    r = oracle.key_conv(K, w, 1, oracle.ROUND_BF16)
    np.testing.assert_array_equal(r, oracle.round_io(a, oracle.ROUND_BF16))
    t = torch.from_numpy(r).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(t, r)                # already bf16 values


@pytest.mark.parametrize("W", [1, 3, 4, 5])
def test_conv_backward_matches_torch_autograd(oracle, W):
    """Appendix B, backward through the convolution: dK and dw against autograd on the
    library formulation (left-padded depthwise conv1d + SiLU + residual), weights shared
    across the batch."""
    N, d, heads, batch = 37, 6, 2, 3
    K = RNG(60 + W).standard_normal((batch * heads, N, d))
    w = RNG(70 + W).standard_normal((heads, d, W)) * 0.5
    G = RNG(80 + W).standard_normal((batch * heads, N, d))
    dK, dw = oracle.key_conv_bwd(K, w, G, heads)
    Kt = torch.from_numpy(K).requires_grad_(True)
    wt = torch.from_numpy(w).requires_grad_(True)
    loss = 0.0
    for s in range(batch * heads):
        x = Kt[s].T[None]                                             # [1, d, N]
        y = torch.nn.functional.conv1d(torch.nn.functional.pad(x, (W - 1, 0)),
                                       wt[s % heads].flip(-1)[:, None, :], groups=d)
        loss = loss + ((x + torch.nn.functional.silu(y))[0].T * torch.from_numpy(G[s])).sum()
    loss.backward()
    np.testing.assert_allclose(dK, Kt.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(dw, wt.grad.numpy(), atol=1e-10)


def test_conv_backward_finite_differences_and_closed_forms(oracle):
    N, d, heads, W = 12, 3, 2, 3
    K = RNG(90).standard_normal((heads, N, d))
    w = RNG(91).standard_normal((heads, d, W)) * 0.7
    G = RNG(92).standard_normal((heads, N, d))
    dK, dw = oracle.key_conv_bwd(K, w, G, heads)
    f = lambda K_, w_: (oracle.key_conv(K_, w_, heads, oracle.ROUND_NONE) * G).sum()
    eps = 1e-6
    for idx in [(0, 0, 0), (1, 5, 2), (0, N - 1, 1), (1, N - 2, 0)]:     # incl. the last rows
        Kp, Km = K.copy(), K.copy()
        Kp[idx] += eps
        Km[idx] -= eps
        assert abs((f(Kp, w) - f(Km, w)) / (2 * eps) - dK[idx]) < 1e-7
    for idx in [(0, 0, 0), (1, 2, 2), (0, 1, 1)]:
        wp, wm = w.copy(), w.copy()
        wp[idx] += eps
        wm[idx] -= eps
        assert abs((f(K, wp) - f(K, wm)) / (2 * eps) - dw[idx]) < 1e-7
    # w = 0: a = 0, SiLU'(0) = 1/2, so dK = G and dw[l] = sum_t G[t]/2 * K[t-l]
    dK0, dw0 = oracle.key_conv_bwd(K, np.zeros_like(w), G, heads)
    np.testing.assert_allclose(dK0, G, atol=1e-14)
    for l in range(W):
        np.testing.assert_allclose(dw0[:, :, l], 0.5 * (G[:, l:] * K[:, :N - l]).sum(1), atol=1e-13)
    # G = 0: no gradient at all
    z = oracle.key_conv_bwd(K, w, np.zeros_like(G), heads)
    assert not z[0].any() and not z[1].any()


def test_bf16_rounding_matches_torch(oracle):
    x = torch.randn(200000, generator=torch.Generator().manual_seed(1)) * 37.0
    x[:1000] *= 1e-38                                   # reach the subnormal range
    x[1000:2000] *= 1e30
    ref = x.to(torch.bfloat16).to(torch.float64).numpy()
    got = oracle.round_io(x.to(torch.float64).numpy(), oracle.ROUND_BF16)
    np.testing.assert_array_equal(got, ref)
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert oracle.round_io(np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8]), oracle.ROUND_BF16).tolist() \
        == [1.0, 1 + 2.0 ** -6]


# ----------------------------------------------------------------- backward

def test_backward_matches_finite_differences(oracle):
    N, d, B, k = 24, 4, 4, 2
    Q, K, V = _rand(50, N, d)
    dO = RNG(51).standard_normal((1, N, d))
    scale = 0.5
    idx = oracle.moba_forward(Q, K, V, B, k, scale)["idx"]     # held fixed below

    def loss(q, kk, v):
        O, _ = oracle.attn_fwd(q, kk, v, idx, B, scale)
        return float((O * dO).sum())

    dQ, dK, dV = oracle.attn_bwd(Q, K, V, idx, dO, B, scale)
    eps = 1e-6
    r = RNG(52)
    for which, grad in (("Q", dQ), ("K", dK), ("V", dV)):
        for _ in range(12):
            t, c = int(r.integers(N)), int(r.integers(d))
            args = {"Q": Q.copy(), "K": K.copy(), "V": V.copy()}
            args[which][0, t, c] += eps
            up = loss(args["Q"], args["K"], args["V"])
            args[which][0, t, c] -= 2 * eps
            dn = loss(args["Q"], args["K"], args["V"])
            assert abs((up - dn) / (2 * eps) - grad[0, t, c]) < 1e-7, (which, t, c)


def test_backward_matches_autograd_on_dense_mask(oracle):
    N, d, B, k = 64, 8, 8, 3
    Q, K, V = _rand(53, N, d, bh=2)
    dO = RNG(54).standard_normal((2, N, d))
    scale = 1 / np.sqrt(d)
    idx = oracle.moba_forward(Q, K, V, B, k, scale)["idx"]
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, idx, dO, B, scale)
    for s in range(2):
        mask = np.zeros((N, N), dtype=bool)
        for t in range(N):
            for j in _sets(idx[s, t]):
                mask[t, j * B:(j + 1) * B] = True
            mask[t, (t // B) * B:t + 1] = True
        q, kk, v = (torch.tensor(x[s], requires_grad=True) for x in (Q, K, V))
        S = scale * q @ kk.T
        S = S.masked_fill(~torch.from_numpy(mask), float("-inf"))
        O = torch.softmax(S, dim=-1) @ v
        (O * torch.from_numpy(dO[s])).sum().backward()
        np.testing.assert_allclose(dQ[s], q.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dK[s], kk.grad.numpy(), atol=1e-12)
        np.testing.assert_allclose(dV[s], v.grad.numpy(), atol=1e-12)


def test_grouped_query_heads_share_keys_and_sum_gradients(oracle):
    """Appendix C, last paragraph.  Forward: each query head against the key/value head
    h // G, by brute force with an explicit mask.  Gradients of the shared heads: torch's
    autograd through repeat_interleave (whose backward is that sum), and finite
    differences of the whole shared-head loss."""
    b, H, Hkv, N, d, B, k = 2, 6, 2, 32, 4, 4, 2
    G = H // Hkv
    r = RNG(70)
    Q = r.standard_normal((b * H, N, d))
    K = r.standard_normal((b * Hkv, N, d))
    V = r.standard_normal((b * Hkv, N, d))
    dO = r.standard_normal((b * H, N, d))
    scale = 0.5
    # the remap itself, against explicit indexing, and G = 1 is the identity
    Ke, Ve = oracle.gqa_expand(K, H, Hkv), oracle.gqa_expand(V, H, Hkv)
    for bb in range(b):
        for h in range(H):
            assert np.array_equal(Ke[bb * H + h], K[bb * Hkv + h // G])
    assert np.array_equal(oracle.gqa_expand(K, Hkv, Hkv), K)
    assert np.array_equal(oracle.gqa_reduce(Ke, Hkv * 1, Hkv)[0], Ke[0])
    res = oracle.moba_forward(Q, Ke, Ve, B, k, scale)
    for bb in range(b):
        for h in range(H):
            s, skv = bb * H + h, bb * Hkv + h // G
            mask, chosen = brute.block_mask(Q[s], K[skv], B, k)
            assert all(_sets(res["idx"][s, t]) == chosen[t] for t in range(N))
            O, lse, _ = brute.dense_attention(Q[s], K[skv], V[skv], mask, scale)
            np.testing.assert_allclose(res["O"][s], O, rtol=0, atol=1e-12)
    idx = res["idx"]
    dQ, dKe, dVe = oracle.attn_bwd(Q, Ke, Ve, idx, dO, B, scale)
    dK, dV = oracle.gqa_reduce(dKe, H, Hkv), oracle.gqa_reduce(dVe, H, Hkv)
    # the sum over sharing heads is the backward of the copy
    x = torch.tensor(K.reshape(b, Hkv, N, d), requires_grad=True)
    (x.repeat_interleave(G, dim=1) * torch.from_numpy(dKe.reshape(b, H, N, d))).sum().backward()
    np.testing.assert_allclose(dK.reshape(b, Hkv, N, d), x.grad.numpy(), atol=1e-12)

    def loss(kk, vv):
        O, _ = oracle.attn_fwd(Q, oracle.gqa_expand(kk, H, Hkv), oracle.gqa_expand(vv, H, Hkv), idx, B, scale)
        return float((O * dO).sum())

    eps = 1e-6
    for which, grad in (("K", dK), ("V", dV)):
        for _ in range(10):
            s, t, c = int(r.integers(b * Hkv)), int(r.integers(N)), int(r.integers(d))
            args = {"K": K.copy(), "V": V.copy()}
            args[which][s, t, c] += eps
            up = loss(args["K"], args["V"])
            args[which][s, t, c] -= 2 * eps
            dn = loss(args["K"], args["V"])
            assert abs((up - dn) / (2 * eps) - grad[s, t, c]) < 2e-7, (which, s, t, c)


def test_backward_invariants(oracle):
    N, d, B, k = 32, 4, 4, 2
    Q, K, V = _rand(55, N, d)
    dO = RNG(56).standard_normal((1, N, d))
    idx = oracle.moba_forward(Q, K, V, B, k, 0.5)["idx"]
    z = oracle.attn_bwd(Q, K, V, idx, np.zeros_like(dO), B, 0.5)
    assert all((g == 0).all() for g in z)
    # rows of dS sum to zero, so shifting every value row by one vector changes
    # neither dQ nor dK, and dV does not depend on V at all
    a = oracle.attn_bwd(Q, K, V, idx, dO, B, 0.5)
    b = oracle.attn_bwd(Q, K, V + np.arange(d), idx, dO, B, 0.5)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, atol=1e-11)
    # column sums of P: sum_u dV_u = sum_t dO_t because each row of P sums to one
    np.testing.assert_allclose(a[2].sum(axis=1), dO.sum(axis=1), atol=1e-12)


def test_sampled_rows_and_blocks_equal_full_evaluation(oracle):
    N, d, B, k = 64, 8, 8, 3
    Q, K, V = _rand(57, N, d, bh=2)
    dO = RNG(58).standard_normal((2, N, d))
    idx = oracle.moba_forward(Q, K, V, B, k, 0.3)["idx"]
    O, lse = oracle.attn_fwd(Q, K, V, idx, B, 0.3)
    rows = np.array([0, 5, 63, 64, 100, 127], dtype=np.int64)
    Or, lr = oracle.attn_fwd(Q, K, V, idx, B, 0.3, rows=rows)
    np.testing.assert_array_equal(Or, O.reshape(-1, d)[rows])
    np.testing.assert_array_equal(lr, lse.reshape(-1)[rows])
    dQ, dK, dV = oracle.attn_bwd(Q, K, V, idx, dO, B, 0.3)
    Dv = (dO * O).sum(-1)
    off, ql = oracle.csr(idx, B)
    np.testing.assert_array_equal(
        oracle.attn_bwd_dq(Q, K, V, idx, dO, lse, Dv, B, 0.3, rows=rows), dQ.reshape(-1, d)[rows])
    blocks = np.array([0, 3, 7, 8, 15], dtype=np.int64)
    bK, bV = oracle.attn_bwd_dkdv(Q, K, V, dO, lse, Dv, off, ql, B, 0.3, blocks=blocks)
    np.testing.assert_array_equal(bK, dK.reshape(-1, B, d)[blocks])
    np.testing.assert_array_equal(bV, dV.reshape(-1, B, d)[blocks])


# --------------------------------------------------------------------- lists

def test_csr_lists(oracle):
    N, d, B, k = 96, 8, 8, 4
    Q, K, V = _rand(60, N, d, bh=3)
    idx = oracle.moba_forward(Q, K, V, B, k, 0.3)["idx"]
    off, ql = oracle.csr(idx, B)
    n = N // B
    R = oracle.routes_per_slice(N, B, k)
    assert R == B * sum(min(c, k) for c in range(n)) == ql.shape[1]
    for s in range(3):
        assert off[s, 0] == 0 and off[s, n] == R
        for j in range(n):
            want = [t for t in range(N) if j in _sets(idx[s, t])]
            assert list(ql[s, off[s, j]:off[s, j + 1]]) == want


# ------------------------------------------------------------- paper's numbers

def test_paper_sparsity_identity():
    """Section 2 / Section 6 of the paper: at N = 8192 the (B, k) pairs (512, 2),
    (256, 4), (128, 8) all keep 1/8 of the blocks ("sparsity 7/8", "12.5 % of the
    computation").  The fixture holds the paper's figures; the work counter used by
    the benchmark must reproduce them to within the extra own block."""
    import workloads
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_sparsity.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for N, B, k, frac in rows:
        N, B, k, frac = int(N), int(B), int(k), float(frac)
        assert k * B / N == frac
        pairs = workloads.attended_pairs_per_slice(N, B, k)
        # kept fraction of the N x N score matrix: k/n for the routed blocks, less the
        # k(k+1)/2 block pairs the first k blocks cannot have, plus the own-block triangle
        n = N // B
        closed = frac - k * (k + 1) / (2 * n * n) + (B + 1) / (2 * N)
        assert abs(pairs / (N * N) - closed) < 1e-12
        assert abs(pairs / (N * N) - frac) < (B + 1) / (2 * N)
        # exact count by enumeration
        ref = sum(min(t // B, k) * B + (t % B) + 1 for t in range(N))
        assert pairs == ref


def test_ragged_pair_count_is_the_size_of_the_mask():
    """The pair counter of the packed-batch benchmark against the explicit mask of a sequence
    with a short last block (tests/brute.py)."""
    import workloads
    rng = np.random.default_rng(77)
    for L, B, k in ((37, 8, 2), (64, 8, 3), (5, 8, 4), (50, 4, 20), (33, 16, 1), (40, 8, 0)):
        Q, K = rng.standard_normal((L, 8)), rng.standard_normal((L, 8))
        mask, _ = brute.ragged_block_mask(Q, K, B, k)
        assert int(mask.sum()) == workloads.ragged_pairs(L, B, k)
        if L % B == 0:
            assert workloads.ragged_pairs(L, B, k) == workloads.attended_pairs_per_slice(L, B, k)
