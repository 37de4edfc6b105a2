"""Brute-force MoBA on tiny inputs: an explicit N x N boolean mask and a dense
softmax in numpy float64.  Written independently of the oracle (different
language, dense instead of sparse evaluation, sort-based selection) so that the
two can pin each other.  Follows the paper's Section 2 definition."""
import numpy as np


def block_mask(Q, K, B, k):
    """Boolean [N, N]: mask[t, u] is True when query t attends key u."""
    N, d = Q.shape
    n = N // B
    cent = K.reshape(n, B, d).mean(axis=1).astype(np.float32).astype(np.float64)
    mask = np.zeros((N, N), dtype=bool)
    chosen = []
    for t in range(N):
        own = t // B
        cand = sorted(range(own), key=lambda j: (-float(Q[t] @ cent[j]), j))
        keep = cand[:k] if k > 0 else []
        chosen.append(set(keep))
        for j in keep:
            mask[t, j * B:(j + 1) * B] = True
        mask[t, own * B:t + 1] = True
    return mask, chosen


def dense_attention(Q, K, V, mask, scale):
    S = scale * (Q @ K.T)
    S = np.where(mask, S, -np.inf)
    m = S.max(axis=1, keepdims=True)
    E = np.exp(S - m)
    l = E.sum(axis=1, keepdims=True)
    P = E / l
    return P @ V, (m + np.log(l))[:, 0], P


def dense_backward(Q, K, V, mask, scale, dO):
    """Gradients of sum(O * dO) through the dense masked softmax, by the textbook
    softmax Jacobian (not the paper's D-vector shortcut)."""
    O, lse, P = dense_attention(Q, K, V, mask, scale)
    dV = P.T @ dO
    dP = dO @ V.T
    # dS = P o (dP - rowsum(P o dP))
    dS = P * (dP - (P * dP).sum(axis=1, keepdims=True))
    dQ = scale * dS @ K
    dK = scale * dS.T @ Q
    return dQ, dK, dV


def ragged_block_mask(Q, K, B, k):
    """The same for a sequence whose length need not be a multiple of B (paper Appendix C.1 cuts
    N keys into ceil(N / B) blocks, the last one shorter): candidates of query t are the complete
    blocks before its own, whose centroids are plain means; its own block, complete or not, is
    attended up to t."""
    N, d = Q.shape
    nfull = N // B
    cent = K[:nfull * B].reshape(nfull, B, d).mean(axis=1).astype(np.float32).astype(np.float64)
    mask = np.zeros((N, N), dtype=bool)
    chosen = []
    for t in range(N):
        own = t // B
        keep = sorted(range(own), key=lambda j: (-float(Q[t] @ cent[j]), j))[:k] if k > 0 else []
        chosen.append(set(keep))
        for j in keep:
            mask[t, j * B:(j + 1) * B] = True
        mask[t, own * B:t + 1] = True
    return mask, chosen
