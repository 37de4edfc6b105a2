"""ctypes front end of the CPU oracle (oracle/moba_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
CPU-baseline leg.  The GPU library never imports or calls anything here, and this
module imports nothing from the GPU package.

All tensors are numpy float64, row-major ``[bh, N, d]`` (batch*heads flattened).
The arithmetic lives in the C file; this module only marshals arguments, plus two
one-line numpy steps that are part of the definition:
``D = rowsum(dO * O)`` (paper Appendix C.3, backward preprocessing), the
count of routed pairs, and the head sharing of grouped-query attention written out
as a copy (forward) and a sum (gradients) -- Appendix C, last paragraph.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moba_oracle.c")
_LIB = os.path.join(_HERE, "libmoba_oracle.so")

ROUND_F32, ROUND_BF16, ROUND_NONE = 0, 1, 2


# plain -O2, no -march, no contraction, no fast-math: the checker is built to be obviously right,
# not fast (the benchmark's CPU baseline reports this line with its rate)
_CFLAGS = ["-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-fno-fast-math", "-ffp-contract=off"]
BUILD_COMMAND = "gcc " + " ".join(_CFLAGS) + " moba_oracle.c -lm"


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over independent rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc"] + _CFLAGS + ["-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_csr.restype = ctypes.c_int64
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _out(shape, dtype=np.float64):
    a = np.empty(shape, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    return int(_L().oracle_num_threads())


def routes_per_slice(N: int, B: int, k: int) -> int:
    """Number of (query, selected past block) pairs of one [N, d] slice:
    the queries of block c each keep min(c, k) past blocks."""
    n = N // B
    return B * sum(min(c, k) for c in range(n))


def round_io(x, mode):
    x, px = _f64(x)
    y, py = _out(x.shape)
    _L().oracle_round_array(px, py, ctypes.c_int64(x.size), ctypes.c_int(mode))
    return y


def key_conv(K, w, heads, round_mode):
    """Appendix B.  K [bh,N,d], w [heads,d,W] (lag-major last axis) -> K' [bh,N,d]."""
    K, pK = _f64(K)
    w, pw = _f64(w)
    bh, N, d = K.shape
    assert w.shape[0] == heads and w.shape[1] == d
    Kp, pP = _out(K.shape)
    _L().oracle_key_conv(pK, pw, pP, bh, heads, N, d, w.shape[2], round_mode)
    return Kp


def key_conv_bwd(K, w, G, heads):
    """Appendix B, backward: G = dL/dK' [bh,N,d] -> (dL/dK [bh,N,d], dL/dw [heads,d,W]); the
    rounding of K' to the storage type is taken as the identity."""
    K, pK = _f64(K)
    w, pw = _f64(w)
    G, pG = _f64(G)
    bh, N, d = K.shape
    assert w.shape[0] == heads and w.shape[1] == d and G.shape == K.shape
    dK, pdK = _out(K.shape)
    dw, pdw = _out(w.shape)
    _L().oracle_key_conv_bwd(pK, pw, pG, pdK, pdw, bh, heads, N, d, w.shape[2])
    return dK, dw


def centroids(K, B):
    """Section 2.  Mean key of each block, stored as fp32 values -> [bh, n, d]."""
    K, pK = _f64(K)
    bh, N, d = K.shape
    assert N % B == 0
    C, pC = _out((bh, N // B, d))
    _L().oracle_centroids(pK, pC, bh, N, d, B)
    return C


def gate_scores(Q, C, rows, B):
    """Gate scores of flat rows (s*N+t) against all n blocks; -inf for own/future."""
    Q, pQ = _f64(Q)
    C, pC = _f64(C)
    bh, N, d = Q.shape
    rows, pr = _i64(rows)
    S, pS = _out((rows.size, N // B))
    _L().oracle_gate_scores(pQ, pC, pr, ctypes.c_int64(rows.size), pS, N, d, B)
    return S


def topk(Q, C, B, k, rows=None):
    """Section 2 + Appendix C.1.  -> idx [bh,N,k] int32 (best first, -1 unused),
    kth [bh,N] score of the last kept block (NaN if none).  With ``rows`` (flat
    s*N+t) only those rows are evaluated: idx [nrows,k], kth [nrows]."""
    Q, pQ = _f64(Q)
    C, pC = _f64(C)
    bh, N, d = Q.shape
    full = rows is None
    rows, pr = _i64(np.arange(bh * N) if full else rows)
    idx, pi = _out((rows.size, max(k, 0)), np.int32)
    kth, pk = _out((rows.size,))
    _L().oracle_topk(pQ, pC, pr, ctypes.c_int64(rows.size), pi, pk, N, d, B, k)
    if full:
        return idx.reshape(bh, N, max(k, 0)), kth.reshape(bh, N)
    return idx, kth


def csr(idx, B):
    """Appendix C.1.  Key-block-major query lists -> off [bh,n+1], qlist [bh,R]."""
    idx, pi = _i32(idx)
    bh, N, k = idx.shape
    n = N // B
    R = routes_per_slice(N, B, k)
    off, po = _out((bh, n + 1), np.int32)
    ql, pq = _out((bh, R), np.int32)
    got = _L().oracle_csr(pi, po, pq, bh, N, B, k, ctypes.c_int64(R))
    if got != R:
        raise ValueError("routing does not keep min(c,k) blocks per query")
    return off, ql


def attn_fwd(Q, K, V, idx, B, scale, rows=None):
    """Section 2.  O [nrows,d] and lse [nrows] for flat rows (default: all, then
    shaped [bh,N,d] / [bh,N])."""
    Q, pQ = _f64(Q)
    K, pK = _f64(K)
    V, pV = _f64(V)
    idx, pi = _i32(idx)
    bh, N, d = Q.shape
    k = idx.shape[2]
    full = rows is None
    rows, pr = _i64(np.arange(bh * N) if full else rows)
    O, pO = _out((rows.size, d))
    lse, pl = _out((rows.size,))
    _L().oracle_attn_fwd(pQ, pK, pV, pi, pr, ctypes.c_int64(rows.size), pO, pl,
                         N, d, B, k, ctypes.c_double(scale))
    if full:
        return O.reshape(bh, N, d), lse.reshape(bh, N)
    return O, lse


def attn_bwd_dq(Q, K, V, idx, dO, lse, Dv, B, scale, rows=None):
    """Appendix C.3.  dQ for flat rows; lse, Dv are full [bh,N] (listed rows read)."""
    Q, pQ = _f64(Q)
    K, pK = _f64(K)
    V, pV = _f64(V)
    dO, pg = _f64(dO)
    lse, pl = _f64(lse)
    Dv, pD = _f64(Dv)
    idx, pi = _i32(idx)
    bh, N, d = Q.shape
    k = idx.shape[2]
    full = rows is None
    rows, pr = _i64(np.arange(bh * N) if full else rows)
    dQ, pq = _out((rows.size, d))
    _L().oracle_attn_bwd_dq(pQ, pK, pV, pi, pg, pl, pD, pr, ctypes.c_int64(rows.size), pq,
                            N, d, B, k, ctypes.c_double(scale))
    return dQ.reshape(bh, N, d) if full else dQ


def attn_bwd_dkdv(Q, K, V, dO, lse, Dv, off, qlist, B, scale, blocks=None):
    """Appendix C.3.  dK, dV for flat key blocks (s*n+j) -> [nblocks,B,d] each
    (default: all blocks, shaped [bh,N,d])."""
    Q, pQ = _f64(Q)
    K, pK = _f64(K)
    V, pV = _f64(V)
    dO, pg = _f64(dO)
    lse, pl = _f64(lse)
    Dv, pD = _f64(Dv)
    off, po = _i32(off)
    qlist, pql = _i32(qlist)
    bh, N, d = Q.shape
    n = N // B
    R = qlist.shape[1]
    full = blocks is None
    blocks, pb = _i64(np.arange(bh * n) if full else blocks)
    dK, pdk = _out((blocks.size, B, d))
    dV, pdv = _out((blocks.size, B, d))
    _L().oracle_attn_bwd_dkdv(pQ, pK, pV, pg, pl, pD, po, pql, ctypes.c_int64(R),
                              pb, ctypes.c_int64(blocks.size), pdk, pdv,
                              N, d, B, ctypes.c_double(scale))
    if full:
        return dK.reshape(bh, N, d), dV.reshape(bh, N, d)
    return dK, dV


def attn_bwd(Q, K, V, idx, dO, B, scale):
    """Whole backward at fixed routing: forward for (O, lse), D = rowsum(dO*O)
    (Appendix C.3, preprocessing), then dQ, dK, dV."""
    O, lse = attn_fwd(Q, K, V, idx, B, scale)
    Dv = (np.asarray(dO, dtype=np.float64) * O).sum(-1)
    off, ql = csr(idx, B)
    dQ = attn_bwd_dq(Q, K, V, idx, dO, lse, Dv, B, scale)
    dK, dV = attn_bwd_dkdv(Q, K, V, dO, lse, Dv, off, ql, B, scale)
    return dQ, dK, dV


def gqa_expand(X, heads, kv_heads):
    """Grouped-query / multi-query attention (Appendix C, last paragraph): query head h
    reads key/value head h // (heads / kv_heads).  The paper's kernels remap indices
    instead of duplicating; the duplication written out is the definition.
    ``X`` is ``[batch*kv_heads, ...]``; returns ``[batch*heads, ...]``, after which
    every other function of this module applies head by head."""
    X = np.asarray(X)
    assert heads % kv_heads == 0 and X.shape[0] % kv_heads == 0
    G, b = heads // kv_heads, X.shape[0] // kv_heads
    Y = np.empty((b, heads) + X.shape[1:], dtype=X.dtype)
    Xv = X.reshape((b, kv_heads) + X.shape[1:])
    for h in range(heads):
        Y[:, h] = Xv[:, h // G]
    return Y.reshape((b * heads,) + X.shape[1:])


def gqa_reduce(dX, heads, kv_heads):
    """Gradients of shared key/value heads are summed over the query heads that share
    them (same paragraph).  ``dX`` is ``[batch*heads, ...]`` (per query head, e.g. from
    attn_bwd on expanded K, V); returns ``[batch*kv_heads, ...]``."""
    dX = np.asarray(dX, dtype=np.float64)
    assert heads % kv_heads == 0 and dX.shape[0] % heads == 0
    G, b = heads // kv_heads, dX.shape[0] // heads
    out = np.zeros((b, kv_heads) + dX.shape[1:], dtype=np.float64)
    dv = dX.reshape((b, heads) + dX.shape[1:])
    for h in range(heads):
        out[:, h // G] += dv[:, h]
    return out.reshape((b * kv_heads,) + dX.shape[1:])


def moba_forward(Q, K, V, B, k, scale, conv_w=None, heads=1, round_mode=ROUND_NONE):
    """The whole forward chain of Section 2 (with Appendix B's conv if given):
    conv -> centroids -> top-k -> attention.  Returns a dict of every stage."""
    Kp = key_conv(K, conv_w, heads, round_mode) if conv_w is not None else np.asarray(K, np.float64)
    C = centroids(Kp, B)
    idx, kth = topk(Q, C, B, k)
    O, lse = attn_fwd(Q, Kp, V, idx, B, scale)
    return dict(K_eff=Kp, centroids=C, idx=idx, kth=kth, O=O, lse=lse)


def _pad_seq(X, lo, hi, B):
    """Rows lo..hi of X [bh, T, d] followed by zero rows up to the next multiple of B."""
    L = hi - lo
    Lp = -(-L // B) * B
    out = np.zeros((X.shape[0], Lp) + X.shape[2:], dtype=np.float64)
    out[:, :L] = X[:, lo:hi]
    return out


def moba_forward_varlen(Q, K, V, seq_offsets, B, k, scale):
    """Packed variable-length batch (Appendix C.1: a sequence of N keys has ceil(N / B) blocks, the
    last one shorter).  Q, K, V are [bh, T, d] with the sequences one after the other along T;
    sequence i is rows seq_offsets[i] .. seq_offsets[i+1].  Every sequence is the operator of
    Section 2 on its own: blocks count from the sequence's first token, candidates of a query are
    the complete blocks before its own block in ITS sequence, the own block (complete or not) is
    attended causally.  Written as a loop over the sequences, each padded with zero rows to a
    multiple of B (tests pin that reading against a dense evaluation of the ragged sequence).
    Returns O [bh, T, d], lse [bh, T] and idx [bh, T, k]: block numbers inside the query's
    sequence, -1 padded."""
    Q, K, V = (np.asarray(x, dtype=np.float64) for x in (Q, K, V))
    bh, T, d = Q.shape
    O = np.zeros((bh, T, d))
    lse = np.zeros((bh, T))
    idx = np.full((bh, T, k), -1, np.int32)
    for lo, hi in zip(seq_offsets[:-1], seq_offsets[1:]):
        if hi == lo:
            continue
        r = moba_forward(_pad_seq(Q, lo, hi, B), _pad_seq(K, lo, hi, B), _pad_seq(V, lo, hi, B), B, k, scale)
        O[:, lo:hi], lse[:, lo:hi], idx[:, lo:hi] = r["O"][:, :hi - lo], r["lse"][:, :hi - lo], r["idx"][:, :hi - lo]
    return dict(O=O, lse=lse, idx=idx)


def attn_varlen(Q, K, V, idx, dO, seq_offsets, B, scale):
    """Forward and backward of a packed variable-length batch at a GIVEN routing (idx as returned by
    moba_forward_varlen: block numbers inside each query's sequence).  -> O, lse, dQ, dK, dV."""
    Q, K, V, dO = (np.asarray(x, dtype=np.float64) for x in (Q, K, V, dO))
    idx = np.asarray(idx, dtype=np.int32)
    bh, T, d = Q.shape
    O, dQ, dK, dV = (np.zeros((bh, T, d)) for _ in range(4))
    lse = np.zeros((bh, T))
    for lo, hi in zip(seq_offsets[:-1], seq_offsets[1:]):
        L = hi - lo
        if L == 0:
            continue
        q, kk, v, g = (_pad_seq(X, lo, hi, B) for X in (Q, K, V, dO))
        ix = np.full((bh, q.shape[1], idx.shape[2]), -1, np.int32)
        ix[:, :L] = idx[:, lo:hi]
        for t in range(L, q.shape[1]):             # padded queries: any valid routing (they are dropped)
            ix[:, t, :min(idx.shape[2], t // B)] = np.arange(min(idx.shape[2], t // B))
        o, l = attn_fwd(q, kk, v, ix, B, scale)
        gq, gk, gv = attn_bwd(q, kk, v, ix, g, B, scale)
        O[:, lo:hi], lse[:, lo:hi] = o[:, :L], l[:, :L]
        dQ[:, lo:hi], dK[:, lo:hi], dV[:, lo:hi] = gq[:, :L], gk[:, :L], gv[:, :L]
    return O, lse, dQ, dK, dV
