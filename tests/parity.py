"""Comparison rules between the GPU library and the CPU oracle.

Routing: per query the GPU's kept set must equal the oracle's, except that blocks in
the symmetric difference are tolerated when both sets have the same size and each
such block's oracle gate score lies within 1e-4 of the oracle's k-th score (fp32
scoring cannot order scores that close).  Outputs: max-abs 1e-4 (fp32 I/O) or 2e-2
(bf16 I/O).  Gradients: relative L2 5e-2 (bf16) or 1e-4 (fp32).
"""
import numpy as np

GAP = 1e-4
O_TOL = {"f32": 1e-4, "bf16": 2e-2}
GRAD_TOL = {"f32": 1e-4, "bf16": 5e-2}
LSE_TOL = {"f32": 1e-4, "bf16": 2e-3}


def routing_check(oracle, got_idx, ref_idx, kth, Q64, C64, B, rows=None):
    """got_idx/ref_idx: [nrows, k] (any order, -1 padded); kth: [nrows]; rows: flat row ids
    of those rows (default all rows of Q64).  Returns (exact_row_mask, exempt_fraction);
    raises AssertionError on a disagreement outside the gap rule."""
    nrows, k = ref_idx.shape
    if k == 0:
        return np.ones(nrows, bool), 0.0
    g = np.sort(got_idx, axis=-1)
    r = np.sort(ref_idx, axis=-1)
    exact = (g == r).all(-1)
    bad = np.nonzero(~exact)[0]
    if bad.size:
        flat = np.arange(nrows, dtype=np.int64) if rows is None else np.asarray(rows, np.int64)
        S = oracle.gate_scores(Q64, C64, flat[bad], B)
        for i, row in enumerate(bad):
            G = set(int(x) for x in got_idx[row] if x >= 0)
            Rr = set(int(x) for x in ref_idx[row] if x >= 0)
            assert len(G) == len(Rr) == (got_idx[row] >= 0).sum(), \
                f"row {flat[row]}: kept {len(G)} blocks, oracle {len(Rr)}"
            for b in G ^ Rr:
                gap = abs(S[i, b] - kth[row])
                assert gap < GAP, f"row {flat[row]}: block {b} differs, score gap {gap:.3g}"
    return exact, bad.size / max(nrows, 1)


def check_lists(off, ql, idx, ref_off, ref_ql, k):
    """off [bh, n+1], ql [bh, R] as the library wrote them; idx [bh, N, k] the routing they were
    built from; ref_off / ref_ql the oracle's lists of the same routing.  A list entry holds the
    query in its low 24 bits; where the key-block-major kernels will run, the high byte holds the
    position of the block in that query's row of idx (checked against idx itself), elsewhere 0."""
    assert np.array_equal(off, ref_off)
    assert np.array_equal(ql & 0xffffff, ref_ql)
    slots = ql >> 24
    if not slots.any():
        return
    assert k <= 64
    for s in range(off.shape[0]):
        blocks = np.repeat(np.arange(off.shape[1] - 1), np.diff(off[s]))      # block of every entry
        R = blocks.size
        assert np.array_equal(idx[s][ref_ql[s, :R], slots[s, :R]], blocks)


def rel_l2(a, b):
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a))


def max_abs(a, b):
    return float(np.abs(np.asarray(a, np.float64) - np.asarray(b, np.float64)).max()) if np.size(a) else 0.0
