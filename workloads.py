"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds no arithmetic of the method: it only draws tensors.  The same
CPU buffers feed the CPU oracle (after an exact widening to float64) and, copied to
the device, the GPU library, so no random generator has to match across languages.

Draw order per workload: Q, K, V, dO, then the conv weights / planted structure.
Values are drawn in fp32 with ``torch.Generator().manual_seed(seed)`` and rounded
once (nearest-even) to the I/O type.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    heads: int
    N: int
    d: int
    B: int
    k: int
    dtype: str = "bf16"        # "bf16" or "f32": type of Q,K,V,O and the gradients
    conv_width: int = 0        # 0: no key convolution
    backward: bool = False
    skew: bool = False         # planted hot blocks (load imbalance)
    seed: int = 0
    kv_heads: int = 0          # grouped-query attention: key/value heads (0 = heads)

    @property
    def bh(self):
        return self.batch * self.heads

    @property
    def hkv(self):
        return self.kv_heads if self.kv_heads > 0 else self.heads

    @property
    def n(self):
        return self.N // self.B

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.d))

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    def scaled(self, **kw):
        return replace(self, **kw)


# The five benchmark configurations (seed = 1000*config + trial).
CONFIGS = {
    1: Workload("cfg1_f32_fwd", 1, 2, 2048, 64, 128, 3, dtype="f32", seed=1000),
    2: Workload("cfg2_bf16_fwd", 1, 16, 8192, 64, 128, 8, seed=2000),
    3: Workload("cfg3_bf16_fwdbwd_B32", 1, 16, 32768, 64, 32, 64, backward=True, seed=3000),
    4: Workload("cfg4_bf16_conv4_d128", 1, 16, 131072, 128, 64, 32, conv_width=4, seed=4000),
    5: Workload("cfg5_bf16_skew", 2, 16, 16384, 64, 64, 32, backward=True, skew=True, seed=5000),
}


def routes_per_slice(N, B, k):
    n = N // B
    return B * sum(min(c, k) for c in range(n))


def attended_pairs_per_slice(N, B, k):
    """(query, key) pairs that survive the mask: B keys per routed block plus the
    causal triangle of the own block."""
    n = N // B
    return B * routes_per_slice(N, B, k) + n * B * (B + 1) // 2


def ragged_pairs(L, B, k):
    """Attended (query, key) pairs of one sequence of L tokens whose last block may be short
    (packed variable-length batches): every query keeps min(k, complete blocks before its own)
    past blocks of B keys and the causal part of its own block."""
    nf, r = divmod(L, B)
    return (B * B * sum(min(c, k) for c in range(nf)) + nf * B * (B + 1) // 2 +
            r * B * min(nf, k) + r * (r + 1) // 2)


def generate(w: Workload, device="cpu"):
    """Returns a dict of CPU tensors: Q,dO [batch,heads,N,d] and K,V [batch,kv_heads,N,d] in
    the I/O type, conv_w [kv_heads,d,W] fp32 (or None)."""
    g = torch.Generator().manual_seed(w.seed)
    shape = (w.batch, w.heads, w.N, w.d)
    kv_shape = (w.batch, w.hkv, w.N, w.d)
    Q = torch.randn(shape, generator=g, dtype=torch.float32)
    K = torch.randn(kv_shape, generator=g, dtype=torch.float32)
    V = torch.randn(kv_shape, generator=g, dtype=torch.float32)
    dO = torch.randn(shape, generator=g, dtype=torch.float32)
    conv_w = None
    if w.conv_width > 0:
        # weights ~ N(0, variance 1/4), one filter per (head, channel), last axis = lag
        conv_w = 0.5 * torch.randn((w.hkv, w.d, w.conv_width), generator=g, dtype=torch.float32)
    if w.skew:
        assert w.hkv == w.heads, "the planted hot blocks are defined per head"
        # per head a direction u with |u| = 3; per (batch, head) 1% of the blocks are hot:
        # u is added to all their keys; every query gets 0.5*u.
        u = torch.randn((w.heads, w.d), generator=g, dtype=torch.float32)
        u = 3.0 * u / u.norm(dim=-1, keepdim=True)
        n_hot = max(1, int(round(0.01 * w.n)))
        for b in range(w.batch):
            for h in range(w.heads):
                hot = torch.randperm(w.n, generator=g)[:n_hot]
                for j in hot.tolist():
                    K[b, h, j * w.B:(j + 1) * w.B] += u[h]
        Q += 0.5 * u[None, :, None, :]
    dt = w.torch_dtype
    out = dict(Q=Q.to(dt), K=K.to(dt), V=V.to(dt), dO=dO.to(dt), conv_w=conv_w)
    if device != "cpu":
        out = {k_: (v.to(device) if v is not None else None) for k_, v in out.items()}
    return out


def to_f64(t):
    """Exact widening of a CPU tensor [batch,heads,...] to numpy float64 with the
    two leading axes flattened."""
    a = t.detach().cpu().to(torch.float64).numpy()
    return a.reshape((a.shape[0] * a.shape[1],) + a.shape[2:])
