"""ctypes binding of libmoba.so.  Function names mirror the C ABI (include/moba.h).

PyTorch is used for device memory and streams only.  There is no fallback: if the
library has not been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libmoba.so")

F32, BF16 = 0, 1
FLAG_REFERENCE_KERNELS = 1
FLAG_KEY_MAJOR = 2
FLAG_QUERY_TILES = 4
FLAG_GATE_EXACT_SEARCH = 8
FLAG_SHARED_WORKSPACE = 16


class MobaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().moba_strerror(status).decode()
        super().__init__(f"{where}: {msg} (status {status}, hip error {lib().moba_last_hip_error()})")


class _CShape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("seqlen", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("block", ctypes.c_int32), ("topk", ctypes.c_int32),
                ("conv_width", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("flags", ctypes.c_uint32),
                ("kv_heads", ctypes.c_int32)]


@dataclass(frozen=True)
class Shape:
    batch: int
    heads: int
    seqlen: int
    head_dim: int
    block: int
    topk: int
    conv_width: int = 0
    dtype: int = BF16
    softmax_scale: float = 0.0
    flags: int = 0
    kv_heads: int = 0          # grouped-query attention: key/value heads (0 = heads)

    def c(self):
        return _CShape(self.batch, self.heads, self.seqlen, self.head_dim, self.block, self.topk,
                       self.conv_width, self.dtype, self.softmax_scale, self.flags, self.kv_heads)

    @property
    def hkv(self):
        return self.kv_heads if self.kv_heads > 0 else self.heads

    @property
    def n(self):
        return self.seqlen // self.block

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == BF16 else torch.float32


_lib = None


def lib():
    """Loads libmoba.so (built in-tree by paper_2511_11571_amd.build); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(_LIB_PATH)
        L.moba_strerror.restype = ctypes.c_char_p
        L.moba_strerror.argtypes = [ctypes.c_int]
        L.moba_last_hip_error.restype = ctypes.c_int
        for name in ("moba_routes_per_slice", "moba_workspace_bytes", "moba_centroids", "moba_topk",
                     "moba_topk_static", "moba_topk_varlen", "moba_varlen_layout", "moba_varlen_pad",
                     "moba_varlen_unpad", "moba_varlen_block_first", "moba_build_lists", "moba_forward", "moba_backward", "moba_backward_parts",
                     "moba_decode_forward",
                     "moba_profile_begin", "moba_profile_end", "moba_key_conv_backward",
                     "moba_key_conv_backward_workspace", "moba_microbench_copy", "moba_microbench_mfma"):
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _p(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(st, where):
    if st != 0:
        raise MobaError(st, where)


def routes_per_slice(shape: Shape) -> int:
    R = ctypes.c_int64(0)
    _check(lib().moba_routes_per_slice(ctypes.byref(shape.c()), ctypes.byref(R)), "moba_routes_per_slice")
    return R.value


def workspace_bytes(shape: Shape):
    a, b, c = ctypes.c_size_t(0), ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().moba_workspace_bytes(ctypes.byref(shape.c()), ctypes.byref(a), ctypes.byref(b),
                                      ctypes.byref(c)), "moba_workspace_bytes")
    return a.value, b.value, c.value


def _ws(nbytes, like):
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=like.device)


def centroids(shape: Shape, K, conv_w=None, K_eff=None, out=None):
    """-> (K_eff or K, centroids [b,h,n,d] fp32)."""
    assert K.is_contiguous() and K.dtype == shape.torch_dtype
    if shape.conv_width > 0 and K_eff is None:
        K_eff = torch.empty_like(K)
    if out is None:
        out = torch.empty((shape.batch, shape.hkv, shape.n, shape.head_dim), dtype=torch.float32,
                          device=K.device)
    _check(lib().moba_centroids(ctypes.byref(shape.c()), _p(K), _p(conv_w), _p(K_eff), _p(out),
                                _stream()), "moba_centroids")
    return (K_eff if K_eff is not None else K), out




def key_conv_backward(shape: Shape, K, conv_w, dK_eff, ws=None):
    """Backward of the key convolution -> (dK [b,h,N,d] in the I/O type, dconv_w [heads,d,W] fp32)."""
    assert K.is_contiguous() and dK_eff.is_contiguous() and K.dtype == shape.torch_dtype
    assert dK_eff.dtype == shape.torch_dtype and conv_w.is_contiguous() and conv_w.dtype == torch.float32
    if ws is None:
        n = ctypes.c_size_t(0)
        _check(lib().moba_key_conv_backward_workspace(ctypes.byref(shape.c()), ctypes.byref(n)),
               "moba_key_conv_backward_workspace")
        ws = _ws(n.value, K)
    dK = torch.empty_like(K)
    dw = torch.empty_like(conv_w)
    _check(lib().moba_key_conv_backward(ctypes.byref(shape.c()), _p(K), _p(conv_w), _p(dK_eff), _p(dK),
                                        _p(dw), _p(ws), ctypes.c_size_t(ws.numel()), _stream()),
           "moba_key_conv_backward")
    return dK, dw


def _list_buffers(shape, like):
    R = routes_per_slice(shape)
    off = torch.empty((shape.batch, shape.heads, shape.n + 1), dtype=torch.int32, device=like.device)
    ql = torch.empty((shape.batch, shape.heads, max(R, 1)), dtype=torch.int32, device=like.device)
    return off, (ql[..., :R] if R > 0 else ql[..., :0])


def topk(shape: Shape, Q, cent, ws=None):
    """-> (topk_idx [b,h,N,k] int32, lists) with lists = (blk_off [b,h,n+1], blk_q [b,h,R]),
    all int32."""
    assert Q.is_contiguous() and cent.is_contiguous()
    idx = torch.empty((shape.batch, shape.heads, shape.seqlen, shape.topk), dtype=torch.int32,
                      device=Q.device)
    off, ql = _list_buffers(shape, Q)
    if ws is None:
        ws = _ws(workspace_bytes(shape)[0], Q)
    _check(lib().moba_topk(ctypes.byref(shape.c()), _p(Q), _p(cent), _p(idx), _p(off), _p(ql),
                           _p(ws), ctypes.c_size_t(ws.numel()), _stream()), "moba_topk")
    return idx, (off, ql)


def topk_static(shape: Shape, Q, cent, out=None):
    """moba_topk_static: as topk, with the library's own static scratch instead of a workspace.
    ``out`` = (idx, (blk_off, blk_q)) lets the caller bring the output tensors, so that the call
    itself allocates nothing."""
    assert Q.is_contiguous() and cent.is_contiguous()
    if out is None:
        idx = torch.empty((shape.batch, shape.heads, shape.seqlen, shape.topk), dtype=torch.int32,
                          device=Q.device)
        off, ql = _list_buffers(shape, Q)
    else:
        idx, (off, ql) = out
    _check(lib().moba_topk_static(ctypes.byref(shape.c()), _p(Q), _p(cent), _p(idx), _p(off), _p(ql),
                                  _stream()), "moba_topk_static")
    return idx, (off, ql)


class VarlenLayout:
    """Padded layout of a packed variable-length batch (moba_varlen_layout): every sequence starts at
    a multiple of the block.  seq_offsets: host sequence of num_seqs + 1 ascending token offsets."""

    def __init__(self, seq_offsets, block, device="cuda"):
        self.num_seqs = len(seq_offsets) - 1
        self.block = block
        self.tokens = int(seq_offsets[-1])
        so = (ctypes.c_int32 * (self.num_seqs + 1))(*[int(x) for x in seq_offsets])
        po = (ctypes.c_int32 * (self.num_seqs + 1))()
        tp = ctypes.c_int32(0)
        _check(lib().moba_varlen_layout(ctypes.c_int32(self.num_seqs), so, ctypes.c_int32(block), po,
                                        ctypes.byref(tp)), "moba_varlen_layout")
        self.padded_tokens = tp.value
        self.seq_offsets_host = list(so)
        self.pad_offsets_host = list(po)
        self.seq_offsets = torch.tensor(self.seq_offsets_host, dtype=torch.int32, device=device)
        self.pad_offsets = torch.tensor(self.pad_offsets_host, dtype=torch.int32, device=device)
        self.block_first = torch.empty(max(self.padded_tokens // block, 1), dtype=torch.int32, device=device)
        _check(lib().moba_varlen_block_first(ctypes.c_int32(self.num_seqs), _p(self.pad_offsets),
                                             ctypes.c_int32(block), ctypes.c_int32(self.padded_tokens),
                                             _p(self.block_first), _stream()), "moba_varlen_block_first")

    def _copy(self, fn, name, X, out_rows):
        assert X.is_contiguous() and X.dim() >= 3
        lead, rows = X.shape[:2], X.shape[2]
        row_bytes = X[0, 0, 0].numel() * X.element_size() if X.dim() > 3 else X.element_size()
        out = torch.empty(lead + (out_rows,) + X.shape[3:], dtype=X.dtype, device=X.device)
        _check(fn(ctypes.c_int32(self.num_seqs), _p(self.seq_offsets), _p(self.pad_offsets),
                  ctypes.c_int32(lead[0] * lead[1]), ctypes.c_int32(self.tokens),
                  ctypes.c_int32(self.padded_tokens), ctypes.c_int32(row_bytes), _p(X), _p(out), _stream()), name)
        return out

    def pad(self, X):
        """[1, heads, T, ...] -> [1, heads, T', ...], zero rows after every sequence."""
        assert X.shape[2] == self.tokens
        return self._copy(lib().moba_varlen_pad, "moba_varlen_pad", X, self.padded_tokens)

    def unpad(self, Xp):
        """[1, heads, T', ...] -> [1, heads, T, ...]."""
        assert Xp.shape[2] == self.padded_tokens
        return self._copy(lib().moba_varlen_unpad, "moba_varlen_unpad", Xp, self.tokens)


def topk_varlen(shape: Shape, layout: VarlenLayout, Q, cent, ws=None):
    """moba_topk_varlen on the padded layout (shape.seqlen = layout.padded_tokens, batch 1)."""
    assert Q.is_contiguous() and cent.is_contiguous() and shape.seqlen == layout.padded_tokens
    idx = torch.empty((shape.batch, shape.heads, shape.seqlen, shape.topk), dtype=torch.int32,
                      device=Q.device)
    off, ql = _list_buffers(shape, Q)
    if ws is None:
        ws = _ws(workspace_bytes(shape)[0], Q)
    _check(lib().moba_topk_varlen(ctypes.byref(shape.c()), _p(Q), _p(cent), _p(layout.block_first), _p(idx),
                                  _p(off), _p(ql), _p(ws), ctypes.c_size_t(ws.numel()), _stream()),
           "moba_topk_varlen")
    return idx, (off, ql)


def build_lists(shape: Shape, idx, ws=None):
    """-> lists = (blk_off, blk_q) for a routing given by the caller."""
    assert idx.is_contiguous() and idx.dtype == torch.int32
    off, ql = _list_buffers(shape, idx)
    if ws is None:
        ws = _ws(workspace_bytes(shape)[0], idx)
    _check(lib().moba_build_lists(ctypes.byref(shape.c()), _p(idx), _p(off), _p(ql),
                                  _p(ws), ctypes.c_size_t(ws.numel()), _stream()), "moba_build_lists")
    return off, ql


def forward(shape: Shape, Q, K_eff, V, idx, lists, ws=None, O=None, lse=None):
    """-> (O [b,h,N,d], lse [b,h,N] fp32).  ``lists`` as returned by topk / build_lists."""
    off, ql = lists
    for t in (Q, K_eff, V):
        assert t.is_contiguous() and t.dtype == shape.torch_dtype
    if O is None:
        O = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    if ws is None:
        ws = _ws(workspace_bytes(shape)[1], Q)
    _check(lib().moba_forward(ctypes.byref(shape.c()), _p(Q), _p(K_eff), _p(V), _p(idx), _p(off),
                              _p(ql), _p(O), _p(lse), _p(ws), ctypes.c_size_t(ws.numel()),
                              _stream()),
           "moba_forward")
    return O, lse


BWD_PREPROCESS, BWD_DQ, BWD_DKDV, BWD_ALL = 1, 2, 4, 7


def backward(shape: Shape, Q, K_eff, V, O, lse, dO, idx, lists, ws=None, out=None, parts=None):
    """-> (dQ, dK, dV), each [b,h,N,d].  ``parts`` (a BWD_* bit set) runs only some of the
    backward's kernels through moba_backward_parts."""
    off, ql = lists
    for t in (Q, K_eff, V, O, dO):
        assert t.is_contiguous() and t.dtype == shape.torch_dtype
    dQ, dK, dV = out if out is not None else (torch.empty_like(Q), torch.empty_like(K_eff),
                                              torch.empty_like(V))
    if ws is None:
        ws = _ws(workspace_bytes(shape)[2], Q)
    if parts is None:
        _check(lib().moba_backward(ctypes.byref(shape.c()), _p(Q), _p(K_eff), _p(V), _p(O), _p(lse),
                                   _p(dO), _p(idx), _p(off), _p(ql), _p(dQ), _p(dK), _p(dV),
                                   _p(ws), ctypes.c_size_t(ws.numel()), _stream()), "moba_backward")
    else:
        _check(lib().moba_backward_parts(ctypes.byref(shape.c()), _p(Q), _p(K_eff), _p(V), _p(O),
                                         _p(lse), _p(dO), _p(idx), _p(off), _p(ql), _p(dQ),
                                         _p(dK), _p(dV), _p(ws), ctypes.c_size_t(ws.numel()), _stream(),
                                         ctypes.c_uint32(parts)), "moba_backward_parts")
    return dQ, dK, dV


def decode_forward(shape: Shape, q_len, Q, K_eff, V, cent, want_idx=True):
    """Decode-shaped forward for the last q_len positions of shape.seqlen keys (any length).
    -> (O [b,h,q_len,d], lse [b,h,q_len] fp32, topk_idx [b,h,q_len,k] int32 or None)."""
    for t in (Q, K_eff, V):
        assert t.is_contiguous() and t.dtype == shape.torch_dtype
    assert Q.shape[2] == q_len and K_eff.shape[2] == shape.seqlen
    blocks = 0
    if cent is not None:
        assert cent.is_contiguous() and cent.dtype == torch.float32
        blocks = cent.shape[2]
    O = torch.empty_like(Q)
    lse = torch.empty(Q.shape[:3], dtype=torch.float32, device=Q.device)
    idx = (torch.empty((shape.batch, shape.heads, q_len, shape.topk), dtype=torch.int32, device=Q.device)
           if want_idx else None)
    _check(lib().moba_decode_forward(ctypes.byref(shape.c()), ctypes.c_int32(q_len), _p(Q), _p(K_eff),
                                     _p(V), _p(cent), ctypes.c_int32(blocks), _p(O), _p(lse), _p(idx),
                                     _stream()), "moba_decode_forward")
    return O, lse, idx


PROFILE_KERNELS = ("topk", "forward", "bwd_dq", "bwd_dkdv")


def profile_begin():
    """Starts timing the main kernels with HIP events on their launch stream."""
    _check(lib().moba_profile_begin(), "moba_profile_begin")


def profile_end():
    """Ends the timing session: {kernel: (total milliseconds, launches)}."""
    ms = (ctypes.c_float * len(PROFILE_KERNELS))()
    calls = (ctypes.c_int32 * len(PROFILE_KERNELS))()
    _check(lib().moba_profile_end(ms, calls), "moba_profile_end")
    return {name: (float(ms[i]), int(calls[i])) for i, name in enumerate(PROFILE_KERNELS)}


def microbench(copy_bytes=1 << 30, mfma_iters=20000):
    """The library's two ceiling measurements: -> {"copy_GBs": ..., "mfma_tflops": {waves per SIMD: ...}}."""
    src = torch.ones(copy_bytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    ms = ctypes.c_float(0)
    _check(lib().moba_microbench_copy(_p(dst), _p(src), ctypes.c_size_t(copy_bytes), ctypes.c_int(5),
                                      ctypes.byref(ms), _stream()), "moba_microbench_copy")
    out = {"copy_bytes": copy_bytes, "copy_ms": ms.value, "copy_GBs": 2.0 * copy_bytes / (ms.value * 1e-3) / 1e9,
           "mfma_tflops": {}}
    flop = ctypes.c_double(0)
    for wps in (1, 2, 4, 8):
        _check(lib().moba_microbench_mfma(ctypes.c_int(wps), ctypes.c_int(mfma_iters), _p(dst), ctypes.byref(ms),
                                          ctypes.byref(flop), _stream()), "moba_microbench_mfma")
        out["mfma_tflops"][wps] = flop.value / (ms.value * 1e-3) / 1e12
    return out
