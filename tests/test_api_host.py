"""Host-side behaviour of the C ABI: the library loads, exports every declared symbol,
and rejects bad arguments before anything is launched (so this runs without a GPU)."""
import ctypes
import os
import re

import pytest

import paper_2511_11571_amd as moba
from paper_2511_11571_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(os.path.join(ROOT, "paper_2511_11571_amd", "libmoba.so")):
        from paper_2511_11571_amd import build
        build.build()
    return moba.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "moba.h")).read()
    names = set(re.findall(r"\b(moba_[a-z_]+)\s*\(", header))
    assert {"moba_centroids", "moba_topk", "moba_forward", "moba_backward"} <= names
    for name in names:
        assert hasattr(lib, name), name


def _shape(**kw):
    base = dict(batch=1, heads=2, seqlen=1024, head_dim=64, block=32, topk=4)
    base.update(kw)
    return binding.Shape(**base)


def test_decode_forward_rejects_bad_arguments(lib):
    """Host-side checks only: every call returns before anything is launched."""
    one = ctypes.c_void_p(256)                 # never dereferenced on these paths
    sh = _shape(seqlen=1000).c()               # any length: the last block may be ragged
    f = lib.moba_decode_forward
    assert f(ctypes.byref(sh), 0, one, one, one, one, 31, one, one, None, None) == -1      # q_len
    assert f(ctypes.byref(sh), 1001, one, one, one, one, 31, one, one, None, None) == -1
    assert f(ctypes.byref(sh), 4, None, one, one, one, 31, one, one, None, None) == -1     # Q
    assert f(ctypes.byref(sh), 4, one, one, one, one, 30, one, one, None, None) == -1      # too few centroids
    assert f(ctypes.byref(sh), 4, one, one, one, None, 0, one, one, None, None) == -1
    big = _shape(seqlen=4098 * 32 + 5).c()     # more than 4096 complete blocks
    assert f(ctypes.byref(big), 1, one, one, one, one, 5000, one, one, None, None) == -2


def test_grouped_query_shapes_are_accepted(lib):
    R = ctypes.c_int64(0)
    for kv in (0, 1, 2, 4):
        sh = _shape(heads=4, kv_heads=kv).c()
        assert lib.moba_routes_per_slice(ctypes.byref(sh), ctypes.byref(R)) == 0
    # sharing key/value heads shrinks the copies of K and V in the forward workspace
    assert moba.workspace_bytes(_shape(heads=4, kv_heads=1))[1] < moba.workspace_bytes(_shape(heads=4))[1]


def test_routes_and_workspace(lib):
    sh = _shape()
    n = 32
    assert moba.routes_per_slice(sh) == 32 * sum(min(c, 4) for c in range(n))
    assert moba.routes_per_slice(_shape(topk=0)) == 0
    assert moba.routes_per_slice(_shape(topk=1000)) == 32 * n * (n - 1) // 2
    a, b, c = moba.workspace_bytes(sh)
    assert a > 0 and b > 0 and c >= 4 * 2 * 1024


@pytest.mark.parametrize("kw,key_major", [
    (dict(heads=16, seqlen=32768, block=32, topk=64), False),                # headline shape: many kept blocks
    (dict(batch=2, heads=16, seqlen=16384, block=64, topk=32), False),       # skewed-routing shape
    (dict(heads=16, seqlen=8192, block=128, topk=8), True),                  # few kept blocks of many keys
    (dict(batch=2, heads=16, seqlen=524288, block=128, topk=8), True),       # the long end of the latency sweep
    (dict(heads=16, seqlen=131072, head_dim=128, block=64, topk=32, conv_width=4), True),
    (dict(heads=16, seqlen=16384, block=64, topk=60), False),                # dense routing: tiles
    (dict(heads=16, seqlen=8192, block=128, topk=0), False),                 # own block only
    # more than 4096 keys per query: too many for the fixed-point accumulators of the query tiles
    (dict(heads=2, seqlen=32768, block=32, topk=64), False),                 # 2080 keys: tiles
    (dict(heads=2, seqlen=32768, block=128, topk=64), True),                 # 8320 keys: key blocks
])
def test_default_cut_of_the_attention(kw, key_major):
    """With neither flag the library sizes (and runs) the forward and backward for the cut it
    estimates to be cheaper; seen from here through the workspace sizes, which differ."""
    kw = dict(dict(dtype=binding.BF16), **kw)
    forced = {f: moba.workspace_bytes(_shape(flags=f, **kw))[1:] for f in (binding.FLAG_KEY_MAJOR,
                                                                          binding.FLAG_QUERY_TILES)}
    picked = moba.workspace_bytes(_shape(**kw))[1:]
    if kw["topk"] > 0:
        assert forced[binding.FLAG_KEY_MAJOR] != forced[binding.FLAG_QUERY_TILES]
    assert picked == forced[binding.FLAG_KEY_MAJOR if key_major else binding.FLAG_QUERY_TILES]


@pytest.mark.parametrize("kw,status", [
    (dict(batch=0), -1), (dict(heads=-1), -1), (dict(seqlen=0), -1), (dict(block=0), -1),
    (dict(seqlen=1000), -1),            # not a multiple of the block
    (dict(topk=-1), -1), (dict(dtype=7), -1), (dict(conv_width=-2), -1), (dict(flags=32), -1),
    (dict(head_dim=96), -2), (dict(conv_width=9), -2), (dict(topk=5000), -2),
    (dict(seqlen=(1 << 24) + 32, topk=0), -2),      # longer than the 32-bit row offsets allow
    (dict(heads=6, kv_heads=4), -1),    # key/value heads must divide the query heads
    (dict(kv_heads=-1), -1), (dict(heads=2, kv_heads=4), -1),
])
def test_bad_shapes_are_rejected(lib, kw, status):
    sh = _shape(**kw).c()
    R = ctypes.c_int64(0)
    assert lib.moba_routes_per_slice(ctypes.byref(sh), ctypes.byref(R)) == status
    assert lib.moba_workspace_bytes(ctypes.byref(sh), None, None, None) == status
    assert lib.moba_strerror(status)


def test_null_pointers_and_short_workspace(lib):
    sh = _shape().c()
    z = ctypes.c_void_p(0)
    one = ctypes.c_void_p(256)          # never dereferenced: checks come first
    big = ctypes.c_size_t(1 << 40)
    assert lib.moba_routes_per_slice(None, None) == -1
    assert lib.moba_centroids(ctypes.byref(sh), z, z, z, one, z) == -1
    assert lib.moba_centroids(ctypes.byref(sh), one, one, z, one, z) == -1     # weights without conv
    conv = _shape(conv_width=4).c()
    assert lib.moba_centroids(ctypes.byref(conv), one, z, one, one, z) == -1   # conv without weights
    assert lib.moba_centroids(ctypes.byref(conv), one, one, z, one, z) == -1   # conv needs K_eff
    assert lib.moba_topk(ctypes.byref(sh), z, one, one, one, one, one, big, z) == -1
    assert lib.moba_topk(ctypes.byref(sh), one, one, one, z, one, one, big, z) == -1           # no blk_off
    assert lib.moba_topk(ctypes.byref(sh), one, one, one, one, one, z, big, z) == -3
    assert lib.moba_topk(ctypes.byref(sh), one, one, one, one, one, one, ctypes.c_size_t(8), z) == -3
    assert lib.moba_build_lists(ctypes.byref(sh), z, one, one, one, big, z) == -1
    assert lib.moba_forward(ctypes.byref(sh), one, one, one, one, one, one, z, one, one, big, z) == -1
    assert lib.moba_forward(ctypes.byref(sh), one, one, one, one, one, one, one, one, z, big, z) == -3
    assert lib.moba_backward(ctypes.byref(sh), one, one, one, one, one, one, one, one, one,
                             one, one, z, one, big, z) == -1
    assert lib.moba_backward(ctypes.byref(sh), one, one, one, one, one, one, one, one, one,
                             one, one, one, one, ctypes.c_size_t(16), z) == -3
    n = ctypes.c_size_t(0)
    assert lib.moba_key_conv_backward_workspace(ctypes.byref(sh), ctypes.byref(n)) == -1       # no conv
    assert lib.moba_key_conv_backward_workspace(ctypes.byref(conv), ctypes.byref(n)) == 0 and n.value > 0
    assert lib.moba_key_conv_backward(ctypes.byref(sh), one, one, one, one, one, one, big, z) == -1
    assert lib.moba_key_conv_backward(ctypes.byref(conv), one, one, z, one, one, one, big, z) == -1
    assert lib.moba_key_conv_backward(ctypes.byref(conv), one, one, one, one, one, one, big, z) == -1  # in place
    two = ctypes.c_void_p(512)
    assert lib.moba_key_conv_backward(ctypes.byref(conv), one, one, one, two, one, one, ctypes.c_size_t(8), z) == -3
    # key blocks per head: 16384 for the bf16 gate kernel, 4096 for the plain one (fp32 tensors,
    # or bf16 with the plain kernels asked for)
    for many in (_shape(seqlen=32 * 17000), _shape(seqlen=32 * 5000, dtype=binding.F32),
                 _shape(seqlen=32 * 5000, flags=binding.FLAG_REFERENCE_KERNELS)):
        assert lib.moba_topk(ctypes.byref(many.c()), one, one, one, one, one, one, big, z) == -2
        assert lib.moba_topk_static(ctypes.byref(many.c()), one, one, one, one, one, z) == -2


def test_binding_raises(lib):
    with pytest.raises(moba.MobaError):
        moba.routes_per_slice(_shape(head_dim=80))


def test_profile_session_misuse_is_rejected(lib):
    import ctypes
    ms = (ctypes.c_float * 4)()
    calls = (ctypes.c_int32 * 4)()
    assert lib.moba_profile_end(ms, calls) == -1            # no session open
    assert lib.moba_profile_begin() == 0
    assert lib.moba_profile_begin() == -1                   # already open
    assert lib.moba_profile_end(None, calls) == -1          # null array: the session stays open
    assert lib.moba_profile_end(ms, calls) == 0             # no launches: all zero, no HIP call
    assert list(calls) == [0, 0, 0, 0] and list(ms) == [0.0] * 4


def test_convolution_in_place_is_rejected(lib):
    one = ctypes.c_void_p(256)                 # never dereferenced on these paths
    sh = _shape(conv_width=4).c()
    assert lib.moba_centroids(ctypes.byref(sh), one, one, one, one, None) == -1      # K_eff == K
    sh1 = _shape(conv_width=0).c()
    assert lib.moba_centroids(ctypes.byref(sh1), None, None, None, one, None) == -1   # K missing
