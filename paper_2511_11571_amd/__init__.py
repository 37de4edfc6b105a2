"""MI355X-native Mixture of Block Attention: thin Python binding over libmoba.so.

Only argument marshalling happens here; every step of the path runs in the HIP
kernels behind the C ABI declared in include/moba.h.
"""
from .binding import (MobaError, Shape, VarlenLayout, topk_varlen, backward, build_lists, centroids, decode_forward, forward,  # noqa: F401
                      key_conv_backward, lib, microbench,
                      profile_begin, profile_end, routes_per_slice, topk, topk_static, workspace_bytes)
