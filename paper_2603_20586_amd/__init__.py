"""MI355X-native FastMKA route-fused attention: thin Python binding over libmka.so.

The package only marshals arguments (torch tensors -> device pointers, shapes -> C structs,
current torch stream -> hipStream_t); every step of the path runs in the HIP kernels behind
the C ABI declared in include/mka.h.  There is no CPU fallback: if the shared library is not
built, importing the binding raises.
"""
from .binding import (  # noqa: F401
    MKA_BF16,
    MKA_F32,
    MkaError,
    lib,
    lib_path,
    mka_fused_attn_bwd,
    mka_fused_attn_decode,
    mka_fused_attn_decode_static,
    mka_fuse_kv,
    mka_full_attn_fwd,
    mka_fused_attn_fwd,
    mka_paged_fused_decode,
    mka_prefix_mean,
    mka_mixture_attn_fwd,
    mka_route,
    mka_route_variant,
    mka_workspace_bytes,
    status_string,
)
