"""MI355X-native selective KV-recompute prefill (CacheClip hot path).

Thin ctypes binding over libcacheclip.so (hand-written HIP for gfx950).  The
binding only marshals arguments: device pointers of torch tensors, sizes and
the current stream.  Every step of the path runs in the library's kernels;
there is no CPU or PyTorch fallback, and importing this package fails loudly
if the library has not been built.
"""
from ._lib import (  # noqa: F401
    CacheClipError, Context, LayerWeights, KVLayer, ModelDesc, lib_path, load_library,
    K_NAMES, select_noalloc,
)
