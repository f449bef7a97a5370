"""MI355X-native hot path of the padding-free MoE layer of X-MoE (arXiv 2508.13337).

The product is libxmoe.so (hand-written HIP kernels for gfx950 behind the C ABI of include/xmoe.h).  This
package is the thin Python binding: the functions in `api` carry the same names as the C entry points and
only marshal arguments (torch tensors provide device memory and the stream).
"""
from .api import *  # noqa: F401,F403
from .layer import XMoE2Layer, XMoELayer, append_shared, capture_step  # noqa: F401
