"""Loads libxmoe.so with ctypes and declares the C ABI of include/xmoe.h.  There is no fallback: if the
library has not been built, importing a symbol from it raises."""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libxmoe.so")

_c_int = ctypes.c_int
_c_void_p = ctypes.c_void_p
_c_size_t = ctypes.c_size_t

# name -> (restype, argtypes); mirrors include/xmoe.h
SIGNATURES = {
    "xmoe_status_string": (ctypes.c_char_p, [_c_int]),
    "xmoe_version": (ctypes.c_char_p, []),
    "xmoe_workspace_bytes": (_c_size_t, [_c_int] * 7),
    "xmoe_gate_logits": (_c_int, [_c_void_p] * 4 + [_c_int] * 4 + [_c_void_p]),
    "xmoe_route": (_c_int, [_c_void_p] + [_c_int] * 3 + [_c_void_p] * 3),
    "xmoe_build_eri": (_c_int, [_c_void_p] * 2 + [_c_int] * 3 + [_c_void_p] * 7 + [_c_size_t, _c_void_p]),
    "xmoe_build_eri_static": (_c_int, [_c_void_p] * 2 + [_c_int] * 3 + [_c_void_p] * 7),
    "xmoe_build_eri_capped": (_c_int, [_c_void_p] * 2 + [_c_int] * 4 + [_c_void_p] * 7 + [_c_size_t, _c_void_p]),
    "xmoe_dispatch": (_c_int, [_c_void_p] * 2 + [_c_int] * 4 + [_c_void_p] * 2),
    "xmoe_expert_ffn_fwd": (_c_int, [_c_void_p] * 3 + [_c_int] * 4 + [_c_void_p] * 6 + [_c_int, _c_void_p, _c_size_t,
                                                                                        _c_void_p]),
    "xmoe_expert_ffn_bwd": (_c_int, [_c_void_p] * 9 + [_c_int] * 4 + [_c_void_p] * 7 + [_c_int, _c_void_p, _c_size_t,
                                                                                        _c_void_p]),
    "xmoe_expert_mlp2_fwd": (_c_int, [_c_void_p] * 3 + [_c_int] * 4 + [_c_void_p] * 2 + [_c_int] + [_c_void_p] * 2 +
                             [_c_int, _c_void_p, _c_size_t, _c_void_p]),
    "xmoe_expert_mlp2_bwd": (_c_int, [_c_void_p] * 8 + [_c_int] * 4 + [_c_void_p] * 2 + [_c_int] + [_c_void_p] * 3 +
                             [_c_int, _c_void_p, _c_size_t, _c_void_p]),
    "xmoe_rbd_stage0": (_c_int, [_c_void_p] * 6 + [_c_int] * 4 + [_c_void_p] * 12 + [_c_size_t, _c_void_p]),
    "xmoe_rbd_absolute_index": (_c_int, [_c_void_p] * 3 + [_c_int] * 2 + [_c_void_p] * 2),
    "xmoe_combine": (_c_int, [_c_void_p] * 4 + [_c_int, _c_void_p, _c_void_p] + [_c_int] * 4 + [_c_void_p] * 2),
    "xmoe_append_shared_segments": (_c_int, [_c_void_p] * 3 + [_c_int] * 3 + [_c_void_p]),
    "xmoe_combine_bwd": (_c_int, [_c_void_p] * 4 + [_c_int] * 4 + [_c_void_p] * 3),
    "xmoe_combine_bwd_weights": (_c_int, [_c_void_p] * 2 + [_c_int] * 2 + [_c_void_p] * 2),
    "xmoe_dispatch_bwd": (_c_int, [_c_void_p] * 3 + [_c_int, _c_void_p, _c_void_p] + [_c_int] * 4 + [_c_void_p] * 2),
    "xmoe_route_bwd": (_c_int, [_c_void_p] * 3 + [_c_int] * 3 + [_c_void_p] * 2),
    "xmoe_gate_logits_bwd": (_c_int, [_c_void_p] * 3 + [_c_int] * 4 + [_c_void_p] * 3 + [_c_size_t, _c_void_p]),
    "xmoe_prof_enable": (None, [_c_int]),
    "xmoe_prof_reset": (None, []),
    "xmoe_prof_num_kernels": (_c_int, []),
    "xmoe_prof_kernel_name": (ctypes.c_char_p, [_c_int]),
    "xmoe_prof_get": (_c_int, [_c_int, ctypes.POINTER(_c_int), ctypes.POINTER(ctypes.c_double)]),
    "xmoe_prof_shader_clock": (_c_int, [_c_int, ctypes.POINTER(ctypes.c_double)]),
    "xmoe_prof_copy": (_c_int, [_c_void_p, _c_void_p, ctypes.c_size_t, _c_void_p]),
}

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2508_13337_amd.build). "
                "There is no CPU or PyTorch fallback for the MoE hot path.")
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib
