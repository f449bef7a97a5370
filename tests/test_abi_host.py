"""Host-side checks that need no GPU: libxmoe loads, exports every symbol the header declares, sizes its
workspaces sanely and rejects bad arguments before anything is enqueued."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "xmoe.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2508_13337_amd import _lib
    if not os.path.exists(_lib.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return _lib.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(xmoe_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2508_13337_amd import _lib
    names = declared_symbols()
    assert len(names) >= 19
    for n in names:
        assert hasattr(lib, n), f"{n} declared in xmoe.h but not exported"
        assert n in _lib.SIGNATURES, f"{n} has no ctypes signature"
    assert sorted(_lib.SIGNATURES) == names


def test_binding_has_same_names():
    import paper_2508_13337_amd as xm
    for n in ("xmoe_gate_logits", "xmoe_route", "xmoe_build_eri", "xmoe_dispatch", "xmoe_expert_ffn_fwd",
              "xmoe_expert_ffn_bwd", "xmoe_combine", "xmoe_combine_bwd", "xmoe_dispatch_bwd", "xmoe_route_bwd",
              "xmoe_gate_logits_bwd"):
        assert callable(getattr(xm, n))


def test_status_strings(lib):
    assert lib.xmoe_status_string(0) == b"XMOE_OK"
    for s in range(1, 5):
        assert lib.xmoe_status_string(s).startswith(b"XMOE_ERR_")
    assert b"unknown" in lib.xmoe_status_string(99)


def test_workspace_sizes(lib):
    B, d, E, k, f = 49152, 2048, 64, 6, 1408
    fwd = lib.xmoe_workspace_bytes(1, B, d, E, k, f, 1)
    bwd = lib.xmoe_workspace_bytes(2, B, d, E, k, f, 1)
    assert fwd >= B * f * 2 and bwd >= 3 * B * f * 2 and bwd < 4 * B * f * 2
    assert lib.xmoe_workspace_bytes(0, 8192, d, E, k, f, 1) >= (8192 * k // 1024) * E * 4
    assert lib.xmoe_workspace_bytes(3, 8192, d, E, k, f, 1) >= d * E * 4
    assert lib.xmoe_workspace_bytes(1, B, d, E, k, f, 7) == 0       # unknown dtype
    # two-matrix expert: tile map + A, and tile map + dH + A; stage 0 of the redundancy-bypassing dispatch: three
    # int32 arrays over the T*k rows
    m_fwd = lib.xmoe_workspace_bytes(5, B, d, E, k, f, 1)
    m_bwd = lib.xmoe_workspace_bytes(6, B, d, E, k, f, 1)
    assert B * f * 2 <= m_fwd < 2 * B * f * 2 and 2 * B * f * 2 <= m_bwd < 3 * B * f * 2
    rbd = lib.xmoe_workspace_bytes(7, 8192, d, E, k, f, 1)
    assert 3 * 8192 * k * 4 <= rbd < 4 * 8192 * k * 4
    assert lib.xmoe_workspace_bytes(8, B, d, E, k, f, 1) == 0       # unknown op
    assert lib.xmoe_workspace_bytes(42, B, d, E, k, f, 1) == 0      # unknown op
    for op in range(4):
        assert lib.xmoe_workspace_bytes(op, B, d, E, k, f, 1) % 256 == 0


def test_bad_arguments_are_rejected_on_the_host(lib):
    """None of these reaches a kernel launch: the status comes back although no GPU is present."""
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3
    p = ctypes.c_void_p(4096)            # never dereferenced on the host
    null = None
    assert lib.xmoe_route(p, 16, 8, 9, p, p, null) == INVALID               # k > E
    assert lib.xmoe_route(p, 16, 8, 0, p, p, null) == INVALID               # k < 1
    assert lib.xmoe_route(p, 16, 1024, 2, p, p, null) == UNSUPPORTED        # E beyond the limit
    assert lib.xmoe_route(p, 1 << 30, 8, 4, p, p, null) == INVALID          # T*k >= 2^31
    assert lib.xmoe_route(null, 16, 8, 2, p, p, null) == INVALID            # null pointer
    assert lib.xmoe_gate_logits(p, p, null, p, 16, 32, 8, 5, null) == UNSUPPORTED      # dtype
    assert lib.xmoe_gate_logits(null, p, null, p, 16, 32, 8, 0, null) == INVALID
    assert lib.xmoe_build_eri(p, p, 16, 8, 9, p, p, p, p, p, p, p, 1 << 20, null) == INVALID
    assert lib.xmoe_build_eri(p, p, 16, 8, 2, p, p, p, p, p, p, null, 0, null) == WORKSPACE
    assert lib.xmoe_build_eri(p, p, 4096, 8, 2, p, p, p, p, p, p, p, 16, null) == WORKSPACE
    assert lib.xmoe_build_eri(p, p, 16, 8, 2, p, p, p, p, p, p, ctypes.c_void_p(4100), 1 << 20, null) == WORKSPACE
    assert lib.xmoe_build_eri_capped(p, p, 16, 8, 2, -1, p, p, p, p, p, p, p, 1 << 20, null) == INVALID   # capacity < 0
    assert lib.xmoe_build_eri_capped(p, p, 16, 8, 2, 4, p, p, p, p, p, p, p, 16, null) == WORKSPACE
    assert lib.xmoe_build_eri_capped(p, p, 16, 8, 2, 4, p, p, null, p, p, p, p, 1 << 20, null) == INVALID
    assert lib.xmoe_dispatch(p, p, 16, 32, 64, 9, p, null) == UNSUPPORTED
    assert lib.xmoe_dispatch(null, p, 16, 32, 64, 0, p, null) == INVALID
    assert lib.xmoe_expert_ffn_fwd(p, null, p, 32, 8, 64, 32, p, p, p, p, p, p, 1, p, 16, null) == WORKSPACE
    assert lib.xmoe_expert_ffn_fwd(p, null, null, 32, 8, 64, 32, p, p, p, p, p, p, 1, p, 1 << 30, null) == INVALID
    assert lib.xmoe_expert_ffn_bwd(p, null, p, p, p, null, null, null, p, 32, 8, 64, 32, p, p, p, p, p, p, p, 1, p, 16,
                                   null) == WORKSPACE
    assert lib.xmoe_expert_ffn_bwd(p, null, p, p, p, null, p, null, p, 32, 8, 64, 32, p, p, p, p, p, p, p, 1, p, 1 << 20,
                                   null) == INVALID                          # a row scale without a row index
    assert lib.xmoe_combine_bwd_weights(null, p, 16, 2, p, null) == INVALID
    assert lib.xmoe_combine_bwd_weights(p, p, 16, 0, p, null) == INVALID     # k < 1
    # the entry point with the static scratch array: sizes beyond the array are refused before anything is enqueued
    assert lib.xmoe_build_eri_static(p, p, 600000, 512, 1, p, p, p, p, p, p, null) == WORKSPACE
    assert lib.xmoe_build_eri_static(p, p, 16, 8, 9, p, p, p, p, p, p, null) == INVALID
    assert lib.xmoe_combine(p, p, p, null, 0, null, null, 16, 0, 64, 1, p, null) == INVALID
    assert lib.xmoe_combine(null, p, p, null, 0, null, null, 16, 2, 64, 1, p, null) == INVALID
    assert lib.xmoe_combine(p, p, p, null, 2, null, null, 16, 2, 64, 1, p, null) == INVALID     # shared rows missing
    assert lib.xmoe_combine(p, p, p, p, -1, null, null, 16, 2, 64, 1, p, null) == INVALID
    assert lib.xmoe_dispatch_bwd(p, p, null, 1, null, null, 16, 2, 64, 1, p, null) == INVALID
    assert lib.xmoe_append_shared_segments(null, p, p, 16, 8, 2, null) == INVALID
    assert lib.xmoe_append_shared_segments(p, p, p, 16, 8, 0, null) == 0     # nothing to append
    assert lib.xmoe_combine_bwd(p, p, p, null, 16, 2, 64, 1, p, p, null) == INVALID   # dy wanted, no weights
    assert lib.xmoe_combine_bwd(p, p, p, null, 16, 2, 64, 1, null, null, null) == INVALID   # no dw
    assert lib.xmoe_route_bwd(p, p, p, 16, 8, 9, p, null) == INVALID
    assert lib.xmoe_gate_logits_bwd(p, p, p, 16, 64, 8, 1, p, p, null, 0, null) == WORKSPACE


def test_empty_inputs_are_ok_without_a_launch(lib):
    p = ctypes.c_void_p(4096)
    assert lib.xmoe_route(p, 0, 8, 2, p, p, None) == 0
    assert lib.xmoe_gate_logits(p, p, None, p, 0, 32, 8, 1, None) == 0
    assert lib.xmoe_dispatch(p, p, 16, 0, 64, 1, p, None) == 0
    assert lib.xmoe_combine(p, p, p, None, 0, None, None, 0, 2, 64, 1, p, None) == 0


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_13337_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.replace("no CPU or PyTorch fallback", ""), fn
