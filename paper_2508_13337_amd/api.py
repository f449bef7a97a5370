"""Python binding of the C ABI (include/xmoe.h): same names, argument marshalling only.

Every function takes torch tensors that live on the GPU (torch supplies device memory and the current stream),
checks dtype / contiguity / shape on the host, passes raw device pointers to libxmoe and raises XMoEError on a
non-zero status.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import ctypes
from typing import Optional

import torch

from ._lib import lib

XMOE_F32, XMOE_BF16 = 0, 1
WS_BUILD_ERI, WS_FFN_FWD, WS_FFN_BWD, WS_GATE_BWD, WS_BUILD_ERI_CAPPED, WS_MLP2_FWD, WS_MLP2_BWD = 0, 1, 2, 3, 4, 5, 6
WS_RBD_STAGE0 = 7
ACT_CODES = {"identity": 0, "gelu": 1, "silu": 2}   # xmoe_act

__all__ = [
    "XMoEError", "xmoe_version", "xmoe_workspace_bytes", "xmoe_gate_logits", "xmoe_route", "xmoe_build_eri",
    "xmoe_dispatch", "xmoe_expert_ffn_fwd", "xmoe_expert_ffn_bwd", "xmoe_combine", "xmoe_combine_bwd",
    "xmoe_dispatch_bwd", "xmoe_route_bwd", "xmoe_gate_logits_bwd", "xmoe_prof_enable", "xmoe_prof_reset",
    "xmoe_prof_read", "xmoe_prof_copy", "xmoe_prof_shader_clocks", "dtype_code", "alloc_workspace",
    "XMOE_F32", "XMOE_BF16", "WS_BUILD_ERI", "WS_FFN_FWD", "WS_FFN_BWD", "WS_GATE_BWD", "WS_BUILD_ERI_CAPPED", "xmoe_build_eri_capped",
    "xmoe_expert_mlp2_fwd", "xmoe_expert_mlp2_bwd", "WS_MLP2_FWD", "WS_MLP2_BWD", "ACT_CODES",
    "xmoe_rbd_stage0", "xmoe_rbd_absolute_index", "WS_RBD_STAGE0", "xmoe_build_eri_static", "xmoe_combine_bwd_weights", "xmoe_append_shared_segments",
]


class XMoEError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().xmoe_status_string(status).decode()} (status {status})")


def _check(status: int, where: str) -> None:
    if status != 0:
        raise XMoEError(status, where)


def dtype_code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return XMOE_F32
    if dt == torch.bfloat16:
        return XMOE_BF16
    raise TypeError(f"xmoe supports float32 and bfloat16 storage, not {dt}")


def _ptr(t: Optional[torch.Tensor], dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def xmoe_version() -> str:
    return lib().xmoe_version().decode()


def xmoe_workspace_bytes(op: int, rows: int, d: int, E: int, k: int, f: int, dt: int) -> int:
    return int(lib().xmoe_workspace_bytes(op, rows, d, E, k, f, dt))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """A byte tensor of at least nbytes whose base is 256-byte aligned (torch's allocator aligns to 512)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def xmoe_gate_logits(x, w_router, bias, logits) -> None:
    T, d = x.shape
    E = w_router.shape[1]
    assert w_router.shape[0] == d and tuple(logits.shape) == (T, E)
    _check(lib().xmoe_gate_logits(_ptr(x, None, "x"), _ptr(w_router, x.dtype, "w_router"),
                                  _ptr(bias, torch.float32, "bias"), _ptr(logits, torch.float32, "logits"),
                                  T, d, E, dtype_code(x.dtype), _stream()), "xmoe_gate_logits")


def xmoe_route(logits, k: int, topk_idx, topk_w) -> None:
    T, E = logits.shape
    assert tuple(topk_idx.shape) == (T, k) and tuple(topk_w.shape) == (T, k)
    _check(lib().xmoe_route(_ptr(logits, torch.float32, "logits"), T, E, k, _ptr(topk_idx, torch.int32, "topk_idx"),
                            _ptr(topk_w, torch.float32, "topk_w"), _stream()), "xmoe_route")


def xmoe_build_eri(topk_idx, topk_w, E: int, tokens_per_expert, expert_offsets, token_ids, expert_ids,
                   combine_weights, row_of_slot, ws) -> None:
    T, k = topk_idx.shape
    B = T * k
    assert tokens_per_expert.numel() == E and expert_offsets.numel() == E + 1
    assert token_ids.numel() == B and expert_ids.numel() == B and combine_weights.numel() == B
    assert row_of_slot.numel() == B
    _check(lib().xmoe_build_eri(
        _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(topk_w, torch.float32, "topk_w"), T, E, k,
        _ptr(tokens_per_expert, torch.int32), _ptr(expert_offsets, torch.int32), _ptr(token_ids, torch.int32),
        _ptr(expert_ids, torch.int32), _ptr(combine_weights, torch.float32), _ptr(row_of_slot, torch.int32),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream()), "xmoe_build_eri")


def xmoe_build_eri_static(topk_idx, topk_w, E: int, tokens_per_expert, expert_offsets, token_ids, expert_ids,
                          combine_weights, row_of_slot) -> None:
    """xmoe_build_eri without a workspace: the scratch is a static array inside the library (for callers that cannot
    allocate)."""
    T, k = topk_idx.shape
    B = T * k
    assert tokens_per_expert.numel() == E and expert_offsets.numel() == E + 1
    assert token_ids.numel() == B and expert_ids.numel() == B and combine_weights.numel() == B
    assert row_of_slot.numel() == B
    _check(lib().xmoe_build_eri_static(
        _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(topk_w, torch.float32, "topk_w"), T, E, k,
        _ptr(tokens_per_expert, torch.int32), _ptr(expert_offsets, torch.int32), _ptr(token_ids, torch.int32),
        _ptr(expert_ids, torch.int32), _ptr(combine_weights, torch.float32), _ptr(row_of_slot, torch.int32),
        _stream()), "xmoe_build_eri_static")


def xmoe_build_eri_capped(topk_idx, topk_w, E: int, max_token_count: int, tokens_per_expert, expert_offsets, token_ids,
                          expert_ids, combine_weights, row_of_slot, ws) -> None:
    T, k = topk_idx.shape
    B = T * k
    assert tokens_per_expert.numel() == E and expert_offsets.numel() == E + 1
    assert token_ids.numel() == B and expert_ids.numel() == B and combine_weights.numel() == B
    assert row_of_slot.numel() == B
    _check(lib().xmoe_build_eri_capped(
        _ptr(topk_idx, torch.int32, "topk_idx"), _ptr(topk_w, torch.float32, "topk_w"), T, E, k, int(max_token_count),
        _ptr(tokens_per_expert, torch.int32), _ptr(expert_offsets, torch.int32), _ptr(token_ids, torch.int32),
        _ptr(expert_ids, torch.int32), _ptr(combine_weights, torch.float32), _ptr(row_of_slot, torch.int32),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream()), "xmoe_build_eri_capped")


def xmoe_rbd_stage0(topk_idx, rand_key, token_ids, expert_ids, expert_offsets, row_of_slot, experts_per_node: int,
                    out: dict, ws) -> None:
    """Stage 0 of the redundancy-bypassing dispatch.  rand_key: int32 tensor holding the uint32 draws' bit patterns.
    out: preallocated int32 tensors pilot_token_ids, pilot_expert_ids, replica_token_ids, replica_expert_ids,
    s1_mapping_indices, s1_mapping_experts, merge_src [T*k]; pilot_tokens_per_expert, replica_tokens_per_expert [E];
    pilot_offsets, replica_offsets [E+1]."""
    T, k = topk_idx.shape
    B = T * k
    E = expert_offsets.numel() - 1
    for name in ("pilot_token_ids", "pilot_expert_ids", "replica_token_ids", "replica_expert_ids",
                 "s1_mapping_indices", "s1_mapping_experts", "merge_src"):
        assert out[name].numel() == B, name
    for name in ("pilot_tokens_per_expert", "replica_tokens_per_expert"):
        assert out[name].numel() == E, name
    for name in ("pilot_offsets", "replica_offsets"):
        assert out[name].numel() == E + 1, name
    assert rand_key.numel() == B and token_ids.numel() == B and expert_ids.numel() == B and row_of_slot.numel() == B
    i32 = torch.int32
    _check(lib().xmoe_rbd_stage0(
        _ptr(topk_idx, i32, "topk_idx"), _ptr(rand_key, i32, "rand_key"), _ptr(token_ids, i32, "token_ids"),
        _ptr(expert_ids, i32, "expert_ids"), _ptr(expert_offsets, i32, "expert_offsets"),
        _ptr(row_of_slot, i32, "row_of_slot"), T, E, k, int(experts_per_node),
        _ptr(out["pilot_token_ids"], i32), _ptr(out["pilot_expert_ids"], i32),
        _ptr(out["pilot_tokens_per_expert"], i32), _ptr(out["pilot_offsets"], i32),
        _ptr(out["replica_token_ids"], i32), _ptr(out["replica_expert_ids"], i32),
        _ptr(out["replica_tokens_per_expert"], i32), _ptr(out["replica_offsets"], i32),
        _ptr(out["s1_mapping_indices"], i32), _ptr(out["s1_mapping_experts"], i32), _ptr(out["merge_src"], i32),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream()), "xmoe_rbd_stage0")


def xmoe_rbd_absolute_index(s1_mapping_indices, s1_mapping_experts, pilot_offsets_at_destination, absolute) -> None:
    n = s1_mapping_indices.numel()
    E = pilot_offsets_at_destination.numel() - 1
    assert s1_mapping_experts.numel() == n and absolute.numel() == n
    i32 = torch.int32
    _check(lib().xmoe_rbd_absolute_index(_ptr(s1_mapping_indices, i32), _ptr(s1_mapping_experts, i32),
                                         _ptr(pilot_offsets_at_destination, i32), n, E, _ptr(absolute, i32),
                                         _stream()), "xmoe_rbd_absolute_index")


def xmoe_dispatch(x, token_ids, xd) -> None:
    T, d = x.shape
    B = token_ids.numel()
    assert tuple(xd.shape) == (B, d) and xd.dtype == x.dtype
    _check(lib().xmoe_dispatch(_ptr(x, None, "x"), _ptr(token_ids, torch.int32, "token_ids"), T, B, d,
                               dtype_code(x.dtype), _ptr(xd, None, "xd"), _stream()), "xmoe_dispatch")


def xmoe_expert_ffn_fwd(xd, expert_offsets, wg, wu, wd, g_save, u_save, y, ws, row_index=None) -> None:
    """row_index: None, or token ids [B]: xd is then the token matrix x [T,d] and row i of the input is x[row_index[i]]."""
    B = xd.shape[0] if row_index is None else row_index.numel()
    d = xd.shape[1]
    E, d2, f = wg.shape
    dt = xd.dtype
    assert d2 == d and tuple(wu.shape) == (E, d, f) and tuple(wd.shape) == (E, f, d)
    assert expert_offsets.numel() == E + 1
    assert tuple(g_save.shape) == (B, f) and tuple(u_save.shape) == (B, f) and tuple(y.shape) == (B, d)
    _check(lib().xmoe_expert_ffn_fwd(
        _ptr(xd, None, "xd"), _ptr(row_index, torch.int32, "row_index"),
        _ptr(expert_offsets, torch.int32, "expert_offsets"), B, E, d, f,
        _ptr(wg, dt, "wg"), _ptr(wu, dt, "wu"), _ptr(wd, dt, "wd"), _ptr(g_save, dt, "g_save"),
        _ptr(u_save, dt, "u_save"), _ptr(y, dt, "y"), dtype_code(dt), _ptr(ws, torch.uint8, "ws"), ws.numel(),
        _stream()), "xmoe_expert_ffn_fwd")


def _check_dy(dy, B, d, dy_row_index, dy_row_scale):
    if dy_row_index is None:
        assert dy_row_scale is None and tuple(dy.shape) == (B, d)
    else:
        assert dy.shape[1] == d and dy_row_index.numel() == B
        assert dy_row_scale is None or dy_row_scale.numel() == B


def xmoe_expert_ffn_bwd(xd, g_save, u_save, dy, expert_offsets, wg, wu, wd, dxd, dwg, dwu, dwd, ws,
                        row_index=None, dy_row_index=None, dy_row_scale=None, dy_row_scale_grad=None) -> None:
    """dy_row_index: None, or token ids [B]: dy is then dout [T,d] and row i of dY is dy_row_scale[i] * dout[dy_row_index[i]]
    (dy_row_scale None = 1): the backward of combine fused into the operand loads.
    dy_row_scale_grad: None, or a float32 [B] output for <row i of dY before the scale, Y[i]>."""
    B = xd.shape[0] if row_index is None else row_index.numel()
    d = xd.shape[1]
    E, d2, f = wg.shape
    dt = xd.dtype
    assert d2 == d and tuple(wu.shape) == (E, d, f) and tuple(wd.shape) == (E, f, d)
    assert tuple(dwg.shape) == (E, d, f) and tuple(dwu.shape) == (E, d, f) and tuple(dwd.shape) == (E, f, d)
    assert tuple(g_save.shape) == (B, f) and tuple(u_save.shape) == (B, f)
    assert tuple(dxd.shape) == (B, d)
    _check_dy(dy, B, d, dy_row_index, dy_row_scale)
    _check(lib().xmoe_expert_ffn_bwd(
        _ptr(xd, None, "xd"), _ptr(row_index, torch.int32, "row_index"), _ptr(g_save, dt, "g_save"),
        _ptr(u_save, dt, "u_save"), _ptr(dy, dt, "dy"), _ptr(dy_row_index, torch.int32, "dy_row_index"),
        _ptr(dy_row_scale, torch.float32, "dy_row_scale"), _ptr(dy_row_scale_grad, torch.float32, "dy_row_scale_grad"),
        _ptr(expert_offsets, torch.int32, "expert_offsets"), B, E, d, f, _ptr(wg, dt), _ptr(wu, dt), _ptr(wd, dt),
        _ptr(dxd, dt, "dxd"), _ptr(dwg, dt, "dwg"), _ptr(dwu, dt, "dwu"), _ptr(dwd, dt, "dwd"), dtype_code(dt),
        _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream()), "xmoe_expert_ffn_bwd")


def xmoe_expert_mlp2_fwd(xd, expert_offsets, w1, w2, act: str, h_save, y, ws, row_index=None) -> None:
    """The paper's two-matrix expert.  act: "identity" | "gelu" | "silu".  row_index: as in xmoe_expert_ffn_fwd."""
    B = xd.shape[0] if row_index is None else row_index.numel()
    d = xd.shape[1]
    E, d2, f = w1.shape
    dt = xd.dtype
    assert d2 == d and tuple(w2.shape) == (E, f, d) and expert_offsets.numel() == E + 1
    assert tuple(h_save.shape) == (B, f) and tuple(y.shape) == (B, d)
    _check(lib().xmoe_expert_mlp2_fwd(
        _ptr(xd, None, "xd"), _ptr(row_index, torch.int32, "row_index"),
        _ptr(expert_offsets, torch.int32, "expert_offsets"), B, E, d, f, _ptr(w1, dt, "w1"), _ptr(w2, dt, "w2"),
        ACT_CODES[act], _ptr(h_save, dt, "h_save"), _ptr(y, dt, "y"), dtype_code(dt), _ptr(ws, torch.uint8, "ws"),
        ws.numel(), _stream()), "xmoe_expert_mlp2_fwd")


def xmoe_expert_mlp2_bwd(xd, h_save, dy, expert_offsets, w1, w2, act: str, dxd, dw1, dw2, ws, row_index=None,
                         dy_row_index=None, dy_row_scale=None, dy_row_scale_grad=None) -> None:
    B = xd.shape[0] if row_index is None else row_index.numel()
    d = xd.shape[1]
    E, d2, f = w1.shape
    dt = xd.dtype
    assert d2 == d and tuple(w2.shape) == (E, f, d)
    assert tuple(dw1.shape) == (E, d, f) and tuple(dw2.shape) == (E, f, d)
    assert tuple(h_save.shape) == (B, f) and tuple(dxd.shape) == (B, d)
    _check_dy(dy, B, d, dy_row_index, dy_row_scale)
    _check(lib().xmoe_expert_mlp2_bwd(
        _ptr(xd, None, "xd"), _ptr(row_index, torch.int32, "row_index"), _ptr(h_save, dt, "h_save"),
        _ptr(dy, dt, "dy"), _ptr(dy_row_index, torch.int32, "dy_row_index"),
        _ptr(dy_row_scale, torch.float32, "dy_row_scale"), _ptr(dy_row_scale_grad, torch.float32, "dy_row_scale_grad"),
        _ptr(expert_offsets, torch.int32, "expert_offsets"), B, E, d, f, _ptr(w1, dt, "w1"),
        _ptr(w2, dt, "w2"), ACT_CODES[act], _ptr(dxd, dt, "dxd"), _ptr(dw1, dt, "dw1"), _ptr(dw2, dt, "dw2"),
        dtype_code(dt), _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream()), "xmoe_expert_mlp2_bwd")


def _shared_args(shared_rows, shared_row0, n_shared, T, d):
    """(rows tensor, count): without shared_row0 the count follows from the tensor; with it (a device int32: the row
    of the larger buffer `shared_rows` at which the shared experts' rows start) the caller states it."""
    if shared_rows is None:
        assert shared_row0 is None
        return 0
    assert shared_rows.shape[1] == d
    if shared_row0 is None:
        assert shared_rows.shape[0] % T == 0
        return shared_rows.shape[0] // T
    assert n_shared is not None and shared_row0.numel() == 1 and shared_rows.shape[0] >= n_shared * T
    return int(n_shared)


def xmoe_combine(y, row_of_slot, topk_w, shared_rows, addend, k: int, out, shared_row0=None, n_shared=None) -> None:
    """shared_rows: None or an [n_shared*T, d] tensor (rows of experts every token visits with weight 1); with
    shared_row0 (one int32 on the device) the whole row buffer, in which those rows start at row shared_row0[0]."""
    T, d = out.shape
    dt = out.dtype
    assert y.shape[1] == d and row_of_slot.numel() == T * k
    n_shared = _shared_args(shared_rows, shared_row0, n_shared, T, d)
    _check(lib().xmoe_combine(_ptr(y, dt, "y"), _ptr(row_of_slot, torch.int32, "row_of_slot"),
                              _ptr(topk_w, torch.float32, "topk_w"), _ptr(shared_rows, dt, "shared_rows"), n_shared,
                              _ptr(shared_row0, torch.int32, "shared_row0"),
                              _ptr(addend, dt, "addend"), T, k, d, dtype_code(dt), _ptr(out, None, "out"),
                              _stream()), "xmoe_combine")


def xmoe_append_shared_segments(expert_offsets, token_ids, combine_weights, T: int, E: int, n_shared: int) -> None:
    """Continues expert_offsets [E+1+n_shared], token_ids and combine_weights behind the last row of a PFT whose row
    count only the device knows, with n_shared all-token segments."""
    assert expert_offsets.numel() >= E + 1 + n_shared
    assert token_ids.numel() == combine_weights.numel()
    _check(lib().xmoe_append_shared_segments(_ptr(expert_offsets, torch.int32, "expert_offsets"),
                                             _ptr(token_ids, torch.int32, "token_ids"),
                                             _ptr(combine_weights, torch.float32, "combine_weights"), T, E, n_shared,
                                             _stream()), "xmoe_append_shared_segments")


def xmoe_combine_bwd(dout, y, row_of_slot, topk_w, dy, dw) -> None:
    """dy None: only dw is computed (the expert MLP's backward then takes dout, token ids and combine weights)."""
    T, d = dout.shape
    k = dw.shape[1]
    dt = dout.dtype
    assert tuple(y.shape) == (T * k, d) and tuple(dw.shape) == (T, k)
    assert dy is None or tuple(dy.shape) == (T * k, d)
    _check(lib().xmoe_combine_bwd(_ptr(dout, None, "dout"), _ptr(y, dt, "y"),
                                  _ptr(row_of_slot, torch.int32, "row_of_slot"),
                                  _ptr(topk_w, torch.float32, "topk_w"), T, k, d, dtype_code(dt), _ptr(dy, dt, "dy"),
                                  _ptr(dw, torch.float32, "dw"), _stream()), "xmoe_combine_bwd")


def xmoe_combine_bwd_weights(row_grad, row_of_slot, dw) -> None:
    """dw[t,j] = row_grad[row_of_slot[t*k+j]] (0 for a dropped entry)."""
    T, k = dw.shape
    assert row_of_slot.numel() == T * k
    _check(lib().xmoe_combine_bwd_weights(_ptr(row_grad, torch.float32, "row_grad"),
                                          _ptr(row_of_slot, torch.int32, "row_of_slot"), T, k,
                                          _ptr(dw, torch.float32, "dw"), _stream()), "xmoe_combine_bwd_weights")


def xmoe_dispatch_bwd(dxd, row_of_slot, shared_rows, addend, k: int, dx, shared_row0=None, n_shared=None) -> None:
    T, d = dx.shape
    dt = dx.dtype
    assert dxd.shape[0] >= T * k and dxd.shape[1] == d
    n_shared = _shared_args(shared_rows, shared_row0, n_shared, T, d)
    _check(lib().xmoe_dispatch_bwd(_ptr(dxd, dt, "dxd"), _ptr(row_of_slot, torch.int32, "row_of_slot"),
                                   _ptr(shared_rows, dt, "shared_rows"), n_shared,
                                   _ptr(shared_row0, torch.int32, "shared_row0"), _ptr(addend, dt, "addend"), T, k, d,
                                   dtype_code(dt), _ptr(dx, None, "dx"), _stream()), "xmoe_dispatch_bwd")


def xmoe_route_bwd(logits, topk_idx, dw, dlogits) -> None:
    T, E = logits.shape
    k = topk_idx.shape[1]
    assert tuple(dw.shape) == (T, k) and tuple(dlogits.shape) == (T, E)
    _check(lib().xmoe_route_bwd(_ptr(logits, torch.float32, "logits"), _ptr(topk_idx, torch.int32, "topk_idx"),
                                _ptr(dw, torch.float32, "dw"), T, E, k, _ptr(dlogits, torch.float32, "dlogits"),
                                _stream()), "xmoe_route_bwd")


def xmoe_gate_logits_bwd(x, w_router, dlogits, dw_router, dx_gate, ws) -> None:
    T, d = x.shape
    E = w_router.shape[1]
    dt = x.dtype
    assert tuple(dlogits.shape) == (T, E) and tuple(dw_router.shape) == (d, E) and tuple(dx_gate.shape) == (T, d)
    _check(lib().xmoe_gate_logits_bwd(_ptr(x, None, "x"), _ptr(w_router, dt, "w_router"),
                                      _ptr(dlogits, torch.float32, "dlogits"), T, d, E, dtype_code(dt),
                                      _ptr(dw_router, dt, "dw_router"), _ptr(dx_gate, dt, "dx_gate"),
                                      _ptr(ws, torch.uint8, "ws"), ws.numel(), _stream()), "xmoe_gate_logits_bwd")


def xmoe_prof_enable(on: bool) -> None:
    lib().xmoe_prof_enable(1 if on else 0)


def xmoe_prof_reset() -> None:
    lib().xmoe_prof_reset()


def xmoe_prof_copy(src, dst) -> None:
    """dst = src through the library's plain copy kernel (counter calibration)."""
    assert src.numel() * src.element_size() == dst.numel() * dst.element_size()
    _check(lib().xmoe_prof_copy(_ptr(src, None, "src"), _ptr(dst, None, "dst"), src.numel() * src.element_size(),
                                _stream()), "xmoe_prof_copy")


def xmoe_prof_shader_clocks() -> dict:
    """{kernel name: GHz} for the matrix-core kernels of the expert MLP that have run (their last launch)."""
    out = {}
    ghz = ctypes.c_double()
    for kid in range(lib().xmoe_prof_num_kernels()):
        _check(lib().xmoe_prof_shader_clock(kid, ctypes.byref(ghz)), "xmoe_prof_shader_clock")
        if ghz.value > 0.0:
            out[lib().xmoe_prof_kernel_name(kid).decode()] = ghz.value
    return out


def xmoe_prof_read() -> dict:
    """{kernel name: (launches, total milliseconds)} for every kernel that was launched while profiling."""
    out = {}
    n = ctypes.c_int()
    ms = ctypes.c_double()
    for kid in range(lib().xmoe_prof_num_kernels()):
        _check(lib().xmoe_prof_get(kid, ctypes.byref(n), ctypes.byref(ms)), "xmoe_prof_get")
        if n.value:
            out[lib().xmoe_prof_kernel_name(kid).decode()] = (n.value, ms.value)
    return out
