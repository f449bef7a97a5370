"""One padding-free MoE layer as a sequence of libxmoe calls (Listing 1's call(): gating -> PFT construction
-> dispatch -> mlp -> combine, then the mirrored backward).  This class only owns the device buffers and the
order of the calls; all arithmetic happens inside the HIP kernels."""
from __future__ import annotations

from typing import Optional

import torch

from . import api


def fuse_shared(w: torch.Tensor, which: str) -> torch.Tensor:
    """Stack E_s shared experts into the one wide expert the library runs them as.
    wg / wu [E_s, d, f] -> [1, d, E_s*f];  wd [E_s, f, d] -> [1, E_s*f, d].  Pure data movement."""
    Es = w.shape[0]
    if which in ("wg", "wu"):
        _, d, f = w.shape
        return w.permute(1, 0, 2).reshape(1, d, Es * f).contiguous()
    _, f, d = w.shape
    return w.reshape(1, Es * f, d).contiguous()


def unfuse_shared_grad(g: torch.Tensor, which: str, Es: int) -> torch.Tensor:
    """Inverse of fuse_shared for gradients."""
    if which in ("wg", "wu"):
        _, d, ff = g.shape
        return g.reshape(d, Es, ff // Es).permute(1, 0, 2).contiguous()
    _, ff, d = g.shape
    return g.reshape(Es, ff // Es, d).contiguous()


class XMoELayer:
    """Buffers and call order for one layer of T tokens; weights are passed in by the caller."""

    def __init__(self, T: int, d: int, E: int, k: int, f: int, dtype: torch.dtype, E_s: int = 0, device="cuda"):
        self.T, self.d, self.E, self.k, self.f, self.E_s = T, d, E, k, f, E_s
        self.dtype, self.device = dtype, device
        B = T * k
        self.B = B
        dt = api.dtype_code(dtype)
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        act = dict(dtype=dtype, device=device)
        self.logits = torch.empty((T, E), **f32)
        self.topk_idx = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), **f32)
        self.tokens_per_expert = torch.empty(E, **i32)
        self.expert_offsets = torch.empty(E + 1, **i32)
        self.token_ids = torch.empty(B, **i32)
        self.expert_ids = torch.empty(B, **i32)
        self.combine_weights = torch.empty(B, **f32)
        self.row_of_slot = torch.empty(B, **i32)
        self.xd = torch.empty((B, d), **act)
        self.g = torch.empty((B, f), **act)
        self.u = torch.empty((B, f), **act)
        self.y = torch.empty((B, d), **act)
        self.out = torch.empty((T, d), **act)
        # backward
        self.dy = torch.empty((B, d), **act)
        self.dw = torch.empty((T, k), **f32)
        self.dxd = torch.empty((B, d), **act)
        self.dlogits = torch.empty((T, E), **f32)
        self.dx_gate = torch.empty((T, d), **act)
        self.dx = torch.empty((T, d), **act)
        ws = max(api.xmoe_workspace_bytes(api.WS_BUILD_ERI, T, d, E, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_FFN_FWD, B, d, E, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_FFN_BWD, B, d, E, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_GATE_BWD, T, d, E, k, f, dt))
        if E_s > 0:
            fs = E_s * f
            self.sg = torch.empty((T, fs), **act)
            self.su = torch.empty((T, fs), **act)
            self.sy = torch.empty((T, d), **act)
            self.sdx = torch.empty((T, d), **act)
            self.shared_offsets = torch.tensor([0, T], **i32)
            ws = max(ws, api.xmoe_workspace_bytes(api.WS_FFN_FWD, T, d, 1, 1, fs, dt),
                     api.xmoe_workspace_bytes(api.WS_FFN_BWD, T, d, 1, 1, fs, dt))
        self.ws = api.alloc_workspace(ws, device)

    # weights: dict with w_router [d,E], bias [E]|None, wg/wu [E,d,f], wd [E,f,d] and, when E_s > 0,
    # shared_wg/shared_wu [1,d,E_s*f], shared_wd [1,E_s*f,d] (see fuse_shared)
    def forward(self, x: torch.Tensor, w: dict) -> torch.Tensor:
        api.xmoe_gate_logits(x, w["w_router"], w.get("bias"), self.logits)
        api.xmoe_route(self.logits, self.k, self.topk_idx, self.topk_w)
        api.xmoe_build_eri(self.topk_idx, self.topk_w, self.E, self.tokens_per_expert, self.expert_offsets,
                           self.token_ids, self.expert_ids, self.combine_weights, self.row_of_slot, self.ws)
        api.xmoe_dispatch(x, self.token_ids, self.xd)
        api.xmoe_expert_ffn_fwd(self.xd, self.expert_offsets, w["wg"], w["wu"], w["wd"], self.g, self.u, self.y,
                                self.ws)
        addend = None
        if self.E_s > 0:
            api.xmoe_expert_ffn_fwd(x, self.shared_offsets, w["shared_wg"], w["shared_wu"], w["shared_wd"],
                                    self.sg, self.su, self.sy, self.ws)
            addend = self.sy
        api.xmoe_combine(self.y, self.row_of_slot, self.topk_w, addend, None, self.k, self.out)
        return self.out

    def backward(self, x: torch.Tensor, w: dict, dout: torch.Tensor, grads: dict) -> torch.Tensor:
        """grads: preallocated dw_router, dwg, dwu, dwd (+ dshared_wg/wu/wd) in the layouts of the weights."""
        api.xmoe_combine_bwd(dout, self.y, self.row_of_slot, self.topk_w, self.dy, self.dw)
        api.xmoe_expert_ffn_bwd(self.xd, self.g, self.u, self.dy, self.expert_offsets, w["wg"], w["wu"], w["wd"],
                                self.dxd, grads["dwg"], grads["dwu"], grads["dwd"], self.ws)
        add1 = None
        if self.E_s > 0:
            api.xmoe_expert_ffn_bwd(x, self.sg, self.su, dout, self.shared_offsets, w["shared_wg"],
                                    w["shared_wu"], w["shared_wd"], self.sdx, grads["dshared_wg"],
                                    grads["dshared_wu"], grads["dshared_wd"], self.ws)
            add1 = self.sdx
        api.xmoe_route_bwd(self.logits, self.topk_idx, self.dw, self.dlogits)
        api.xmoe_gate_logits_bwd(x, w["w_router"], self.dlogits, grads["dw_router"], self.dx_gate, self.ws)
        api.xmoe_dispatch_bwd(self.dxd, self.row_of_slot, add1, self.dx_gate, self.k, self.dx)
        return self.dx
