"""One padding-free MoE layer as a sequence of libxmoe calls (Listing 1's call(): gating -> PFT construction
-> dispatch -> mlp -> combine, then the mirrored backward).  This class only owns the device buffers and the
order of the calls; all arithmetic happens inside the HIP kernels."""
from __future__ import annotations

from typing import Optional

import torch

from . import api


def append_shared(w_routed: torch.Tensor, w_shared: Optional[torch.Tensor]) -> torch.Tensor:
    """Weights of the E routed experts followed by those of the E_s shared experts, [E+E_s, ...]: the layout the
    layer hands to the expert-MLP calls.  Pure data movement."""
    if w_shared is None or w_shared.shape[0] == 0:
        return w_routed
    return torch.cat([w_routed, w_shared], dim=0).contiguous()


class XMoELayer:
    """Buffers and call order for one layer of T tokens; weights are passed in by the caller.

    The gather of dispatch is fused into the expert MLP's operand loads: the MLP reads x through token_ids, and no
    [B,d] copy of the tokens exists.  The backward of combine is fused the same way (fuse_combine_bwd, the default):
    the MLP's backward reads dOut through token_ids and scales by combine_weights, so no [B,d] gradient of the expert
    outputs exists, and it also returns the gradient of every row's combine weight (dy_row_scale_grad), which
    xmoe_combine_bwd_weights puts into slot order: the expert outputs Y are then read by the forward combine only
    and nothing but G and U is held between forward and backward.  (Without fuse_combine_bwd, xmoe_combine_bwd
    reads Y back for the weights' gradient and writes dY, and xmoe_dispatch copies dOut into the shared experts'
    dY rows.)
    Shared experts (every token, weight 1) run inside the same grouped-GEMM launches as the routed ones: they are
    experts E .. E+E_s-1 whose segments are rows [B + s*T, B + (s+1)*T) and read x[0..T-1], so the tail of
    expert_offsets and of token_ids is constant and written once here."""

    def __init__(self, T: int, d: int, E: int, k: int, f: int, dtype: torch.dtype, E_s: int = 0, device="cuda",
                 max_token_count: Optional[int] = None, fuse_combine_bwd: bool = True):
        self.T, self.d, self.E, self.k, self.f, self.E_s = T, d, E, k, f, E_s
        self.fuse_combine_bwd = fuse_combine_bwd
        # None: dropless.  Else the per-expert capacity of the token-dropping PFT construction; the number of
        # retained rows is then known on the device only, and xmoe_append_shared_segments continues the index arrays
        # with the shared experts' segments behind them, every step.
        self.max_token_count = max_token_count
        self.dtype, self.device = dtype, device
        B = T * k
        R = B + E_s * T          # rows of the expert MLP
        Ea = E + E_s             # experts of the expert MLP
        self.B, self.R, self.Ea = B, R, Ea
        dt = api.dtype_code(dtype)
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        act = dict(dtype=dtype, device=device)
        self.logits = torch.empty((T, E), **f32)
        self.topk_idx = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), **f32)
        self.tokens_per_expert = torch.empty(E, **i32)
        self.offsets_all = torch.empty(Ea + 1, **i32)
        self.token_ids_all = torch.empty(R, **i32)
        if E_s > 0:
            self.offsets_all[E + 1:] = B + T * torch.arange(1, E_s + 1, **i32)
            self.token_ids_all[B:] = torch.arange(T, **i32).repeat(E_s)
        self.expert_offsets = self.offsets_all[:E + 1]
        self.token_ids = self.token_ids_all[:B]
        self.expert_ids = torch.empty(B, **i32)
        # combine weight of every row of the expert MLP: the ERI-array for the routed rows, 1 for a shared expert's
        self.combine_weights_all = torch.ones(R, **f32)
        self.combine_weights = self.combine_weights_all[:B]
        self.row_of_slot = torch.empty(B, **i32)
        self.g = torch.empty((R, f), **act)
        self.u = torch.empty((R, f), **act)
        self.y = torch.empty((R, d), **act)
        self.out = torch.empty((T, d), **act)
        # backward
        self.dy = None if fuse_combine_bwd else torch.empty((R, d), **act)
        self.row_grad = torch.empty(R, **f32) if fuse_combine_bwd else None   # gradient of every row's combine weight
        self.dw = torch.empty((T, k), **f32)
        self.dxd = torch.empty((R, d), **act)
        self.dlogits = torch.empty((T, E), **f32)
        self.dx_gate = torch.empty((T, d), **act)
        self.dx = torch.empty((T, d), **act)
        ws = max(api.xmoe_workspace_bytes(api.WS_BUILD_ERI, T, d, E, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_FFN_FWD, R, d, Ea, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_FFN_BWD, R, d, Ea, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_GATE_BWD, T, d, E, k, f, dt))
        if max_token_count is not None:
            ws = max(ws, api.xmoe_workspace_bytes(api.WS_BUILD_ERI_CAPPED, T, d, E, k, f, dt))
        self.ws = api.alloc_workspace(ws, device)

    # weights: dict with w_router [d,E], bias [E]|None, wg/wu [E+E_s,d,f], wd [E+E_s,f,d] (routed experts first,
    # see append_shared)
    def forward(self, x: torch.Tensor, w: dict) -> torch.Tensor:
        api.xmoe_gate_logits(x, w["w_router"], w.get("bias"), self.logits)
        api.xmoe_route(self.logits, self.k, self.topk_idx, self.topk_w)
        B, E, T, E_s = self.B, self.E, self.T, self.E_s
        if self.max_token_count is None:
            api.xmoe_build_eri(self.topk_idx, self.topk_w, E, self.tokens_per_expert, self.expert_offsets,
                               self.token_ids, self.expert_ids, self.combine_weights, self.row_of_slot, self.ws)
        else:
            api.xmoe_build_eri_capped(self.topk_idx, self.topk_w, E, self.max_token_count, self.tokens_per_expert,
                                      self.expert_offsets, self.token_ids, self.expert_ids, self.combine_weights,
                                      self.row_of_slot, self.ws)
            if E_s > 0:   # the shared experts' segments start behind the retained rows, a count only the device has
                api.xmoe_append_shared_segments(self.offsets_all, self.token_ids_all, self.combine_weights_all, T, E,
                                                E_s)
        api.xmoe_expert_ffn_fwd(x, self.offsets_all, w["wg"], w["wu"], w["wd"], self.g, self.u, self.y,
                                self.ws, row_index=self.token_ids_all)
        y, y_shared, kw = self._row_args(self.y)
        api.xmoe_combine(y, self.row_of_slot, self.topk_w, y_shared, None, self.k, self.out, **kw)
        return self.out

    def _row_args(self, rows: torch.Tensor):
        """How xmoe_combine / xmoe_dispatch_bwd find the routed and the shared experts' rows in `rows` [R,d]:
        (routed rows, shared rows, keyword arguments)."""
        B, E, E_s = self.B, self.E, self.E_s
        if E_s == 0:
            return rows[:B], None, {}
        if self.max_token_count is None:
            return rows[:B], rows[B:], {}
        # the shared segments start behind the retained rows: their first row is expert_offsets[E], on the device
        return rows, rows, {"shared_row0": self.offsets_all[E:E + 1], "n_shared": E_s}

    def backward(self, x: torch.Tensor, w: dict, dout: torch.Tensor, grads: dict) -> torch.Tensor:
        """grads: preallocated dw_router, dwg, dwu, dwd in the layouts of the weights."""
        B = self.B
        if self.fuse_combine_bwd:
            api.xmoe_expert_ffn_bwd(x, self.g, self.u, dout, self.offsets_all, w["wg"], w["wu"], w["wd"],
                                    self.dxd, grads["dwg"], grads["dwu"], grads["dwd"], self.ws,
                                    row_index=self.token_ids_all, dy_row_index=self.token_ids_all,
                                    dy_row_scale=self.combine_weights_all, dy_row_scale_grad=self.row_grad)
            api.xmoe_combine_bwd_weights(self.row_grad, self.row_of_slot, self.dw)
        else:
            if self.E_s > 0:   # dY of a shared expert's rows is dout itself
                if self.max_token_count is None:
                    api.xmoe_dispatch(dout, self.token_ids_all[B:], self.dy[B:])
                else:          # their first row is known on the device only: every row, the routed ones overwritten next
                    api.xmoe_dispatch(dout, self.token_ids_all, self.dy)
            api.xmoe_combine_bwd(dout, self.y[:B], self.row_of_slot, self.topk_w, self.dy[:B], self.dw)
            api.xmoe_expert_ffn_bwd(x, self.g, self.u, self.dy, self.offsets_all, w["wg"], w["wu"], w["wd"],
                                    self.dxd, grads["dwg"], grads["dwu"], grads["dwd"], self.ws,
                                    row_index=self.token_ids_all)
        api.xmoe_route_bwd(self.logits, self.topk_idx, self.dw, self.dlogits)
        api.xmoe_gate_logits_bwd(x, w["w_router"], self.dlogits, grads["dw_router"], self.dx_gate, self.ws)
        dxd, dxd_shared, kw = self._row_args(self.dxd)
        api.xmoe_dispatch_bwd(dxd, self.row_of_slot, dxd_shared, self.dx_gate, self.k, self.dx, **kw)
        return self.dx


def capture_step(layer, x: torch.Tensor, w: dict, dout: torch.Tensor, grads: dict) -> "torch.cuda.CUDAGraph":
    """Records one forward + backward of `layer` (either class) into a HIP graph and returns it; `graph.replay()`
    then runs the step with one launch instead of two dozen.  The library's calls only enqueue kernels on the current
    stream (no allocation, no synchronisation, no memset nodes: counters are cleared by kernels), so they can be
    captured as they are.  All tensors are captured by address: refill x, dout and the weights in place."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):          # warm-up outside the capture (first-use initialisation of the library)
        layer.forward(x, w)
        layer.backward(x, w, dout, grads)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        layer.forward(x, w)
        layer.backward(x, w, dout, grads)
    return graph


class XMoE2Layer:
    """The same layer with the paper's own expert, Y = act(X W1) W2 (Listing 1's call(tokens, k, max_token_count,
    w1, w2)).  Buffers and call order only; dropless; the gather of dispatch is fused into the expert MLP's loads."""

    def __init__(self, T: int, d: int, E: int, k: int, f: int, dtype: torch.dtype, act: str = "gelu", device="cuda",
                 fuse_combine_bwd: bool = True):
        self.T, self.d, self.E, self.k, self.f, self.act = T, d, E, k, f, act
        self.fuse_combine_bwd = fuse_combine_bwd
        B = T * k
        self.B = B
        dt = api.dtype_code(dtype)
        i32 = dict(dtype=torch.int32, device=device)
        f32 = dict(dtype=torch.float32, device=device)
        tt = dict(dtype=dtype, device=device)
        self.logits = torch.empty((T, E), **f32)
        self.topk_idx = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), **f32)
        self.tokens_per_expert = torch.empty(E, **i32)
        self.expert_offsets = torch.empty(E + 1, **i32)
        self.token_ids = torch.empty(B, **i32)
        self.expert_ids = torch.empty(B, **i32)
        self.combine_weights = torch.empty(B, **f32)
        self.row_of_slot = torch.empty(B, **i32)
        self.h = torch.empty((B, f), **tt)
        self.y = torch.empty((B, d), **tt)
        self.out = torch.empty((T, d), **tt)
        self.dy = None if fuse_combine_bwd else torch.empty((B, d), **tt)
        self.row_grad = torch.empty(B, **f32) if fuse_combine_bwd else None
        self.dw = torch.empty((T, k), **f32)
        self.dxd = torch.empty((B, d), **tt)
        self.dlogits = torch.empty((T, E), **f32)
        self.dx_gate = torch.empty((T, d), **tt)
        self.dx = torch.empty((T, d), **tt)
        ws = max(api.xmoe_workspace_bytes(api.WS_BUILD_ERI, T, d, E, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_MLP2_FWD, B, d, E, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_MLP2_BWD, B, d, E, k, f, dt),
                 api.xmoe_workspace_bytes(api.WS_GATE_BWD, T, d, E, k, f, dt))
        self.ws = api.alloc_workspace(ws, device)

    # weights: dict with w_router [d,E], bias [E]|None, w1 [E,d,f], w2 [E,f,d]
    def forward(self, x: torch.Tensor, w: dict) -> torch.Tensor:
        api.xmoe_gate_logits(x, w["w_router"], w.get("bias"), self.logits)
        api.xmoe_route(self.logits, self.k, self.topk_idx, self.topk_w)
        api.xmoe_build_eri(self.topk_idx, self.topk_w, self.E, self.tokens_per_expert, self.expert_offsets,
                           self.token_ids, self.expert_ids, self.combine_weights, self.row_of_slot, self.ws)
        api.xmoe_expert_mlp2_fwd(x, self.expert_offsets, w["w1"], w["w2"], self.act, self.h, self.y, self.ws,
                                 row_index=self.token_ids)
        api.xmoe_combine(self.y, self.row_of_slot, self.topk_w, None, None, self.k, self.out)
        return self.out

    def backward(self, x: torch.Tensor, w: dict, dout: torch.Tensor, grads: dict) -> torch.Tensor:
        """grads: preallocated dw_router, dw1, dw2 in the layouts of the weights."""
        if self.fuse_combine_bwd:   # dY is never written and Y is not read back (see XMoELayer)
            api.xmoe_expert_mlp2_bwd(x, self.h, dout, self.expert_offsets, w["w1"], w["w2"], self.act, self.dxd,
                                     grads["dw1"], grads["dw2"], self.ws, row_index=self.token_ids,
                                     dy_row_index=self.token_ids, dy_row_scale=self.combine_weights,
                                     dy_row_scale_grad=self.row_grad)
            api.xmoe_combine_bwd_weights(self.row_grad, self.row_of_slot, self.dw)
        else:
            api.xmoe_combine_bwd(dout, self.y, self.row_of_slot, self.topk_w, self.dy, self.dw)
            api.xmoe_expert_mlp2_bwd(x, self.h, self.dy, self.expert_offsets, w["w1"], w["w2"], self.act, self.dxd,
                                     grads["dw1"], grads["dw2"], self.ws, row_index=self.token_ids)
        api.xmoe_route_bwd(self.logits, self.topk_idx, self.dw, self.dlogits)
        api.xmoe_gate_logits_bwd(x, w["w_router"], self.dlogits, grads["dw_router"], self.dx_gate, self.ws)
        api.xmoe_dispatch_bwd(self.dxd, self.row_of_slot, None, self.dx_gate, self.k, self.dx)
        return self.dx
