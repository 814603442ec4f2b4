"""The MoE-layer hot path as one object: preallocated buffers and the order of library calls.

Forward:  moe_route_topk -> moe_permute -> moe_grouped_gemm_swiglu_fwd -> moe_unpermute_combine_fwd
Backward: moe_unpermute_combine_bwd -> moe_grouped_gemm_swiglu_bwd -> moe_unpermute_combine_fwd
          (unit weights = permute backward) -> moe_route_topk_bwd

With gather=True the two copies into expert order disappear (xp and dyp are never written):
Forward:  moe_route_topk -> moe_permute (maps only) -> moe_grouped_gemm_swiglu_fwd_gather -> moe_unpermute_combine_fwd
Backward: moe_grouped_gemm_swiglu_bwd_gather -> moe_unpermute_combine_fwd (unit weights) -> moe_route_topk_bwd
and, with weight_in_forward (the default of the gathered path), the combine weight is applied inside the forward
products (act and yp leave scaled by it), so the forward combine is a plain sum and the backward finds w * act written.

Nothing is computed here; every step is a call into libmoe on the current stream, with no
host synchronisation in between, and no allocation after construction.
"""
import torch

from . import libmoe as L


class MoELayer:
    """One GPU's share of a top-k SwiGLU MoE layer.

    prerouted=True is the expert-parallel share: each of the T rows already carries one
    local expert id and its combine weight (k must be 1); routing and its backward are
    skipped and moe_expert_offsets provides the segment offsets.
    """

    def __init__(self, T, d, E, k, f, dtype, w_gate, w_up, w_down, renorm=1, prerouted=False,
                 save_gu=True, device="cuda", w_router=None, gather=False, weight_in_forward=None):
        """w_router [E, d], if given, makes the layer start from hidden states: forward() computes the logits
        itself and backward() also returns the router's weight gradient and adds the router term to dx."""
        assert not prerouted or k == 1
        assert w_router is None or not prerouted
        self.w_router = w_router
        self.gather = gather
        self.weight_in_forward = gather if weight_in_forward is None else bool(weight_in_forward)
        assert gather or not self.weight_in_forward, "the weight can ride in the forward products only on the gathered path"
        self.T, self.d, self.E, self.k, self.f = T, d, E, k, f
        self.P = T * k
        self.dtype, self.renorm, self.prerouted, self.save_gu = dtype, renorm, prerouted, save_gu
        self.w_gate, self.w_up, self.w_down = w_gate, w_up, w_down
        dev = torch.device(device)
        P = self.P
        code = L.MOE_BF16 if dtype == torch.bfloat16 else L.MOE_F32
        i32 = lambda *s: torch.empty(s, dtype=torch.int32, device=dev)
        f32 = lambda *s: torch.empty(s, dtype=torch.float32, device=dev)
        el = lambda *s: torch.empty(s, dtype=dtype, device=dev)
        self.topk_idx, self.topk_w = i32(T, k), f32(T, k)
        self.counts, self.offsets = i32(E), i32(E + 1)
        self.xp, self.row_of_pair, self.pair_of_row = None if gather else el(P, d), i32(P), i32(P)
        self.act, self.yp = el(P, f), el(P, d)
        self.g = el(P, f) if save_gu else None
        self.u = el(P, f) if save_gu else None
        self.y = el(T, d)
        self.dyp, self.dw = None if gather else el(P, d), f32(T, k)
        self.dxp = el(P, d)
        self.dw_gate, self.dw_up, self.dw_down = torch.empty_like(w_gate), torch.empty_like(w_up), torch.empty_like(w_down)
        self.dx = el(T, d)
        self.dlogits = None if prerouted else f32(T, E)
        self.logits = f32(T, E) if w_router is not None else None
        self.dw_router = torch.empty_like(w_router) if w_router is not None else None
        ws_bytes = max(
            L.lib.moe_router_logits_workspace_bytes(code, T, d, E) if w_router is not None else 0,
            L.lib.moe_router_bwd_workspace_bytes(code, T, d, E) if w_router is not None else 0,
            L.lib.moe_route_topk_workspace_bytes(T, E, k),
            L.lib.moe_expert_offsets_workspace_bytes(P, E),
            L.lib.moe_permute_workspace_bytes(T, E, k),
            L.lib.moe_grouped_gemm_swiglu_fwd_workspace_bytes(code, P, d, f, E),
            L.lib.moe_grouped_gemm_swiglu_bwd_workspace_bytes(code, P, d, f, E, int(save_gu)),
            L.lib.moe_grouped_gemm_swiglu_fwd_gather_workspace_bytes(code, P, d, f, E) if gather else 0,
            L.lib.moe_grouped_gemm_swiglu_bwd_gather_workspace_bytes(code, P, d, f, E, int(save_gu)) if gather else 0,
            256)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def forward(self, x, logits=None, topk_idx=None, topk_w=None):
        self.x = x
        if self.prerouted:
            self.topk_idx.copy_(topk_idx.view(self.T, 1))
            self.topk_w.copy_(topk_w.view(self.T, 1))
            L.moe_expert_offsets(self.topk_idx, self.E, out=(self.counts, self.offsets), ws=self.ws)
        else:
            if self.w_router is not None:
                logits = L.moe_router_logits(x, self.w_router, out=self.logits, ws=self.ws)
            L.moe_route_topk(logits, self.k, self.renorm,
                             out=(self.topk_idx, self.topk_w, self.counts, self.offsets), ws=self.ws)
        if self.gather:
            L.moe_permute(None, self.topk_idx, self.offsets, self.E, out=(None, self.row_of_pair, self.pair_of_row), ws=self.ws)
            L.moe_grouped_gemm_swiglu_fwd_gather(x, self.k, self.pair_of_row, self.w_gate, self.w_up, self.w_down, self.offsets,
                                                 save_gu=self.save_gu, out=(self.act, self.yp, self.g, self.u), ws=self.ws,
                                                 topk_w=self.topk_w if self.weight_in_forward else None)
        else:
            L.moe_permute(x, self.topk_idx, self.offsets, self.E,
                          out=(self.xp, self.row_of_pair, self.pair_of_row), ws=self.ws)
            L.moe_grouped_gemm_swiglu_fwd(self.xp, self.w_gate, self.w_up, self.w_down, self.offsets,
                                          save_gu=self.save_gu, out=(self.act, self.yp, self.g, self.u), ws=self.ws)
        L.moe_unpermute_combine_fwd(self.yp, None if self.weight_in_forward else self.topk_w, self.row_of_pair, self.T, self.k,
                                    out=self.y)
        return self.y

    def backward(self, dy, logits=None):
        if self.gather:
            L.moe_grouped_gemm_swiglu_bwd_gather(dy, self.x, self.topk_w, self.pair_of_row, self.g, self.u, self.w_gate,
                                                 self.w_up, self.w_down, self.offsets,
                                                 out=(self.dxp, self.dw_gate, self.dw_up, self.dw_down, self.dw), ws=self.ws,
                                                 act_w=self.act if self.weight_in_forward else None)
        else:
            L.moe_unpermute_combine_bwd(dy, self.yp, self.topk_w, self.row_of_pair, out=(self.dyp, self.dw))
            L.moe_grouped_gemm_swiglu_bwd(self.dyp, self.xp, self.g, self.u, self.act, self.w_gate, self.w_up,
                                          self.w_down, self.offsets,
                                          out=(self.dxp, self.dw_gate, self.dw_up, self.dw_down), ws=self.ws)
        L.moe_unpermute_combine_fwd(self.dxp, None, self.row_of_pair, self.T, self.k, out=self.dx)
        if not self.prerouted:
            if self.w_router is not None:
                logits = self.logits
            L.moe_route_topk_bwd(self.dw, self.topk_w, self.topk_idx, logits, self.E, self.renorm, out=self.dlogits)
            if self.w_router is not None:
                L.moe_router_bwd(self.dlogits, self.x, self.w_router, dx=self.dx, out_dw=self.dw_router, ws=self.ws)
        return self.dx, self.dw_gate, self.dw_up, self.dw_down, self.dlogits
